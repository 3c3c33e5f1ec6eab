"""Writes tests/golden/oracle_digests.txt: SHA-256 digests of what the CPU oracle produces on small seeded
workloads (frames, winning ids, kinematics poses).  Calls only oracle/ and the input generators.  The stored
digests pin the oracle against silent drift: a change of its arithmetic has to re-run this script on purpose,
and the commit that does so says which passage, or reading of it, justifies the change.

    python tests/golden/make_oracle_digests.py            # rewrite the file
    python tests/golden/make_oracle_digests.py --check    # compare, exit 1 on a difference
"""
import hashlib
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from oracle import orc  # noqa: E402
from paper_2502_00021_amd import workloads as wl  # noqa: E402

OUT = os.path.join(HERE, "oracle_digests.txt")


def _sha(*arrays):
    h = hashlib.sha256()
    for a in arrays:
        h.update(np.ascontiguousarray(a).tobytes())
    return h.hexdigest()


def digests():
    out = {}
    cases = [("cfg1", wl.make(1, B=8)), ("cfg2", wl.make(2, B=6)), ("cfg3", wl.make(3, B=6)), ("cfg4", wl.make(4, B=4)),
             ("cfg5", wl.make(5, B=4)), ("mesh", wl.cfg_mesh(B=6))]
    for name, w in cases:
        r = orc.Scene(w["desc"]).render(w["poses"], w["shapes"], step0=3, env0=11, distractor=w["distractor"])
        out[name + ".frames"] = _sha(r["frames"])
        out[name + ".ids"] = _sha(r["ids"])
        if "fk" in w:
            fk = w["fk"]
            out[name + ".poses"] = _sha(orc.fk(fk["skel"], fk["free_poses"], fk["angles"]).view(np.uint32))
    # a scene whose triangles cross the near plane (clipping)
    rng = np.random.default_rng(5)
    hv, ht, hm = wl.heightfield_mesh(rng, 5, 9.0, 0.25)
    d = wl.default_scene(56, 44, [wl.sphere(0.05, (0.6, 0.4, 0.8), 6, 2), wl.mesh(hv, ht, (0.6, 0.4, 0.8), mul=hm)])
    d["cam_offset"] = (-1.0, 0.0, 0.5)
    poses = np.array([[[[0, 0, 1, 1, 0, 0, 0], [-1.0, 0.0, 0.85, 1, 0, 0, 0]]]], np.float32)
    r = orc.Scene(d).render(poses)
    out["clip.frames"] = _sha(r["frames"])
    out["clip.ids"] = _sha(r["ids"])
    return out


def main():
    got = digests()
    if "--check" in sys.argv:
        want = dict(l.split() for l in open(OUT) if l.strip() and not l.startswith("#"))
        bad = [k for k in sorted(set(got) | set(want)) if got.get(k) != want.get(k)]
        for k in bad:
            print("differs:", k)
        sys.exit(1 if bad else 0)
    with open(OUT, "w") as f:
        f.write("# SHA-256 of the CPU oracle's outputs on small seeded workloads; written by make_oracle_digests.py\n")
        for k in sorted(got):
            f.write(f"{k} {got[k]}\n")
    print("wrote", OUT)


if __name__ == "__main__":
    main()
