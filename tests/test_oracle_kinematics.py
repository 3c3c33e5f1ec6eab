"""Pins for the oracle's kinematics stage: its sin/cos against libm, and hinge chains against the workload
generators' float64 quaternion algebra (an independent numpy implementation)."""
import math

import numpy as np
import pytest

from paper_2502_00021_amd import workloads as wl


def test_sincos_half_against_libm(orc):
    worst = 0.0
    for t in np.concatenate([np.linspace(-7, 7, 4001), np.linspace(-300, 300, 2001), [0.0, math.pi, -math.pi, 2 * math.pi]]):
        t = float(np.float32(t))
        s, c = orc.sincos_half(t)
        worst = max(worst, abs(s - math.sin(t / 2)), abs(c - math.cos(t / 2)))
        assert abs(s * s + c * c - 1.0) < 3e-7
    assert worst < 1.5e-7
    assert orc.sincos_half(0.0) == (0.0, 1.0)
    # quadrants: theta/2 = pi/2, pi, 3pi/2
    for t, (es, ec) in [(math.pi, (1, 0)), (2 * math.pi, (0, -1)), (3 * math.pi, (-1, 0)), (-math.pi, (-1, 0))]:
        s, c = orc.sincos_half(t)
        assert abs(s - es) < 2e-7 and abs(c - ec) < 2e-7


@pytest.mark.parametrize("cfg,B", [(2, 64), (3, 64), (4, 64), (5, 32)])
def test_chain_poses_match_float64_generators(orc, cfg, B):
    w = wl.make(cfg, B=B)
    fk = w["fk"]
    got = orc.fk(fk["skel"], fk["free_poses"], fk["angles"])
    ref = w["poses"].astype(np.float64)
    assert got.shape == ref.shape
    assert np.abs(got[..., :3] - ref[..., :3]).max() < 2e-6
    # quaternions agree up to sign (q and -q are the same rotation)
    dot = np.abs(np.einsum("...i,...i->...", got[..., 3:].astype(np.float64), ref[..., 3:]))
    assert np.all(dot > 1 - 1e-6)
    sign = np.sign(np.einsum("...i,...i->...", got[..., 3:].astype(np.float64), ref[..., 3:]))[..., None]
    assert np.abs(got[..., 3:] * sign - ref[..., 3:]).max() < 2e-6
    # free bodies are copied bit for bit
    free = np.nonzero(fk["skel"]["parent"] < 0)[0]
    assert np.array_equal(got[:, :, free], fk["free_poses"][:, :, fk["skel"]["slot"][free]])


def test_hinge_geometry_closed_forms(orc):
    """One hinge about x by 90 degrees: the child's centre swings from +z to -y of the anchor."""
    skel = wl._skeleton(3)
    skel["slot"][0] = 0
    wl._hinge(skel, 1, parent=0, slot=0, anchor=(0.0, 0.0, 0.5), axis=(1, 0, 0), offset=(0.0, 0.0, 0.25))
    wl._hinge(skel, 2, parent=1, slot=-1, anchor=(0.0, 0.0, 0.25), axis=(0, 1, 0), offset=(0.1, 0.0, 0.0))
    free = np.array([[[1.0, 2.0, 3.0, 1.0, 0.0, 0.0, 0.0]]], np.float32)
    out = orc.fk(skel, free, np.array([[math.pi / 2]], np.float32))[0]
    assert np.allclose(out[0], free[0, 0])
    assert np.allclose(out[1, :3], [1.0, 2.0 - 0.25, 3.5], atol=1e-6)
    assert np.allclose(out[1, 3:], [math.sqrt(0.5), math.sqrt(0.5), 0, 0], atol=1e-6)
    assert np.allclose(out[2, :3], [1.1, 2.0 - 0.5, 3.5], atol=1e-6)  # rigid child: same rotation, offset along x
    assert np.allclose(out[2, 3:], out[1, 3:], atol=1e-7)
    out0 = orc.fk(skel, free, np.array([[0.0]], np.float32))[0]
    assert np.array_equal(out0[1], np.array([1, 2, 3.75, 1, 0, 0, 0], np.float32))
    # rotated parent: everything turns with it
    q = wl.random_quats(np.random.default_rng(4), ())
    free2 = np.array([[[0.0, 0.0, 0.0, *q]]], np.float32)
    a = orc.fk(skel, free2, np.array([[0.7]], np.float32))[0]
    b = orc.fk(skel, np.array([[[0, 0, 0, 1, 0, 0, 0]]], np.float32), np.array([[0.7]], np.float32))[0]
    assert np.allclose(a[1:, :3], wl.q_rotate(q, b[1:, :3].astype(np.float64)), atol=1e-6)


def test_malformed_skeletons_are_rejected(orc):
    skel = wl._skeleton(2)
    with pytest.raises(ValueError):  # a free body needs a slot
        orc.fk(skel, np.zeros((1, 1, 7), np.float32), np.zeros((1, 1), np.float32))
    skel["slot"][0] = 0
    wl._hinge(skel, 1, parent=1, slot=0, anchor=(0, 0, 0), axis=(1, 0, 0), offset=(0, 0, 0))
    with pytest.raises(ValueError):  # parent must precede child
        orc.fk(skel, np.zeros((1, 1, 7), np.float32), np.zeros((1, 1), np.float32))
