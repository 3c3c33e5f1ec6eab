"""Pins for the oracle's near-plane clipping: winners and depths against a per-pixel ray cast that only
accepts hits at view depth >= z_near on camera-facing triangles (what clipping is supposed to leave)."""
import numpy as np
import pytest

from helpers import pose_row, world_positions
from paper_2502_00021_amd import workloads as wl
from test_oracle_scene import _pixel_rays

BG = 0xFFFFFFFF
GROUND = 0xFFFFFFFE
RGB = (0.6, 0.4, 0.8)


def _front_hits(eye, dirs, tri, t_min):
    """Ray parameter (= view depth) of the hit of each ray with a camera-facing triangle, np.inf otherwise."""
    a, b, c = tri
    e1, e2 = b - a, c - a
    p = np.cross(dirs, e2)
    det = p @ e1
    ok = det > 1e-14  # det = -dir . (e1 x e2): positive when the counter-clockwise side faces the camera
    inv = np.where(ok, 1.0 / np.where(ok, det, 1.0), 0.0)
    tv = eye - a
    u = (p @ tv) * inv
    q = np.cross(tv, e1)
    v = (dirs @ q) * inv
    t = (e2 @ q) * inv
    hit = ok & (u >= 0) & (v >= 0) & (u + v <= 1) & (t >= t_min)
    return np.where(hit, t, np.inf)


def _cast(desc, world, tris, root_pos, di=0.0, dj=0.0):
    eye, dirs = _pixel_rays(desc, root_pos, di, dj)
    best_t = np.full(dirs.shape[:2], np.inf)
    second = np.full(dirs.shape[:2], np.inf)
    best = np.full(dirs.shape[:2], BG, dtype=np.int64)
    for g, t3 in enumerate(tris):
        t = _front_hits(eye, dirs, world[t3], desc["z_near"])
        upd = t < best_t
        second = np.where(upd, best_t, np.minimum(second, t))
        best_t = np.where(upd, t, best_t)
        best[upd] = g
    return best, best_t, second


def _check_against_cast(orc, desc, poses, min_owned, min_clipped):
    s = orc.Scene(desc)
    mesh = s.mesh()
    tris = mesh["tris"].astype(np.int64)
    shapes = [b["shape"] for b in desc["bodies"]]
    owned = clipped = 0
    for pose in poses:
        out = s.render(pose[None, None], want_depth=True)
        ids = out["ids"][0, 0].astype(np.int64)
        vs = s.vertex_stage(pose)
        behind = vs["rejected"] == 2
        assert not np.any(vs["rejected"] == 1)
        straddling = behind[tris].any(axis=1) & ~behind[tris].all(axis=1)
        world = world_positions(mesh, shapes, pose.astype(np.float64))
        root = pose[desc["root_body"], :3]
        ref, t1, t2 = _cast(desc, world, tris, root)
        eps = 3.0 / 256.0
        stable = np.ones_like(ref, dtype=bool)
        for di, dj in [(-eps, 0), (eps, 0), (0, -eps), (0, eps), (-eps, -eps), (eps, eps), (-eps, eps), (eps, -eps)]:
            stable &= _cast(desc, world, tris, root, di, dj)[0] == ref
        with np.errstate(divide="ignore", invalid="ignore"):
            tie = np.abs(0.1 / t1 - 0.1 / t2) < 1e-5
        stable &= ~np.where(np.isfinite(t2), tie, False)
        assert stable.mean() > 0.8
        assert np.array_equal(ids[stable], ref[stable])
        hit = stable & (ref != BG)
        depth = out["depth_bits"][0, 0].view(np.float32)
        assert np.allclose(depth[hit], desc["z_near"] / t1[hit], rtol=4e-3)
        owned += int(hit.sum())
        clipped += int((hit & straddling[np.where(ref == BG, 0, ref)]).sum())
    assert owned >= min_owned and clipped >= min_clipped, (owned, clipped)


def _one_triangle_scene(verts, W=48, H=40):
    """A tiny anchor sphere as the root (the camera follows it) plus one two-sided triangle given in WORLD
    coordinates (its body sits at the origin with the identity rotation)."""
    tri = wl.mesh(np.asarray(verts, np.float32), np.array([[0, 1, 2], [0, 2, 1]], np.uint32), RGB)
    d = wl.default_scene(W, H, [wl.sphere(0.01, RGB, 4, 2), tri])
    d["ground_enabled"] = False
    d["cam_offset"] = (-2.0, 0.0, 0.0)  # eye at (-2,0,1) looking along +x, near plane at x = -1.9
    return d, np.stack([pose_row((0, 0, 1)), pose_row((0, 0, 0))])


def test_single_triangles_one_and_two_corners_in_front(orc):
    cases = [
        # one corner in front, two behind the camera
        [(-0.5, 0.0, 1.0), (-4.0, 0.9, 0.4), (-4.0, -0.7, 1.8)],
        # two corners in front, one behind
        [(0.5, -0.8, 0.5), (0.8, 0.9, 1.6), (-5.0, 0.1, 1.0)],
        # every corner order of the same triangle cuts the same region
        [(-5.0, 0.1, 1.0), (0.5, -0.8, 0.5), (0.8, 0.9, 1.6)],
        [(0.8, 0.9, 1.6), (-5.0, 0.1, 1.0), (0.5, -0.8, 0.5)],
        # a corner exactly on the near plane (x = -1.9 is not representable: slightly in front / behind)
        [(-1.9, 0.0, 1.3), (1.0, 0.5, 0.8), (-3.0, -0.4, 0.7)],
    ]
    maps = []
    for verts in cases:
        d, pose = _one_triangle_scene(verts)
        _check_against_cast(orc, d, [pose], min_owned=60, min_clipped=60)
        maps.append(orc.Scene(d).render(pose[None, None])["ids"][0, 0] != BG)
    assert np.array_equal(maps[1], maps[2]) and np.array_equal(maps[1], maps[3])


def test_triangle_entirely_behind_or_in_front(orc):
    d, pose = _one_triangle_scene([(-3.0, 0.0, 1.0), (-4.0, 0.9, 0.4), (-4.0, -0.7, 1.8)])
    s = orc.Scene(d)
    ids = s.render(pose[None, None])["ids"][0, 0]
    assert not np.any((ids >= s.T - 2) & (ids < GROUND))  # nothing of the triangle; only the anchor sphere
    # in front of the plane the clipper is never entered: same image as a soup raster of the snapped vertices
    d, pose = _one_triangle_scene([(0.5, -0.8, 0.5), (0.8, 0.9, 1.6), (0.2, 0.1, 1.9)])
    s = orc.Scene(d)
    vs = s.vertex_stage(pose)
    soup_ids, _, _ = orc.raster(s.W, s.H, vs["X"], vs["Y"], vs["D"], s.mesh()["tris"], rejected=vs["rejected"])
    assert np.array_equal(s.render(pose[None, None])["ids"][0, 0], soup_ids)


def test_floor_mesh_running_under_and_behind_the_camera(orc):
    """A 6 m x 6 m terrain grid below the camera: rows of triangles straddle the near plane, neighbours must
    meet without cracks (every stable pixel the ray cast assigns to the floor is the floor's)."""
    rng = np.random.default_rng(5)
    hv, ht, hm = wl.heightfield_mesh(rng, 5, 9.0, 0.25)
    d = wl.default_scene(56, 44, [wl.sphere(0.05, RGB, 6, 2), wl.mesh(hv, ht, RGB, mul=hm)])
    d["ground_enabled"] = False
    d["cam_offset"] = (-1.0, 0.0, 0.5)
    poses = []
    for k in range(4):
        q = wl.q_axis_angle(wl.EZ, np.array(0.4 * k))
        poses.append(np.stack([pose_row((0, 0, 1)), np.array([-1.0 + 0.1 * k, 0.05 * k, 0.85, *q], np.float32)]))
    _check_against_cast(orc, d, poses, min_owned=3000, min_clipped=300)


def test_primitives_crossing_the_near_plane(orc):
    """A long capsule and a big box pass the camera from in front to behind: the parts in front stay visible."""
    bodies = [wl.sphere(0.05, RGB, 6, 2), wl.capsule(0.3, 3.0, RGB, 10, 3), wl.box(0.8, 0.6, 0.4, RGB, 3)]
    d = wl.default_scene(48, 48, bodies)
    d["ground_enabled"] = False
    d["cam_offset"] = (-1.5, 0.0, 0.4)
    rng = np.random.default_rng(6)
    poses = []
    for k in range(4):
        ax = wl.q_normalize(np.array([0.0, 1.0, 0.15 * k]))
        q = wl.q_axis_angle(ax, np.array(np.pi / 2 + 0.1 * k))  # capsule axis roughly along the view direction
        poses.append(np.stack([pose_row((0, 0, 1)), np.array([-1.0, 0.5 - 0.2 * k, 1.0 + 0.1 * k, *q], np.float32),
                               np.array([-1.2, -0.9 + 0.1 * k, 1.2, *wl.random_quats(rng, ())], np.float32)]))
    _check_against_cast(orc, d, poses, min_owned=2500, min_clipped=200)


def test_clipped_scene_is_permutation_invariant_and_deterministic(orc):
    rng = np.random.default_rng(7)
    hv, ht, hm = wl.heightfield_mesh(rng, 6, 5.0, 0.4)
    d = wl.default_scene(40, 32, [wl.sphere(0.05, RGB, 6, 2), wl.mesh(hv, ht, RGB, mul=hm)])
    d["cam_offset"] = (-1.0, 0.0, 0.5)
    s = orc.Scene(d)
    pose = np.stack([pose_row((0, 0, 1)), pose_row((-0.8, 0.0, 0.3))])[None, None]
    a = s.render(pose, want_depth=True)
    b = s.render(pose, order=rng.permutation(s.T), want_depth=True)
    for k in ("ids", "frames", "depth_bits"):
        assert np.array_equal(a[k], b[k])
