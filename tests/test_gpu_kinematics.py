"""GPU parity of the kinematics stage (joint angles -> poses -> frames) against the CPU oracle.

The oracle takes sin and cos of the half angle from the C library in double (rounded once); the kernel
evaluates a range reduction and two polynomials in fp32.  Poses are therefore compared within a bound, derived
here (u = 2^-24, the fp32 unit roundoff; d = a body's depth below its free root):

  joint quaternion j = (cos, sin * axis): the kernel's sin / cos are within 1.25u of the true values on the
      stage's domain (|angle| <= 65536), the oracle's within 0.5u, the product with the axis adds 0.5u on each
      side: |dj| <= 4u in the 2-norm.
  orientation q = q_parent (x) j: the quaternion product is norm-multiplicative, so in the 2-norm
      e_q(d) <= e_q(d-1) |j| + |q_parent| |dj| + rounding; each of the four components is a chain of four
      operations on partial sums below 2 (<= 4u per side, 16u in the 2-norm for both sides together):
      e_q(d) <= (1 + 4u) e_q(d-1) + 20u,  e_q(free body) = 0 (copied).
  position p = (p_parent + R(q_parent) a) + R(q) c: an entry of R moves by at most 5.7 e_q (it is bilinear in
      a quaternion whose 1-norm is at most 2) and carries 4u of rounding from both sides, a row times a vector
      3u more per unit of the vector's 1-norm, the two additions 2u |p|:
      e_p <= e_p(parent) + (5.7 e_q(parent) + 7u) |a|_1 + (5.7 e_q + 7u) |c|_1 + 2u max|p|.

These are worst-case sums; typical differences are around 1u (asserted as a median).  Frames are then checked
exactly: the oracle renders the poses THE KERNEL produced, and ids must agree bit for bit, RGB with difference 0.
"""
import numpy as np
import pytest

from paper_2502_00021_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch():
    import torch as _torch
    assert _torch.cuda.is_available(), "these tests need the MI355X"
    return _torch


@pytest.fixture(scope="module")
def pxr():
    from paper_2502_00021_amd import pxr as _pxr
    _pxr.lib()
    return _pxr


def _bits(a):
    return np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)


U = 2.0 ** -24


def assert_poses_close(got, ref, skel):
    """got, ref [..., K, 7] against the bound derived in this file's header."""
    got, ref = np.asarray(got, np.float32), np.asarray(ref, np.float32)
    K = ref.shape[-2]
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan)
    g, r = np.where(nan, 0.0, got.astype(np.float64)), np.where(nan, 0.0, ref.astype(np.float64))
    e_q, e_p = np.zeros(K), [None] * K
    pmax = np.abs(r[..., :3]).max(axis=(-1, -2))  # per frame
    for k in range(K):
        par = int(skel["parent"][k])
        if par < 0:
            e_p[k] = np.zeros_like(pmax)
            assert np.array_equal(got[..., k, :].view(np.uint32)[~nan[..., k, :]], ref[..., k, :].view(np.uint32)[~nan[..., k, :]])
            continue
        e_q[k] = (1 + 4 * U) * e_q[par] + 20 * U
        a1, c1 = np.abs(skel["anchor"][k]).sum(), np.abs(skel["offset"][k]).sum()
        e_p[k] = e_p[par] + (5.7 * e_q[par] + 7 * U) * a1 + (5.7 * e_q[k] + 7 * U) * c1 + 2 * U * pmax
        dq = np.abs(g[..., k, 3:] - r[..., k, 3:]).max(axis=-1)
        dp = np.abs(g[..., k, :3] - r[..., k, :3]).max(axis=-1)
        assert np.all(dq <= e_q[k]), (k, dq.max(), e_q[k])
        assert np.all(dp <= e_p[k]), (k, dp.max(), e_p[k].min())
    hinged = np.asarray(skel["parent"]) >= 0
    if hinged.any() and not nan.any():  # roundings add up like a random walk along a chain, not linearly
        assert np.median(np.abs(g[..., hinged, 3:] - r[..., hinged, 3:])) <= U * (1 + np.sqrt(e_q.max() / (20 * U)))
    return float(np.abs(g - r).max())


def _scene_with_skeleton(pxr, w):
    fk = w["fk"]
    sc = pxr.Scene(w["desc"])
    sc.set_skeleton(fk["skel"], fk["free_poses"].shape[-2], fk["angles"].shape[-1])
    return sc


@pytest.mark.parametrize("cfg,B", [(2, 150), (3, 64), (3, 1), (4, 131), (5, 50)])
def test_poses_within_the_derived_bound(torch, pxr, orc, cfg, B):
    """Several 64-frame workgroups and a ragged tail."""
    w = wl.make(cfg, B=B)
    fk = w["fk"]
    sc = _scene_with_skeleton(pxr, w)
    got = sc.pose_batch(torch.from_numpy(fk["free_poses"]).cuda(), torch.from_numpy(fk["angles"]).cuda())
    torch.cuda.synchronize()
    ref = orc.fk(fk["skel"], fk["free_poses"], fk["angles"])
    worst = assert_poses_close(got.cpu().numpy(), ref, fk["skel"])
    assert worst < 2e-6  # (what the bound comes to for these shallow trees is a few times this)
    sc.close()


def test_extreme_angles_and_non_finite_inputs(torch, pxr, orc):
    w = wl.make(4, B=96)
    fk = w["fk"]
    ang = fk["angles"].copy()
    rng = np.random.default_rng(7)
    ang[:32] = rng.uniform(-300.0, 300.0, ang[:32].shape).astype(np.float32)
    ang[32:40] = np.float32(np.pi) * rng.integers(-8, 9, ang[32:40].shape).astype(np.float32)  # quadrant edges
    ang[40, 0, 3] = np.nan
    ang[41, 0, 5] = np.inf
    ang[42] = 0.0
    ang[45, 0, 2] = 1e10      # outside the stage's domain: NaN on both sides
    ang[46, 0, 4] = -65540.0
    ang[47] = rng.uniform(-65536.0, 65536.0, ang[47].shape).astype(np.float32)  # its far end
    free = fk["free_poses"].copy()
    free[43, 0, 0, 3:] = 0.0  # zero root quaternion
    free[44, 0, 0, 0] = np.nan
    sc = _scene_with_skeleton(pxr, w)
    got = sc.pose_batch(torch.from_numpy(free).cuda(), torch.from_numpy(ang).cuda()).cpu().numpy()
    ref = orc.fk(fk["skel"], free, ang)
    assert np.isnan(ref).any() and np.isnan(ref[45]).any() and np.isnan(ref[46]).any() and not np.isnan(ref[47]).any()
    assert_poses_close(got, ref, fk["skel"])
    sc.close()


def test_free_only_and_rigid_only_skeletons(torch, pxr, orc):
    w = wl.make(1, B=70)  # four free capsules: the stage is a copy
    skel = wl._skeleton(4)
    skel["slot"][:] = [2, 0, 3, 1]
    sc = pxr.Scene(w["desc"])
    sc.set_skeleton(skel, 4, 0)
    free = w["poses"]
    got = sc.pose_batch(torch.from_numpy(free).cuda(), None).cpu().numpy()
    assert np.array_equal(_bits(got), _bits(free[:, :, [2, 0, 3, 1]]))
    # one free root, three bodies welded to it in a chain (no angles)
    skel = wl._skeleton(4)
    skel["slot"][0] = 0
    for k in (1, 2, 3):
        wl._hinge(skel, k, parent=k - 1, slot=-1, anchor=(0.1, 0.0, 0.2), axis=(0, 0, 1), offset=(0.0, 0.05, 0.1))
    sc.set_skeleton(skel, 1, 0)
    free = np.ascontiguousarray(w["poses"][:, :, :1])
    got = sc.pose_batch(torch.from_numpy(free).cuda(), None).cpu().numpy()
    assert_poses_close(got, orc.fk(skel, free, np.zeros((70, 1, 0), np.float32)), skel)
    sc.close()


def test_sixty_four_link_chain(torch, pxr, orc):
    """The body-count limit as one chain of depth 63."""
    rng = np.random.default_rng(66)
    K = 64
    bodies = [wl.capsule(0.03, 0.05, rng.uniform(0.2, 0.9, 3), 4, 1) for _ in range(K)]
    skel = wl._skeleton(K)
    skel["slot"][0] = 0
    for k in range(1, K):
        ax = wl.q_normalize(rng.standard_normal(3))
        wl._hinge(skel, k, parent=k - 1, slot=(k - 1) if k % 5 else -1, anchor=(0, 0, 0.05), axis=ax, offset=(0, 0, 0.05))
    sc = pxr.Scene(wl.default_scene(32, 32, bodies))
    sc.set_skeleton(skel, 1, K - 1)
    N = 130
    free = np.zeros((N, 1, 7), np.float32)
    free[:, 0, :3] = (0, 0, 1)
    free[:, 0, 3:] = wl.random_quats(rng, (N,))
    ang = rng.uniform(-1.5, 1.5, (N, K - 1)).astype(np.float32)
    got = sc.pose_batch(torch.from_numpy(free).cuda(), torch.from_numpy(ang).cuda()).cpu().numpy()
    assert_poses_close(got, orc.fk(skel, free, ang), skel)
    sc.close()


def _random_tree(seed):
    """A seeded random forest over K bodies: several free roots, hinged and welded children in any shape (stars,
    chains, bushes), angle slots in shuffled order, frame counts around the 64-frame workgroups."""
    rng = np.random.default_rng(4400 + seed)
    K = int(rng.integers(1, 65))
    skel = wl._skeleton(K)
    n_free = n_ang = 0
    depth = np.zeros(K, int)
    for k in range(K):
        if k == 0 or rng.random() < 0.08:
            skel["slot"][k] = n_free
            n_free += 1
            continue
        shallow = [j for j in range(k) if depth[j] < 12] or [0]  # (keeps the error bound of deep chains meaningful)
        par = int(rng.choice(shallow)) if rng.random() < 0.7 else int(shallow[-1])
        depth[k] = depth[par] + 1
        welded = rng.random() < 0.15
        wl._hinge(skel, k, parent=par, slot=-1 if welded else n_ang, anchor=rng.uniform(-0.3, 0.3, 3),
                  axis=wl.q_normalize(rng.standard_normal(3)), offset=rng.uniform(-0.3, 0.3, 3))
        n_ang += 0 if welded else 1
    hinged = np.flatnonzero((skel["parent"] >= 0) & (skel["slot"] >= 0))
    skel["slot"][hinged] = rng.permutation(n_ang)           # angles in any order
    roots = np.flatnonzero(skel["parent"] < 0)
    skel["slot"][roots] = rng.permutation(n_free)
    N = int(rng.choice([1, 63, 64, 65, 130, 200]))
    free = np.zeros((N, n_free, 7), np.float32)
    free[..., :3] = rng.uniform(-2.0, 2.0, (N, n_free, 3))
    free[..., 3:] = wl.random_quats(rng, (N, n_free))
    ang = rng.uniform(-3.2, 3.2, (N, n_ang)).astype(np.float32)
    return K, skel, n_free, n_ang, free, ang


@pytest.mark.parametrize("seed", range(10))
def test_random_trees(torch, pxr, orc, seed):
    K, skel, n_free, n_ang, free, ang = _random_tree(seed)
    bodies = [wl.sphere(0.05, (0.5, 0.5, 0.5), 3, 1) for _ in range(K)]
    sc = pxr.Scene(wl.default_scene(16, 16, bodies))
    sc.set_skeleton(skel, n_free, n_ang)
    got = sc.pose_batch(torch.from_numpy(free).cuda(), torch.from_numpy(ang).cuda() if n_ang else None).cpu().numpy()
    assert_poses_close(got, orc.fk(skel, free, ang), skel)
    sc.close()


@pytest.mark.parametrize("cfg,B", [(2, 40), (3, 24), (4, 20), (5, 16)])
def test_angles_to_frames_match_oracle(torch, pxr, orc, cfg, B):
    from test_gpu_parity import _bind, assert_parity
    w = wl.make(cfg, B=B)
    fk = w["fk"]
    sc = _scene_with_skeleton(pxr, w)
    _bind(torch, sc, w["distractor"])
    shapes = None if w["shapes"] is None else torch.from_numpy(w["shapes"]).cuda()
    frames, ids, poses = sc.render_batch_kinematic(torch.from_numpy(fk["free_poses"]).cuda(),
                                                   torch.from_numpy(fk["angles"]).cuda(), shapes, step0=4, env0=9,
                                                   want_ids=True)
    torch.cuda.synchronize()
    got_poses = poses.cpu().numpy()
    ref_poses = orc.fk(fk["skel"], fk["free_poses"], fk["angles"])
    assert_poses_close(got_poses, ref_poses, fk["skel"])
    # the frames are exactly those of the poses the kernel produced ...
    ref = orc.Scene(w["desc"]).render(got_poses, w["shapes"], step0=4, env0=9, distractor=w["distractor"])
    assert_parity(dict(frames=frames.cpu().numpy(), ids=pxr.ids_to_numpy(ids)), ref)
    # ... and differ from those of the oracle's own poses, and of the float64-generated ones, only where the
    # last bits of a pose moved a vertex across a pixel centre
    for other in (ref_poses, w["poses"]):
        base = orc.Scene(w["desc"]).render(other, w["shapes"], step0=4, env0=9, distractor=w["distractor"])
        assert (base["ids"] != ref["ids"]).mean() < 0.01
    sc.close()


@pytest.mark.parametrize("env", ["halfcheetah", "ant", "walker2d", "humanoid"])
def test_paper_environment_stand_ins(torch, pxr, orc, env):
    """The four environments the paper supports, as skeleton workloads: angles -> poses -> frames on the device."""
    from test_gpu_parity import assert_parity
    w = wl.PAPER_ENVIRONMENTS[env](B=70)
    fk = w["fk"]
    sc = _scene_with_skeleton(pxr, w)
    frames, ids, poses = sc.render_batch_kinematic(torch.from_numpy(fk["free_poses"]).cuda(),
                                                   torch.from_numpy(fk["angles"]).cuda(), None, want_ids=True)
    torch.cuda.synchronize()
    got_poses = poses.cpu().numpy()
    assert_poses_close(got_poses, orc.fk(fk["skel"], fk["free_poses"], fk["angles"]), fk["skel"])
    ref = orc.Scene(w["desc"]).render(got_poses)
    assert (ref["ids"] < 0xFFFFFFFE).mean() > 0.015
    assert_parity(dict(frames=frames.cpu().numpy(), ids=pxr.ids_to_numpy(ids)), ref)
    sc.close()


def test_full_size_pose_batch(torch, pxr, orc):
    """The headline workload's 196 608 frames, every pose compared."""
    w = wl.make(5)
    fk = w["fk"]
    sc = _scene_with_skeleton(pxr, w)
    got = sc.pose_batch(torch.from_numpy(fk["free_poses"]).cuda(), torch.from_numpy(fk["angles"]).cuda())
    torch.cuda.synchronize()
    got = got.cpu().numpy()
    n = 16384  # the oracle's per-frame Python loop: check the first, the last and a middle run of environments
    B = got.shape[0]
    for lo in (0, B // 2 - n // 2, B - n):
        ref = orc.fk(fk["skel"], fk["free_poses"][lo:lo + n], fk["angles"][lo:lo + n])
        assert_poses_close(got[lo:lo + n], ref, fk["skel"])
    sc.close()


def test_skeleton_argument_errors(torch, pxr):
    w = wl.make(3, B=4)
    fk = w["fk"]
    sc = pxr.Scene(w["desc"])
    free = torch.from_numpy(fk["free_poses"]).cuda()
    ang = torch.from_numpy(fk["angles"]).cuda()
    with pytest.raises(pxr.PxrError):  # nothing bound yet
        sc.pose_batch(free, ang)
    out = torch.empty((4, 1, 9, 7), device="cuda")
    assert pxr.lib().pxr_pose_batch(sc._h, free.data_ptr(), ang.data_ptr(), 4, out.data_ptr(), None) == pxr.ERR_INVALID_ARG
    bad = {k: np.array(v, copy=True) for k, v in fk["skel"].items()}
    bad["parent"][3] = 5  # parent after child
    with pytest.raises(pxr.PxrError):
        sc.set_skeleton(bad, 1, 8)
    bad = {k: np.array(v, copy=True) for k, v in fk["skel"].items()}
    bad["slot"][4] = 8  # angle index out of range
    with pytest.raises(pxr.PxrError):
        sc.set_skeleton(bad, 1, 8)
    bad = {k: np.array(v, copy=True) for k, v in fk["skel"].items()}
    bad["axis"][2, 1] = np.inf
    with pytest.raises(pxr.PxrError):
        sc.set_skeleton(bad, 1, 8)
    with pytest.raises(pxr.PxrError):  # wrong body count
        sc.set_skeleton({k: v[:5] for k, v in fk["skel"].items()}, 1, 8)
    sc.set_skeleton(fk["skel"], 1, 8)
    L = pxr.lib()
    assert L.pxr_pose_batch(sc._h, free.data_ptr(), ang.data_ptr(), 0, out.data_ptr(), None) == pxr.ERR_INVALID_ARG
    assert L.pxr_pose_batch(sc._h, None, ang.data_ptr(), 4, out.data_ptr(), None) == pxr.ERR_INVALID_ARG
    assert L.pxr_pose_batch(sc._h, free.data_ptr(), ang.data_ptr(), 4, out.data_ptr() + 2, None) == pxr.ERR_INVALID_ARG
    sc.pose_batch(free, ang, poses=out)  # still usable
    torch.cuda.synchronize()
    sc.set_skeleton(None, 0, 0)
    with pytest.raises(pxr.PxrError):
        sc.pose_batch(free, ang)
    sc.close()
