"""GPU parity of the kinematics stage (joint angles -> poses -> frames) against the CPU oracle.

Bar: poses bit-exact (both sides run the same fp32 operation sequence, including their own sin/cos);
frames rendered from them: ids bit-exact, RGB equal.
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


def _scene_with_skeleton(pxr, w):
    fk = w["fk"]
    sc = pxr.Scene(w["desc"])
    sc.set_skeleton(fk["skel"], fk["free_poses"].shape[-2], fk["angles"].shape[-1])
    return sc


@pytest.mark.parametrize("cfg,B", [(2, 150), (3, 64), (3, 1), (4, 131), (5, 50)])
def test_poses_bit_exact(torch, pxr, orc, cfg, B):
    """Several 64-frame workgroups and a ragged tail."""
    w = wl.make(cfg, B=B)
    fk = w["fk"]
    sc = _scene_with_skeleton(pxr, w)
    got = sc.pose_batch(torch.from_numpy(fk["free_poses"]).cuda(), torch.from_numpy(fk["angles"]).cuda())
    torch.cuda.synchronize()
    ref = orc.fk(fk["skel"], fk["free_poses"], fk["angles"])
    assert np.array_equal(_bits(got.cpu().numpy()), _bits(ref))
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
    free = fk["free_poses"].copy()
    free[43, 0, 0, 3:] = 0.0  # zero root quaternion
    free[44, 0, 0, 0] = np.nan
    sc = _scene_with_skeleton(pxr, w)
    got = sc.pose_batch(torch.from_numpy(free).cuda(), torch.from_numpy(ang).cuda()).cpu().numpy()
    ref = orc.fk(fk["skel"], free, ang)
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan) and nan.any()
    assert np.array_equal(_bits(got)[~nan], _bits(ref)[~nan])  # NaN payloads are not part of the contract
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
    assert np.array_equal(_bits(got), _bits(orc.fk(skel, free, np.zeros((70, 1, 0), np.float32))))
    sc.close()


def test_sixty_four_link_chain(torch, pxr, orc):
    """The body-count limit as one chain of depth 63 (rounding accumulates identically on both sides)."""
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
    assert np.array_equal(_bits(got), _bits(orc.fk(skel, free, ang)))
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
    ref_poses = orc.fk(fk["skel"], fk["free_poses"], fk["angles"])
    assert np.array_equal(_bits(poses.cpu().numpy()), _bits(ref_poses))
    ref = orc.Scene(w["desc"]).render(ref_poses, w["shapes"], step0=4, env0=9, distractor=w["distractor"])
    assert_parity(dict(frames=frames.cpu().numpy(), ids=pxr.ids_to_numpy(ids)), ref)
    # the frames differ from those of the float64-generated poses only where rounding moved a vertex
    base = orc.Scene(w["desc"]).render(w["poses"], w["shapes"], step0=4, env0=9, distractor=w["distractor"])
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
    ref_poses = orc.fk(fk["skel"], fk["free_poses"], fk["angles"])
    assert np.array_equal(_bits(poses.cpu().numpy()), _bits(ref_poses))
    ref = orc.Scene(w["desc"]).render(ref_poses)
    assert (ref["ids"] < 0xFFFFFFFE).mean() > 0.015
    assert_parity(dict(frames=frames.cpu().numpy(), ids=pxr.ids_to_numpy(ids)), ref)
    sc.close()


def test_full_size_pose_batch_bit_exact(torch, pxr, orc):
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
        assert np.array_equal(_bits(got[lo:lo + n]), _bits(ref))
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
