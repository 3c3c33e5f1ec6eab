"""GPU parity: libpxr (HIP, through the C ABI) against the CPU oracle on the same seeded inputs.

Bar: winning-id maps bit-exact; RGB within 1/255 per channel after uint8 rounding (the same fp32
operation order is used on both sides, so the expected difference is 0 and is asserted where noted).
"""
import numpy as np
import pytest

from paper_2502_00021_amd import workloads as wl

pytestmark = pytest.mark.gpu

BG = 0xFFFFFFFF
GROUND = 0xFFFFFFFE


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


def _bind(torch, scene, dis):
    if dis is None:
        scene.apply_distractor(None)
        return
    d = dict(dis)
    if d["mode"] == "video":
        d["video"] = torch.from_numpy(np.ascontiguousarray(d["video"])).cuda()
        if d.get("env_offset") is not None:
            d["env_offset"] = torch.from_numpy(np.asarray(d["env_offset"]).astype(np.int32)).cuda()
        if d.get("env_video") is not None:
            d["env_video"] = torch.from_numpy(np.asarray(d["env_video"]).astype(np.int32)).cuda()
    scene.apply_distractor(d)


def gpu_render(torch, pxr, w, step0=0, env0=0, threads=None, scene=None):
    own = scene is None
    if own:
        scene = pxr.Scene(w["desc"])
    if threads:
        scene.set_block_threads(threads)
    _bind(torch, scene, w["distractor"])
    poses = torch.from_numpy(w["poses"]).cuda()
    shapes = None if w["shapes"] is None else torch.from_numpy(w["shapes"]).cuda()
    frames, ids = scene.render_batch(poses, shapes, step0=step0, env0=env0, want_ids=True)
    torch.cuda.synchronize()
    out = dict(frames=frames.cpu().numpy(), ids=pxr.ids_to_numpy(ids))
    if own:
        scene.close()
    return out


def assert_parity(got, ref, exact_rgb=True):
    assert got["ids"].shape == ref["ids"].shape and got["frames"].shape == ref["frames"].shape
    bad = np.argwhere(got["ids"] != ref["ids"])
    assert len(bad) == 0, f"{len(bad)} id mismatches, first at {bad[0]}: gpu {got['ids'][tuple(bad[0])]:#x} oracle {ref['ids'][tuple(bad[0])]:#x}"
    diff = np.abs(got["frames"].astype(np.int16) - ref["frames"].astype(np.int16))
    assert diff.max() <= 1, f"RGB differs by {diff.max()} LSB at {np.argwhere(diff > 1)[0]}"
    if exact_rgb:
        assert diff.max() == 0, f"{int((diff > 0).sum())} channels differ by 1 LSB"


def oracle_render(orc, w, step0=0, env0=0):
    s = orc.Scene(w["desc"])
    return s.render(w["poses"], w["shapes"], step0=step0, env0=env0, distractor=w["distractor"])


# ---------------------------------------------------------------- the five configurations

@pytest.mark.parametrize("cfg,B,threads", [(1, 16, 256), (1, 16, 1024), (2, 48, 512), (2, 24, 256), (3, 40, 512),
                                           (3, 24, 1024), (3, 17, 768), (4, 24, 1024), (4, 16, 512), (5, 20, 512), (5, 12, 256)])
def test_configs_match_oracle(torch, pxr, orc, cfg, B, threads):
    w = wl.make(cfg, B=B)
    got = gpu_render(torch, pxr, w, step0=3, env0=11, threads=threads)
    ref = oracle_render(orc, w, step0=3, env0=11)
    assert_parity(got, ref)
    tri = ref["ids"] < GROUND
    assert tri.any() and (ref["ids"] == GROUND).any() and (ref["ids"] == BG).any()


def test_default_block_threads_and_info(torch, pxr, orc):
    for cfg in (1, 2, 3, 4, 5):
        w = wl.make(cfg, B=2)
        sc = pxr.Scene(w["desc"])
        info = sc.info()
        o = orc.Scene(w["desc"])
        assert (info["n_verts"], info["n_tris"]) == (o.V, o.T)
        assert info["block_threads"] in (256, 512, 768, 1024) and info["lds_bytes"] <= 160 * 1024
        got = gpu_render(torch, pxr, w, scene=sc)
        assert_parity(got, oracle_render(orc, w))
        sc.close()


# ---------------------------------------------------------------- structure of the path

def test_determinism_and_slice_and_step_split(torch, pxr, orc):
    w = wl.make(5, B=24)
    a = gpu_render(torch, pxr, w, step0=7, env0=100)
    b = gpu_render(torch, pxr, w, step0=7, env0=100)
    assert np.array_equal(a["frames"], b["frames"]) and np.array_equal(a["ids"], b["ids"])
    # one env alone, with its global index
    e = 13
    one = dict(w, poses=w["poses"][e:e + 1], shapes=w["shapes"][e:e + 1])
    c = gpu_render(torch, pxr, one, step0=7, env0=100 + e)
    assert np.array_equal(c["frames"][0], a["frames"][e]) and np.array_equal(c["ids"][0], a["ids"][e])
    # steps 7,8,9 in one call == step 7 then steps 8,9
    first = dict(w, poses=np.ascontiguousarray(w["poses"][:, :1]))
    rest = dict(w, poses=np.ascontiguousarray(w["poses"][:, 1:]))
    f0 = gpu_render(torch, pxr, first, step0=7, env0=100)
    f1 = gpu_render(torch, pxr, rest, step0=8, env0=100)
    assert np.array_equal(np.concatenate([f0["frames"], f1["frames"]], axis=1), a["frames"])


def test_block_size_does_not_change_output(torch, pxr):
    w = wl.make(4, B=20)
    outs = [gpu_render(torch, pxr, w, threads=t) for t in (256, 512, 768, 1024)]
    for o in outs[1:]:
        assert np.array_equal(o["frames"], outs[0]["frames"]) and np.array_equal(o["ids"], outs[0]["ids"])


def test_batch_sizes_around_the_xcd_remap(torch, pxr, orc):
    """Frame <-> workgroup renumbering must be a bijection for every grid size modulo 8."""
    base = wl.make(3, B=41)
    ref = oracle_render(orc, base)
    for B in (1, 2, 7, 8, 9, 15, 16, 17, 33, 41):
        w = dict(base, poses=base["poses"][:B])
        got = gpu_render(torch, pxr, w)
        assert_parity(got, dict(frames=ref["frames"][:B], ids=ref["ids"][:B]))


# ---------------------------------------------------------------- image shapes

@pytest.mark.parametrize("W,H", [(8, 8), (33, 27), (40, 24), (127, 9), (128, 128), (31, 31), (84, 84), (9, 128)])
def test_image_shapes_including_unpacked_store_path(torch, pxr, orc, W, H):
    """W*H not a multiple of 4 takes the byte-store epilogue; 128x128 is the largest frame."""
    w = wl.make(3, B=6)
    w["desc"]["width"], w["desc"]["height"] = W, H
    assert_parity(gpu_render(torch, pxr, w, step0=2), oracle_render(orc, w, step0=2))
    rng = np.random.default_rng(W * 131 + H)
    video = rng.integers(0, 256, (7, H, W, 3), dtype=np.uint8)
    w["distractor"] = dict(mode="video", seed=5, video=video, alpha=0.5, env_offset=None)
    assert_parity(gpu_render(torch, pxr, w, step0=2), oracle_render(orc, w, step0=2))


@pytest.mark.parametrize("cfg,W,H,B", [(5, 256, 256, 3), (4, 200, 312, 2), (3, 512, 512, 2), (2, 500, 36, 3), (5, 132, 130, 3),
                                       (3, 250, 300, 2), (4, 86, 90, 3), (5, 96, 96, 4), (5, 192, 160, 2), (4, 84, 100, 3)])
def test_frames_larger_than_one_key_buffer(torch, pxr, orc, cfg, W, H, B):
    """Up to 512x512: the pixel keys are held a band of rows at a time.  Two or three bands of half a compute unit's
    LDS (a first band of whole resolve trips where there are two), or, from six bands on, all of the LDS and bands
    that pick their own triangles; widths that are no multiple of 4 take the byte-store loop, which clears its keys
    behind itself as well."""
    w = wl.make(cfg, B=B)
    w["desc"]["width"], w["desc"]["height"] = W, H
    if w["distractor"] is not None and w["distractor"]["mode"] == "video":
        rng = np.random.default_rng(W + H)
        w["distractor"] = dict(w["distractor"], video=rng.integers(0, 256, (5, H, W, 3), dtype=np.uint8))
    ref = oracle_render(orc, w, step0=1)
    assert (ref["ids"] < GROUND).mean() > 0.001
    assert_parity(gpu_render(torch, pxr, w, step0=1), ref)


def test_close_up_at_512(torch, pxr, orc):
    """Triangles hundreds of pixels wide crossing many bands."""
    rng = np.random.default_rng(77)
    B = 2
    poses = np.zeros((B, 1, 3, 7), np.float32)
    poses[:, 0, 0, :3] = (0, 0, 1)
    poses[:, 0, 0, 3:] = wl.random_quats(rng, (B,))
    for b in (1, 2):
        poses[:, 0, b, :3] = np.array([0, 0, 1]) + rng.uniform(-0.5, 0.5, (B, 3))
        poses[:, 0, b, 3:] = wl.random_quats(rng, (B,))
    w = dict(desc=_close_up(512, 384), poses=poses, shapes=None, distractor=None)
    ref = oracle_render(orc, w)
    assert (ref["ids"] < GROUND).mean() > 0.3
    assert_parity(gpu_render(torch, pxr, w), ref)


# ---------------------------------------------------------------- caller-supplied meshes

@pytest.mark.parametrize("W,H,B,threads", [(64, 64, 40, None), (84, 84, 17, 512), (32, 32, 24, 256), (200, 160, 5, None)])
def test_mesh_bodies_match_oracle(torch, pxr, orc, W, H, B, threads):
    w = wl.cfg_mesh(B=B, W=W, H=H)
    ref = oracle_render(orc, w, step0=2, env0=5)
    for lo, hi in [(0, 288), (288, 688), (688, 1008), (1008, 1296)]:
        assert ((ref["ids"] >= lo) & (ref["ids"] < hi)).any()
    assert_parity(gpu_render(torch, pxr, w, step0=2, env0=5, threads=threads), ref)


def test_mesh_close_up_and_degenerate_triangles(torch, pxr, orc):
    """Mesh triangles tens of pixels wide, a mesh with zero-area and repeated-vertex triangles, per-env scales."""
    rng = np.random.default_rng(12)
    tv, tt = wl.torus_mesh(0.35, 0.15, 7, 5)
    fan_v = np.array([[0, 0, 0]] + [[0.4 * np.cos(a), 0.4 * np.sin(a), 0.05 * a] for a in np.linspace(0, 5, 8)], np.float32)
    fan_t = np.array([[0, i, i + 1] for i in range(1, 8)] + [[0, i + 1, i] for i in range(1, 8)] + [[3, 3, 4], [5, 6, 5]], np.uint32)
    hv, ht, hm = wl.heightfield_mesh(rng, 5, 1.2, 0.4)
    bodies = [wl.mesh(tv, tt, (0.8, 0.5, 0.3)), wl.mesh(fan_v, fan_t, (0.3, 0.7, 0.5), mul=rng.uniform(0.3, 1.0, len(fan_t))),
              wl.mesh(hv, ht, (0.6, 0.6, 0.3), mul=hm)]
    d = wl.default_scene(96, 72, bodies)
    d["cam_offset"] = (-1.0, 0.1, 0.4)
    B = 20
    poses = np.zeros((B, 1, 3, 7), np.float32)
    poses[:, 0, 0, :3] = (0, 0, 1)
    poses[:, 0, 0, 3:] = wl.random_quats(rng, (B,))
    for b in (1, 2):
        poses[:, 0, b, :3] = np.array([0.1, 0, 1]) + rng.uniform(-0.5, 0.5, (B, 3))
        poses[:, 0, b, 3:] = wl.random_quats(rng, (B,))
    shapes = rng.uniform(0.6, 1.5, (B, 3, 4)).astype(np.float32)
    w = dict(desc=d, poses=poses, shapes=shapes, distractor=None)
    ref = oracle_render(orc, w)
    assert (ref["ids"] < GROUND).mean() > 0.25
    assert_parity(gpu_render(torch, pxr, w), ref)


# ---------------------------------------------------------------- maximum sizes

def test_sixty_four_bodies(torch, pxr, orc):
    """The body-count limit: 64 bodies of mixed kinds, per-environment shapes."""
    rng = np.random.default_rng(64)
    bodies = []
    for k in range(64):
        rgb = rng.uniform(0.2, 0.9, 3)
        bodies.append([wl.capsule(0.05, 0.12, rgb, 5, 2), wl.sphere(0.08, rgb, 6, 2), wl.box(0.07, 0.05, 0.06, rgb, 1)][k % 3])
    d = wl.default_scene(64, 48, bodies, root_body=63)
    B = 10
    poses = np.zeros((B, 1, 64, 7), np.float32)
    poses[..., :3] = np.array([0.0, 0.0, 1.0]) + rng.uniform(-0.9, 0.9, (B, 1, 64, 3)) * np.array([1.0, 1.0, 0.6])
    poses[..., 3:] = wl.random_quats(rng, (B, 1, 64))
    shapes = np.array([b["shape"] for b in bodies], np.float32)[None] * rng.uniform(0.7, 1.4, (B, 64, 1)).astype(np.float32)
    w = dict(desc=d, poses=poses, shapes=np.ascontiguousarray(shapes), distractor=None)
    ref = oracle_render(orc, w)
    assert len(np.unique(ref["ids"])) > 300
    assert_parity(gpu_render(torch, pxr, w), ref)


def test_scene_at_the_lds_limit(torch, pxr, orc):
    """The finest tessellation that still fits one compute unit's LDS (one workgroup per unit, many bands)."""
    bodies = [wl.sphere(0.5, (0.7, 0.4, 0.3), 64, 32), wl.capsule(0.2, 0.4, (0.3, 0.6, 0.8), 64, 8)]
    d = wl.default_scene(128, 96, bodies)
    d["cam_offset"] = (-1.8, 0.0, 0.5)
    sc = pxr.Scene(d)
    info = sc.info()
    assert info["lds_bytes"] > 120 * 1024 and info["n_verts"] > 5000 and info["n_tris"] > 10000
    rng = np.random.default_rng(65)
    B = 3
    poses = np.zeros((B, 1, 2, 7), np.float32)
    poses[:, 0, 0, :3] = (0, 0, 1)
    poses[:, 0, 0, 3:] = wl.random_quats(rng, (B,))
    poses[:, 0, 1, :3] = np.array([0.0, 0.6, 1.0]) + rng.uniform(-0.2, 0.2, (B, 3))
    poses[:, 0, 1, 3:] = wl.random_quats(rng, (B,))
    w = dict(desc=d, poses=poses, shapes=None, distractor=None)
    assert_parity(gpu_render(torch, pxr, w, scene=sc), oracle_render(orc, w))
    sc.close()


# ---------------------------------------------------------------- near-plane clipping

def _clip_scenes():
    RGB = (0.6, 0.4, 0.8)
    rng = np.random.default_rng(41)
    out = []
    # a terrain grid running under and behind the camera, 1 and 2 corners in front, several yaws
    hv, ht, hm = wl.heightfield_mesh(rng, 5, 9.0, 0.25)
    d = wl.default_scene(72, 56, [wl.sphere(0.05, RGB, 6, 2), wl.mesh(hv, ht, (0.7, 0.6, 0.4), mul=hm)])
    d["cam_offset"] = (-1.0, 0.0, 0.5)
    B = 12
    poses = np.zeros((B, 1, 2, 7), np.float32)
    poses[:, 0, 0] = (0, 0, 1, 1, 0, 0, 0)
    poses[:, 0, 1, :3] = np.array([-1.0, 0.0, 0.85]) + rng.uniform(-0.3, 0.3, (B, 3)) * np.array([1, 1, 0.2])
    poses[:, 0, 1, 3:] = wl.q_axis_angle(wl.EZ, rng.uniform(0, 2 * np.pi, B))
    out.append(dict(desc=d, poses=poses, shapes=None, distractor=None))
    # a long capsule and a big box passing the camera; colour distractor; tumbling
    bodies = [wl.sphere(0.05, RGB, 6, 2), wl.capsule(0.3, 3.0, (0.8, 0.3, 0.3), 10, 3), wl.box(0.8, 0.6, 0.4, (0.3, 0.5, 0.8), 3)]
    d = wl.default_scene(64, 64, bodies)
    d["cam_offset"] = (-1.5, 0.0, 0.4)
    B = 16
    poses = np.zeros((B, 1, 3, 7), np.float32)
    poses[:, 0, 0] = (0, 0, 1, 1, 0, 0, 0)
    poses[:, 0, 1, :3] = np.array([-1.0, 0.2, 1.1]) + rng.uniform(-0.4, 0.4, (B, 3))
    poses[:, 0, 1, 3:] = wl.random_quats(rng, (B,))
    poses[:, 0, 2, :3] = np.array([-1.2, -0.6, 1.2]) + rng.uniform(-0.4, 0.4, (B, 3))
    poses[:, 0, 2, 3:] = wl.random_quats(rng, (B,))
    out.append(dict(desc=d, poses=poses, shapes=None,
                    distractor=dict(mode="color", seed=3, scale=(0.5, 1.5), offset=(-0.2, 0.2))))
    # the camera inside a huge sphere and next to a huge box (everything visible is clipped or enormous)
    bodies = [wl.sphere(0.05, RGB, 6, 2), wl.sphere(3.0, (0.5, 0.7, 0.5), 12, 5), wl.box(2.0, 2.0, 0.05, (0.7, 0.7, 0.3), 4)]
    d = wl.default_scene(48, 40, bodies)
    d["cam_offset"] = (-0.8, 0.0, 0.3)
    B = 10
    poses = np.zeros((B, 1, 3, 7), np.float32)
    poses[:, 0, 0] = (0, 0, 1, 1, 0, 0, 0)
    poses[:, 0, 1, :3] = np.array([2.0, 0.0, 1.0]) + rng.uniform(-0.5, 0.5, (B, 3))
    poses[:, 0, 1, 3:] = wl.random_quats(rng, (B,))
    poses[:, 0, 2, :3] = np.array([-0.5, 0.0, 1.0]) + rng.uniform(-0.3, 0.3, (B, 3))
    poses[:, 0, 2, 3:] = wl.random_quats(rng, (B,))
    out.append(dict(desc=d, poses=poses, shapes=None, distractor=None))
    return out


@pytest.mark.parametrize("which", [0, 1, 2])
def test_triangles_crossing_the_near_plane_are_clipped(torch, pxr, orc, which):
    w = _clip_scenes()[which]
    o = orc.Scene(w["desc"])
    tris = o.mesh()["tris"]
    n_straddling = 0
    for e in range(w["poses"].shape[0]):
        behind = o.vertex_stage(w["poses"][e, 0])["rejected"] == 2
        n_straddling += int((behind[tris].any(axis=1) & ~behind[tris].all(axis=1)).sum())
    assert n_straddling > 20 * w["poses"].shape[0] // 4
    ref = oracle_render(orc, w, step0=1)
    assert (ref["ids"] < GROUND).mean() > 0.15
    for threads in (None, 256, 1024):
        assert_parity(gpu_render(torch, pxr, w, step0=1, threads=threads), ref)


def test_clipping_in_banded_frames(torch, pxr, orc):
    w = _clip_scenes()[1]
    w["desc"]["width"], w["desc"]["height"] = 260, 200
    w = dict(w, poses=w["poses"][:4])
    assert_parity(gpu_render(torch, pxr, w), oracle_render(orc, w))


# ---------------------------------------------------------------- large triangles, clipping, rejects

def _close_up(W=64, H=64, offset=(-0.9, 0.1, 0.35)):
    bodies = [wl.box(0.3, 0.25, 0.2, (0.8, 0.5, 0.3), 2), wl.capsule(0.15, 0.3, (0.2, 0.7, 0.4), 8, 3),
              wl.sphere(0.25, (0.5, 0.5, 0.9), 10, 4)]
    d = wl.default_scene(W, H, bodies)
    d["cam_offset"] = offset
    return d


def test_large_triangles_take_the_wave_path(torch, pxr, orc):
    rng = np.random.default_rng(101)
    B = 24
    poses = np.zeros((B, 1, 3, 7), np.float32)
    poses[:, 0, 0, :3] = (0, 0, 1)
    poses[:, 0, 0, 3:] = wl.random_quats(rng, (B,))
    for b in (1, 2):
        poses[:, 0, b, :3] = np.array([0, 0, 1]) + rng.uniform(-0.5, 0.5, (B, 3))
        poses[:, 0, b, 3:] = wl.random_quats(rng, (B,))
    for W, H in [(64, 64), (128, 128), (33, 27)]:
        w = dict(desc=_close_up(W, H), poses=poses, shapes=None, distractor=None)
        ref = oracle_render(orc, w)
        assert ((ref["ids"] < GROUND).mean() > 0.3)  # triangles tens of pixels wide
        assert_parity(gpu_render(torch, pxr, w), ref)


def test_huge_offscreen_extents_use_64bit_edges(torch, pxr, orc):
    """Camera almost touching a big box: snapped coordinates run to millions, products beyond 2^31."""
    bodies = [wl.sphere(0.05, (0.5, 0.5, 0.5), 8, 4), wl.box(3.0, 3.0, 0.5, (0.7, 0.6, 0.2), 3),
              wl.capsule(0.4, 2.0, (0.3, 0.6, 0.8), 6, 2)]
    d = wl.default_scene(64, 64, bodies)
    d["cam_offset"] = (-0.6, 0.0, 0.25)
    rng = np.random.default_rng(103)
    B = 16
    poses = np.zeros((B, 1, 3, 7), np.float32)
    poses[:, 0, 0, :3] = (0, 0, 1.2)
    poses[:, 0, 0, 3] = 1
    poses[:, 0, 1, :3] = np.array([1.5, 0, 0.6]) + rng.uniform(-1.0, 1.0, (B, 3)) * np.array([1.0, 1.0, 0.3])
    poses[:, 0, 1, 3:] = wl.random_quats(rng, (B,))
    poses[:, 0, 2, :3] = np.array([0.5, 0, 1.2]) + rng.uniform(-0.5, 0.5, (B, 3))
    poses[:, 0, 2, 3:] = wl.random_quats(rng, (B,))
    w = dict(desc=d, poses=poses, shapes=None, distractor=None)
    ref = oracle_render(orc, w)
    s = orc.Scene(d)
    spans = []
    for e in range(B):
        vs = s.vertex_stage(poses[e, 0])
        ok = vs["rejected"] == 0
        spans.append(int(np.ptp(vs["X"][ok])) if ok.any() else 0)
    assert max(spans) > 1 << 17, "scene does not exercise the 64-bit path"
    assert (ref["ids"] < GROUND).mean() > 0.2
    assert_parity(gpu_render(torch, pxr, w), ref)


def test_rejected_and_degenerate_inputs(torch, pxr, orc):
    w = wl.make(2, B=12)
    p = w["poses"].copy()
    p[8, 0, 0, 0] = np.nan         # non-finite root x: no usable vertex, ground cells decided by y alone
    p[9, 0, 0, 0] = 3.0e9          # ground cell index beyond int32: the conversion saturates on both sides
    p[10, 0, 0, 1] = -np.inf
    p[11, 0, 0, :2] = (-7.0e9, 5.0e9)
    p[0, 0, :, 0] -= 10.0          # whole chain far behind the camera (root too: camera follows it) -> visible
    p[1, 0, 1:, 0] = -5.0          # links behind the camera: rejected
    p[2, 0, 3, :3] = np.nan        # non-finite position
    p[3, 0, 2, 3:] = np.nan        # non-finite quaternion
    p[4, 0, 0, 2] = -3.0           # root (and the camera) below the ground plane
    p[5, 0, 4, :3] = p[5, 0, 0, :3] + np.array([-2.45, 0, 1.0], np.float32)  # a link straddling the near plane
    p[6, 0, :, 3:] = 0.0           # zero quaternions: bodies collapse to their centres
    p[7, 0, 5, 1] = 1e6            # far off to the side: guard band
    w["poses"] = p
    ref = oracle_render(orc, w)
    got = gpu_render(torch, pxr, w)
    assert_parity(got, ref)
    assert not np.any(ref["ids"][4] == GROUND)  # camera below the plane: no ground


@pytest.mark.parametrize("over", [dict(), dict(cam_up=(0.2, 0.1, 1.0)), dict(z_far=1.0e30),
                                  dict(z_far=3.0e38, cam_up=(0.2, 0.1, 1.0)), dict(ground_cell=0.37)])
def test_checker_cells_of_non_finite_and_huge_ground_points(torch, pxr, orc, over):
    """The unit-cell checker takes a shorter floor-and-convert that is only right when the ground point is no NaN:
    frames whose eye is a NaN, and scenes whose far plane lets the ray parameter overflow, must take the long form."""
    w = wl.make(1, B=12)
    p = w["poses"].copy()
    r = w["desc"]["root_body"]
    p[0, 0, r, 0] = np.nan
    p[1, 0, r, 1] = np.nan
    p[2, 0, r, 0] = np.inf
    p[3, 0, r, 1] = -np.inf
    p[4, 0, r, :2] = (np.inf, np.nan)
    p[5, 0, r, :2] = (-3.0e38, 3.0e38)
    p[6, 0, r, :2] = (2147483647.0, -2147483648.0)   # cell indices at the ends of int32
    p[7, 0, r, :2] = (2147483520.0, -2147483904.0)   # the floats next to them
    p[8, 0, r, :2] = (-0.0, 1.0e-30)
    p[9, 0, r, 2] = 3.0e38                           # eye so high that the ground is beyond any far plane
    p[10, 0, r, 2] = np.inf
    w = dict(w, poses=p, desc=dict(w["desc"], **over))
    assert_parity(gpu_render(torch, pxr, w), oracle_render(orc, w))


def test_ground_variants(torch, pxr, orc):
    w = wl.make(1, B=8)
    for over in (dict(ground_enabled=False), dict(ground_cell=0.37), dict(z_far=4.0), dict(cam_up=(0.2, 0.1, 1.0)),
                 dict(cam_offset=(1.5, 2.0, 3.0)), dict(fov_y_deg=25.0), dict(light_dir=(0.5, 0.2, -0.4))):
        w2 = dict(w, desc=dict(w["desc"], **over))
        assert_parity(gpu_render(torch, pxr, w2), oracle_render(orc, w2))


@pytest.mark.parametrize("seed", range(24))
def test_random_scenes_match_oracle(torch, pxr, orc, seed):
    """Seeded random scenes: image shapes, cameras (with and without roll), body mixes and sizes (triangles of
    every raster bin, bodies crossing the near plane), shapes per environment, all distractor modes."""
    w = wl.random_scene(seed)
    ref = oracle_render(orc, w, step0=3, env0=5)
    assert_parity(gpu_render(torch, pxr, w, step0=3, env0=5), ref)
    assert_parity(gpu_render(torch, pxr, w, step0=3, env0=5, threads=(256, 512, 768, 1024)[seed % 4]), ref)


# ---------------------------------------------------------------- distractors

def test_colour_distractor_per_step_and_identity(torch, pxr, orc):
    w = wl.make(3, B=12)
    plain = gpu_render(torch, pxr, dict(w, distractor=None))
    ident = gpu_render(torch, pxr, dict(w, distractor=dict(mode="color", seed=1, scale=(1.0, 1.0), offset=(0.0, 0.0))))
    assert np.array_equal(plain["frames"], ident["frames"])
    a = gpu_render(torch, pxr, w, step0=0)
    b = gpu_render(torch, pxr, w, step0=1)
    assert np.array_equal(a["ids"], b["ids"]) and not np.array_equal(a["frames"], b["frames"])
    for step0, env0 in [(0, 0), (1, 0), (0xFFFFFFFE, 0), (5, 0xFFFFFFF0)]:
        assert_parity(gpu_render(torch, pxr, w, step0=step0, env0=env0), oracle_render(orc, w, step0=step0, env0=env0))
    big_seed = dict(w, distractor=dict(w["distractor"], seed=0xFEDCBA9876543210))
    assert_parity(gpu_render(torch, pxr, big_seed, step0=9), oracle_render(orc, big_seed, step0=9))


def test_video_distractor_offsets_alpha_and_wrap(torch, pxr, orc):
    w = wl.make(4, B=12)
    video = w["distractor"]["video"]
    for dis, step0 in [(dict(mode="video", seed=4, video=video, alpha=0.5, env_offset=None), 0),
                       (dict(mode="video", seed=4, video=video, alpha=0.5, env_offset=None), 63),
                       (dict(mode="video", seed=9, video=video[:5], alpha=0.25, env_offset=None), 0xFFFFFFF0),
                       (dict(mode="video", seed=4, video=video, alpha=1.0, env_offset=np.arange(12) * 7 + 60), 3),
                       (dict(mode="video", seed=4, video=video, alpha=0.0, env_offset=None), 3)]:
        w2 = dict(w, distractor=dis)
        ref = oracle_render(orc, w2, step0=step0, env0=5)
        assert_parity(gpu_render(torch, pxr, w2, step0=step0, env0=5), ref)
    plain = gpu_render(torch, pxr, dict(w, distractor=None))
    assert np.array_equal(plain["frames"], gpu_render(torch, pxr, w2, step0=3)["frames"])  # alpha = 0


def test_video_distractor_with_and_without_blend_tables(torch, pxr, orc):
    """The video blend reads per-frame tables from LDS where the frame's LDS has room for them (small scenes, banded
    frames) and does the arithmetic per pixel where it has not (the largest unbanded scenes), or when the camera rolls."""
    rng = np.random.default_rng(99)
    for cfg, B, roll, has_tables in [(5, 10, False, False), (3, 12, False, True), (3, 8, True, True), (4, 6, False, True)]:
        w = wl.make(cfg, B=B)
        H, W = w["desc"]["height"], w["desc"]["width"]
        if roll:
            w["desc"]["cam_up"] = (0.0, 0.3, 1.0)
        w["distractor"] = dict(mode="video", seed=cfg, video=rng.integers(0, 256, (9, H, W, 3), dtype=np.uint8),
                               alpha=0.35, env_offset=None)
        sc = pxr.Scene(w["desc"])
        lds = sc.info()["lds_bytes"]
        sc.close()
        if not has_tables:  # two workgroups per compute unit as it is, one if the 2304 bytes of tables were added
            assert lds <= 80 * 1024 < lds + 2304
        assert_parity(gpu_render(torch, pxr, w, step0=5), oracle_render(orc, w, step0=5))


def test_video_sets_one_clip_per_environment(torch, pxr, orc):
    """A set of clips [n_videos, n_frames, H, W, 3]: each environment plays one, drawn from the generator or given."""
    w = wl.make(4, B=14)
    rng = np.random.default_rng(21)
    clips = rng.integers(0, 256, (5, 9, 84, 84, 3), dtype=np.uint8)
    for dis, step0 in [(dict(mode="video", seed=4, video=clips, alpha=0.5), 0),
                       (dict(mode="video", seed=77, video=clips, alpha=0.7, env_offset=np.arange(14) * 3), 8),
                       (dict(mode="video", seed=4, video=clips, alpha=0.5, env_video=np.arange(14) % 5), 2),
                       (dict(mode="video", seed=4, video=clips, alpha=0.5, env_video=np.arange(14) + 3,
                             env_offset=np.arange(14)[::-1].copy()), 0xFFFFFFF8),
                       (dict(mode="video", seed=4, video=clips[:1], alpha=0.5), 3)]:
        w2 = dict(w, distractor=dis)
        assert_parity(gpu_render(torch, pxr, w2, step0=step0, env0=3), oracle_render(orc, w2, step0=step0, env0=3))
    # a set of one clip is the single-clip case
    a = gpu_render(torch, pxr, dict(w, distractor=dict(mode="video", seed=4, video=clips[:1], alpha=0.5)), step0=3)
    b = gpu_render(torch, pxr, dict(w, distractor=dict(mode="video", seed=4, video=clips[0], alpha=0.5)), step0=3)
    assert np.array_equal(a["frames"], b["frames"])


def test_rebinding_and_unbinding(torch, pxr, orc):
    w = wl.make(3, B=6)
    sc = pxr.Scene(w["desc"])
    col = gpu_render(torch, pxr, w, scene=sc)
    none = gpu_render(torch, pxr, dict(w, distractor=None), scene=sc)
    col2 = gpu_render(torch, pxr, w, scene=sc)
    assert np.array_equal(col["frames"], col2["frames"]) and not np.array_equal(col["frames"], none["frames"])
    assert_parity(none, oracle_render(orc, dict(w, distractor=None)))
    sc.close()


# ---------------------------------------------------------------- argument errors on a live scene

def test_render_argument_errors(torch, pxr):
    w = wl.make(1, B=4)
    sc = pxr.Scene(w["desc"])
    L = pxr.lib()
    poses = torch.from_numpy(w["poses"]).cuda()
    frames = torch.empty((4, 1, 32, 32, 3), dtype=torch.uint8, device="cuda")
    h = sc._h
    assert L.pxr_render_batch(h, None, None, 4, 1, 0, 0, frames.data_ptr(), None, None) == pxr.ERR_INVALID_ARG
    assert L.pxr_render_batch(h, poses.data_ptr(), None, 0, 1, 0, 0, frames.data_ptr(), None, None) == pxr.ERR_INVALID_ARG
    poses2 = torch.cat([poses, poses], dim=1).contiguous()
    frames2 = torch.empty((4, 2, 32, 32, 3), dtype=torch.uint8, device="cuda")
    assert L.pxr_render_batch(h, poses2.data_ptr(), None, 4, 2, 0xFFFFFFFF, 0, frames2.data_ptr(), None, None) == pxr.ERR_INVALID_ARG
    assert L.pxr_render_batch(h, poses2.data_ptr(), None, 4, 2, 0, 0xFFFFFFFD, frames2.data_ptr(), None, None) == pxr.ERR_INVALID_ARG
    assert L.pxr_render_batch(h, poses.data_ptr(), None, 4, 1, 0, 0, frames.data_ptr() + 1, None, None) == pxr.ERR_INVALID_ARG
    shapes = torch.ones((5, w["poses"].shape[2], 4), dtype=torch.float32, device="cuda")
    assert L.pxr_render_batch(h, poses.data_ptr(), shapes.data_ptr() + 4, 4, 1, 0, 0, frames.data_ptr(), None, None) == pxr.ERR_INVALID_ARG
    assert L.pxr_render_batch(h, poses.data_ptr(), shapes.data_ptr() + 16, 4, 1, 0, 0, frames.data_ptr(), None, None) == pxr.OK
    assert L.pxr_render_batch(h, poses.data_ptr(), None, 1 << 31, 1, 0, 0, frames.data_ptr(), None, None) == pxr.ERR_INVALID_ARG
    assert b"pxr_render_batch" in L.pxr_last_error()
    with pytest.raises(pxr.PxrError):
        sc.set_block_threads(128)
    d = pxr.DistractorDesc()
    d.mode = 2
    import ctypes as C
    assert L.pxr_apply_distractor(h, C.byref(d)) == pxr.ERR_INVALID_ARG  # video without a clip
    d.mode = 9
    assert L.pxr_apply_distractor(h, C.byref(d)) == pxr.ERR_INVALID_ARG
    # the scene is still usable after the rejected calls
    f, _ = sc.render_batch(poses)
    torch.cuda.synchronize()
    assert f.shape == (4, 1, 32, 32, 3)
    sc.close()


# ---------------------------------------------------------------- full benchmark sizes, sampled

@pytest.mark.parametrize("cfg", [2, 3, 4, 5])
def test_full_size_batches_sampled_against_oracle(torch, pxr, orc, cfg):
    """The configurations at their full batch size, in the launch configuration bench.py times
    (library-default workgroup size, ids off for the timed buffer), checked on sampled environments
    the oracle renders one by one, plus run-to-run determinism of the whole output."""
    w = wl.make(cfg)
    B, S = w["poses"].shape[:2]
    scene = pxr.Scene(w["desc"])
    _bind(torch, scene, w["distractor"])
    poses = torch.from_numpy(w["poses"]).cuda()
    shapes = None if w["shapes"] is None else torch.from_numpy(w["shapes"]).cuda()
    frames, _ = scene.render_batch(poses, shapes, step0=5, env0=0)
    again, ids = scene.render_batch(poses, shapes, step0=5, env0=0, want_ids=True)
    torch.cuda.synchronize()
    assert torch.equal(frames, again)
    rng = np.random.default_rng(cfg)
    chunk = (B * S + 7) // 8 // S  # environments per XCD run of the workgroup renumbering
    picks = sorted(set([0, 1, B - 1, B - 2, B // 2] + [min(B - 1, k * chunk + d) for k in range(1, 8) for d in (-1, 0)]
                       + [int(e) for e in rng.integers(0, B, 24)]))
    o = orc.Scene(w["desc"])
    for e in picks:
        sh = None if w["shapes"] is None else w["shapes"][e:e + 1]
        ref = o.render(w["poses"][e:e + 1], sh, step0=5, env0=e, distractor=w["distractor"])
        got = dict(frames=frames[e:e + 1].cpu().numpy(), ids=pxr.ids_to_numpy(ids[e:e + 1]))
        assert_parity(got, ref)
    scene.close()


def test_outputs_beyond_four_gibibytes(torch, pxr, orc):
    """A batch whose frames (4.5 GB) and id maps (6 GB) pass 2^32 bytes: offsets are 64-bit all the way.
    Sampled environments from both ends and around the 4 GiB mark against the oracle."""
    w = wl.make(4, B=16)
    B = 212992
    rng = np.random.default_rng(44)
    poses = np.ascontiguousarray(w["poses"][rng.integers(0, 16, B)])
    poses[..., 0, :2] += rng.uniform(-0.3, 0.3, (B, 1, 2)).astype(np.float32)  # (the root moves: every frame differs)
    scene = pxr.Scene(w["desc"])
    _bind(torch, scene, w["distractor"])
    frames, ids = scene.render_batch(torch.from_numpy(poses).cuda(), None, step0=2, want_ids=True)
    torch.cuda.synchronize()
    frame_bytes = frames[0].numel()
    assert frames.numel() > 2 ** 32 and ids.numel() * 4 > 2 ** 32
    mark = 2 ** 32 // frame_bytes
    o = orc.Scene(w["desc"])
    for e in (0, 1, mark - 1, mark, mark + 1, 2 ** 32 // (4 * 84 * 84), B - 2, B - 1):
        ref = o.render(poses[e:e + 1], None, step0=2, env0=e, distractor=w["distractor"])
        got = dict(frames=frames[e:e + 1].cpu().numpy(), ids=pxr.ids_to_numpy(ids[e:e + 1]))
        assert_parity(got, ref)
    scene.close()
