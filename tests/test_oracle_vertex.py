"""Pins for the oracle's camera constants and vertex stage against double-precision geometry."""
import numpy as np
import pytest

from helpers import look_at, one_body_scene, pose_row, world_positions
from paper_2502_00021_amd import workloads as wl

RGB = (0.5, 0.5, 0.5)


def _project(desc, world, root_pos):
    """Double-precision pinhole projection to snapped fixed point (8 sub-pixel bits)."""
    Rv, f = look_at(desc)
    eye = np.asarray(root_pos, dtype=np.float64) + np.array(desc["cam_offset"], dtype=np.float64)
    pv = (world - eye) @ Rv.T
    sx = desc["width"] / 2.0 + f * pv[:, 0] / pv[:, 2]
    sy = desc["height"] / 2.0 - f * pv[:, 1] / pv[:, 2]
    return sx * 256.0, sy * 256.0, desc["z_near"] / pv[:, 2], pv


def test_camera_constants(orc):
    desc = one_body_scene(wl.sphere(0.25, RGB), 64, 48, fov_y_deg=50.0, cam_offset=(-2.0, 0.7, 1.3))
    cam = orc.Scene(desc).camera()
    Rv = cam["Rv"].astype(np.float64)
    assert np.allclose(Rv @ Rv.T, np.eye(3), atol=2e-7)
    # right x up points back at the viewer (the camera looks down -z of a right-handed eye frame)
    assert np.allclose(np.cross(Rv[0], Rv[1]), -Rv[2], atol=2e-7)
    Rref, fref = look_at(desc)
    assert np.allclose(Rv, Rref, atol=1e-7)
    assert cam["f"] == pytest.approx(fref, rel=1e-7)
    assert cam["f"] == pytest.approx(24.0 / np.tan(np.radians(25.0)), rel=1e-7)
    i = np.arange(64)
    j = np.arange(48)
    assert np.allclose(cam["cx"], ((i + 0.5) - 32.0) / fref, atol=1e-7)
    assert np.allclose(cam["cy"], -((j + 0.5) - 24.0) / fref, atol=1e-7)
    # antisymmetric about the image centre; rows above the centre look up (positive)
    assert np.array_equal(cam["cx"], -cam["cx"][::-1])
    assert cam["cy"][0] > 0 > cam["cy"][-1]
    lref = np.array(desc["light_dir"]) / np.linalg.norm(desc["light_dir"])
    assert np.allclose(cam["l"], lref, atol=1e-7)
    lit = 0.3 + 0.7 * lref[2]
    assert np.allclose(cam["gs"], np.array([0.35, 0.65]) * lit, atol=1e-7)


@pytest.mark.parametrize("W,H", [(32, 32), (64, 64), (84, 84), (40, 24)])
def test_root_centre_projects_to_image_centre(orc, W, H):
    """The camera looks at the root body: a zero-size root collapses onto exactly (W/2, H/2)."""
    desc = one_body_scene(wl.sphere(0.25, RGB), W, H)
    s = orc.Scene(desc)
    rng = np.random.default_rng(7)
    for _ in range(20):
        pos = rng.uniform(-3, 3, 3)
        pos[2] = abs(pos[2])
        q = wl.random_quats(rng, ())
        out = s.vertex_stage(np.array([[*pos, *q]]), shapes=np.zeros((1, 4)))
        assert not out["rejected"].any()
        assert np.all(np.abs(out["X"] - 128 * W) <= 1) and np.all(np.abs(out["Y"] - 128 * H) <= 1)
        # reversed depth of the look-at point: near / |offset|
        assert np.allclose(out["D"], 0.1 / np.linalg.norm(desc["cam_offset"]), rtol=1e-6)
    out = s.vertex_stage(pose_row((0, 0, 1)), shapes=np.zeros((1, 4)))
    assert np.all(out["X"] == 128 * W) and np.all(out["Y"] == 128 * H)
    assert np.allclose(out["eye"], [-2.5, 0.0, 2.0])


def test_lateral_offset_closed_form(orc):
    """A point at view depth d and lateral offset x lands at W/2 + f*x/d; vertical likewise (y up = smaller row)."""
    W = H = 64
    bodies = [wl.sphere(0.1, RGB), wl.sphere(0.1, RGB)]
    desc = wl.default_scene(W, H, bodies)
    desc["cam_offset"] = (-4.0, 0.0, 0.0)  # looking along +x, right = -y?  computed below, not assumed
    s = orc.Scene(desc)
    Rv, f = look_at(desc)
    root = np.array([0.0, 0.0, 1.0])
    for lateral, vertical, depth in [(0.5, 0.0, 4.0), (0.0, 0.25, 4.0), (-0.3, 0.7, 6.5), (1.0, -0.5, 2.0)]:
        p = root + np.array(desc["cam_offset"]) + depth * Rv[2] + lateral * Rv[0] + vertical * Rv[1]
        poses = np.stack([pose_row(root), pose_row(p)])
        out = s.vertex_stage(poses, shapes=np.zeros((2, 4)))
        v = np.nonzero(s.mesh()["vert_body"] == 1)[0][0]
        assert abs(out["X"][v] - 256.0 * (W / 2 + f * lateral / depth)) <= 1.0
        assert abs(out["Y"][v] - 256.0 * (H / 2 - f * vertical / depth)) <= 1.0
        assert out["D"][v] == pytest.approx(0.1 / depth, rel=1e-6)


@pytest.mark.parametrize("body,shape", [
    (wl.capsule(0.07, 0.2, RGB, 12, 6), (0.07, 0.07, 0.07, 0.2)),
    (wl.sphere(0.25, RGB, 16, 8), (0.25, 0.25, 0.25, 0.0)),
    (wl.box(0.3, 0.2, 0.1, RGB, 4), (0.3, 0.2, 0.1, 0.0)),
])
def test_vertex_stage_matches_double_reference(orc, body, shape):
    """Full chain pose -> rotation -> view -> divide -> snap against float64 textbook formulas."""
    W = H = 64
    bodies = [wl.sphere(0.1, RGB), body]
    desc = wl.default_scene(W, H, bodies)
    s = orc.Scene(desc)
    mesh = s.mesh()
    rng = np.random.default_rng(11)
    worst = 0.0
    for _ in range(25):
        root = np.array([rng.uniform(-1, 1), rng.uniform(-1, 1), rng.uniform(0.5, 1.5)])
        pos = root + rng.uniform(-0.6, 0.6, 3)
        poses = np.stack([np.array([*root, *wl.random_quats(rng, ())]), np.array([*pos, *wl.random_quats(rng, ())])])
        poses = poses.astype(np.float32)
        shapes = [(0.1, 0.1, 0.1, 0.0), shape]
        out = s.vertex_stage(poses, None)
        world = world_positions(mesh, shapes, poses.astype(np.float64))
        X, Y, D, pv = _project(desc, world, poses[0, :3].astype(np.float64))
        assert not out["rejected"].any()
        worst = max(worst, np.abs(out["X"] - X).max(), np.abs(out["Y"] - Y).max())
        assert np.allclose(out["D"], D, rtol=2e-6)
    # fp32 chain error is a small fraction of a sub-pixel unit; rounding adds 0.5
    assert worst <= 0.75


def test_per_env_shape_override(orc):
    """Shapes passed per call replace the scene's (instancing: the template is the unit shape)."""
    desc = one_body_scene(wl.box(0.3, 0.2, 0.1, RGB, 2), 64, 64)
    s = orc.Scene(desc)
    pose = pose_row((0, 0, 1), wl.random_quats(np.random.default_rng(3), ()))
    a = s.vertex_stage(pose, None)
    b = s.vertex_stage(pose, np.array([[0.3, 0.2, 0.1, 0.0]], np.float32))
    c = s.vertex_stage(pose, np.array([[0.6, 0.2, 0.1, 0.0]], np.float32))
    assert np.array_equal(a["X"], b["X"]) and np.array_equal(a["Y"], b["Y"]) and np.array_equal(a["D"], b["D"])
    assert not np.array_equal(a["X"], c["X"])


def test_near_and_guard_rejection(orc):
    bodies = [wl.sphere(0.1, RGB), wl.sphere(0.05, RGB, 8, 4)]
    desc = wl.default_scene(32, 32, bodies)
    s = orc.Scene(desc)
    Rv, f = look_at(desc)
    eye = np.array([0, 0, 1.0]) + np.array(desc["cam_offset"])
    vb = s.mesh()["vert_body"]

    def rejected(p):
        out = s.vertex_stage(np.stack([pose_row((0, 0, 1)), pose_row(p)]))
        r = out["rejected"][vb == 1]
        assert np.all(out["X"][vb == 1][r == 1] == 0)
        return r

    assert rejected(eye - 1.0 * Rv[2]).all()            # behind the camera
    assert rejected(eye + 0.02 * Rv[2]).all()           # in front but inside z_near - radius
    assert not rejected(eye + 0.5 * Rv[2]).any()        # comfortably in front
    r = rejected(eye + 0.1 * Rv[2])                     # straddles the near plane: some in, some out
    assert r.any() and not r.all()
    # far off to the side: |sx| > 16384 px  <=>  |x/z| > (16384 - W/2) / f
    assert rejected(eye + 0.2 * Rv[2] + 200.0 * Rv[0]).all()
    # non-finite pose: everything rejected, no crash
    out = s.vertex_stage(np.stack([pose_row((0, 0, 1)), pose_row((np.nan, 0, 1))]))
    assert out["rejected"][vb == 1].all() and not out["rejected"][vb == 0].any()
