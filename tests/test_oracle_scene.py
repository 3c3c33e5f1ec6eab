"""Scene-level pins for the oracle: orientation, convexity, ray casts, ground plane, shading."""
import numpy as np
import pytest

from helpers import look_at, one_body_scene, pose_row, quat_to_mat, world_positions
from paper_2502_00021_amd import workloads as wl

BG = 0xFFFFFFFF
GROUND = 0xFFFFFFFE
RGB = (0.6, 0.4, 0.8)


def _raster_scene(orc, s, poses, shapes=None, cull=0):
    vs = s.vertex_stage(poses, shapes)
    return orc.raster(s.W, s.H, vs["X"], vs["Y"], vs["D"], s.mesh()["tris"], rejected=vs["rejected"], cull=cull)


# ---------------------------------------------------------------- orientation / convexity

def test_sphere_at_look_at_point_is_a_centred_disc(orc):
    W = H = 128
    r = 0.25
    desc = one_body_scene(wl.sphere(r, RGB, 16, 8), W, H, ground_enabled=False, cam_offset=(-1.5, 0.0, 0.6))
    s = orc.Scene(desc)
    ids, dep, cov = _raster_scene(orc, s, pose_row((0, 0, 1)))
    _, f = look_at(desc)
    d = np.linalg.norm(desc["cam_offset"])
    # silhouette of a sphere under perspective: angular radius asin(r/d) -> image radius f*tan(asin(r/d))
    rad = f * np.tan(np.arcsin(r / d))
    area = np.pi * rad * rad
    n = int((cov > 0).sum())
    assert abs(n - area) <= 2.0 * np.pi * rad * 0.75, (n, area)
    jj, ii = np.nonzero(cov)
    assert abs(ii.mean() + 0.5 - W / 2) < 0.3 and abs(jj.mean() + 0.5 - H / 2) < 0.3
    # roughly half of the triangles face the camera
    front = len(np.unique(ids[ids != BG]))
    assert cov.max() == 1
    assert 0.3 * s.T < front <= 0.55 * s.T
    # nearest point of the sphere is the centre pixel: reversed depth near/(d - r)
    centre = dep[H // 2 - 1:H // 2 + 1, W // 2 - 1:W // 2 + 1].view(np.float32)
    assert np.allclose(centre, 0.1 / (d - r), rtol=2e-3)
    assert centre.max() == dep.view(np.float32).max()


@pytest.mark.parametrize("body", [wl.capsule(0.12, 0.3, RGB, 12, 6), wl.sphere(0.3, RGB, 16, 8),
                                  wl.box(0.3, 0.2, 0.25, RGB, 4), wl.capsule(0.046, 0.2, RGB, 12, 6)])
def test_convex_body_cover_count_and_front_equals_back(orc, body):
    """Closed convex mesh: each pixel is under at most one front face, and the back faces cover the same set."""
    W = H = 48
    desc = one_body_scene(body, W, H, cam_offset=(-1.4, 0.0, 0.6))
    s = orc.Scene(desc)
    rng = np.random.default_rng(17)
    for _ in range(12):
        pose = pose_row((0, 0, 1), wl.random_quats(rng, ()))
        _, _, cov_f = _raster_scene(orc, s, pose, cull=0)
        _, _, cov_b = _raster_scene(orc, s, pose, cull=1)
        assert cov_f.max() == 1 and cov_b.max() == 1
        assert np.array_equal(cov_f, cov_b)
        assert cov_f.sum() > 10


# ---------------------------------------------------------------- ray casts

def _pixel_rays(desc, root_pos, di=0.0, dj=0.0):
    Rv, f = look_at(desc)
    W, H = desc["width"], desc["height"]
    i = np.arange(W)[None, :] + 0.5 + di
    j = np.arange(H)[:, None] + 0.5 + dj
    cx = (i - W / 2) / f
    cy = -(j - H / 2) / f
    dirs = cx[..., None] * Rv[0] + cy[..., None] * Rv[1] + Rv[2]
    eye = np.asarray(root_pos, dtype=np.float64) + np.array(desc["cam_offset"], dtype=np.float64)
    return eye, dirs  # dirs have unit view depth: the ray parameter IS the view depth


def _ray_sphere(eye, dirs, c, r):
    oc = eye - c
    a = np.einsum("...k,...k->...", dirs, dirs)
    b = 2.0 * np.einsum("...k,k->...", dirs, oc)
    cc = oc @ oc - r * r
    disc = b * b - 4 * a * cc
    t = np.where(disc >= 0, (-b - np.sqrt(np.maximum(disc, 0))) / (2 * a), np.inf)
    return np.where(t > 0, t, np.inf)


def _ray_capsule(eye, dirs, c, R, r, h):
    """Nearest hit of a capsule (axis = R[:,2], half-length h, radius r): cylinder part + two cap spheres."""
    ax = R[:, 2]
    oc = eye - c
    dpar = dirs @ ax
    dperp = dirs - dpar[..., None] * ax
    opar = oc @ ax
    operp = oc - opar * ax
    a = np.einsum("...k,...k->...", dperp, dperp)
    b = 2.0 * np.einsum("...k,k->...", dperp, operp)
    cc = operp @ operp - r * r
    disc = b * b - 4 * a * cc
    t = np.where(disc >= 0, (-b - np.sqrt(np.maximum(disc, 0))) / (2 * a), np.inf)
    z = opar + t * dpar
    t_cyl = np.where((t > 0) & (np.abs(z) <= h), t, np.inf)
    return np.minimum(t_cyl, np.minimum(_ray_sphere(eye, dirs, c + h * ax, r), _ray_sphere(eye, dirs, c - h * ax, r)))


def _analytic_body_map(desc, poses, di=0.0, dj=0.0):
    eye, dirs = _pixel_rays(desc, poses[desc["root_body"], :3], di, dj)
    best_t = np.full(dirs.shape[:2], np.inf)
    best = np.full(dirs.shape[:2], -1)
    for b, body in enumerate(desc["bodies"]):
        c = poses[b, :3].astype(np.float64)
        if body["kind"] == "sphere":
            t = _ray_sphere(eye, dirs, c, body["shape"][0])
        else:
            t = _ray_capsule(eye, dirs, c, quat_to_mat(poses[b, 3:7]), body["shape"][0], body["shape"][3])
        upd = t < best_t
        best_t[upd] = t[upd]
        best[upd] = b
    return best, best_t


def test_body_map_matches_analytic_ray_cast(orc):
    """Which body owns a pixel equals an exact ray cast against the true capsules/spheres, away from silhouettes."""
    W = H = 48
    bodies = [wl.sphere(0.22, RGB, 16, 8), wl.capsule(0.1, 0.25, RGB, 12, 6), wl.capsule(0.08, 0.2, RGB, 12, 6)]
    desc = wl.default_scene(W, H, bodies)
    desc["cam_offset"] = (-1.6, 0.0, 0.7)
    desc["ground_enabled"] = False
    s = orc.Scene(desc)
    tri_body = s.mesh()["tri_body"]
    rng = np.random.default_rng(23)
    checked = owned = 0
    for _ in range(10):
        poses = np.zeros((3, 7), np.float32)
        poses[0] = pose_row((0, 0, 1), wl.random_quats(rng, ()))
        for b in (1, 2):
            poses[b] = pose_row((rng.uniform(-0.3, 0.3), rng.uniform(-0.45, 0.45), 1 + rng.uniform(-0.35, 0.35)),
                                wl.random_quats(rng, ()))
        ids = s.render(poses[None, None])["ids"][0, 0]
        got = np.where(ids == BG, -1, tri_body[np.minimum(ids, s.T - 1)].astype(np.int64))
        got[ids == BG] = -1
        ref, _ = _analytic_body_map(desc, poses)
        stable = np.ones_like(ref, dtype=bool)
        for di, dj in [(-.75, 0), (.75, 0), (0, -.75), (0, .75), (-.55, -.55), (.55, .55), (-.55, .55), (.55, -.55)]:
            stable &= _analytic_body_map(desc, poses, di, dj)[0] == ref
        assert np.array_equal(got[stable], ref[stable])
        checked += int(stable.sum())
        owned += int((ref[stable] >= 0).sum())
    assert checked > 0.8 * 10 * W * H and owned > 1000


def _moller_trumbore(eye, dirs, tri):
    """Ray/triangle parameter (np.inf for a miss) for a grid of rays, double precision, front or back."""
    a, b, c = tri
    e1, e2 = b - a, c - a
    p = np.cross(dirs, e2)
    det = p @ e1
    ok = np.abs(det) > 1e-14
    inv = np.where(ok, 1.0 / np.where(ok, det, 1.0), 0.0)
    tv = eye - a
    u = (p @ tv) * inv
    q = np.cross(tv, e1)
    v = (dirs @ q) * inv
    t = (e2 @ q) * inv
    hit = ok & (u >= 0) & (v >= 0) & (u + v <= 1) & (t > 0)
    return np.where(hit, t, np.inf)


def _brute_force_ids(desc, world, tris, root_pos, di=0.0, dj=0.0):
    eye, dirs = _pixel_rays(desc, root_pos, di, dj)
    best_t = np.full(dirs.shape[:2], np.inf)
    second = np.full(dirs.shape[:2], np.inf)
    best = np.full(dirs.shape[:2], BG, dtype=np.int64)
    for g, t3 in enumerate(tris):
        t = _moller_trumbore(eye, dirs, world[t3])
        upd = t < best_t
        second = np.where(upd, best_t, np.minimum(second, t))
        best_t = np.where(upd, t, best_t)
        best[upd] = g
    return best, best_t, second


def test_triangle_ids_match_brute_force_ray_cast(orc):
    """Winning triangle per pixel equals a per-pixel ray cast against the un-snapped world triangles."""
    W = H = 24
    bodies = [wl.box(0.3, 0.25, 0.2, RGB, 2), wl.capsule(0.12, 0.2, RGB, 6, 2), wl.sphere(0.2, RGB, 8, 3)]
    desc = wl.default_scene(W, H, bodies)
    desc["cam_offset"] = (-1.3, 0.0, 0.6)
    desc["ground_enabled"] = False
    s = orc.Scene(desc)
    mesh = s.mesh()
    tris = mesh["tris"].astype(np.int64)
    shapes = [b["shape"] for b in bodies]
    rng = np.random.default_rng(29)
    checked = owned = 0
    for _ in range(6):
        poses = np.zeros((3, 7), np.float32)
        poses[0] = pose_row((0, 0, 1), wl.random_quats(rng, ()))
        for b in (1, 2):
            poses[b] = pose_row((rng.uniform(-0.2, 0.3), rng.uniform(-0.4, 0.4), 1 + rng.uniform(-0.3, 0.3)),
                                wl.random_quats(rng, ()))
        out = s.render(poses[None, None], want_depth=True)
        ids = out["ids"][0, 0].astype(np.int64)
        world = world_positions(mesh, shapes, poses.astype(np.float64))
        ref, t1, t2 = _brute_force_ids(desc, world, tris, poses[0, :3])
        eps = 3.0 / 256.0
        stable = np.ones_like(ref, dtype=bool)
        for di, dj in [(-eps, 0), (eps, 0), (0, -eps), (0, eps), (-eps, -eps), (eps, eps), (-eps, eps), (eps, -eps)]:
            stable &= _brute_force_ids(desc, world, tris, poses[0, :3], di, dj)[0] == ref
        # interpenetrating bodies: skip pixels whose two nearest hits nearly tie in reversed depth
        with np.errstate(divide="ignore", invalid="ignore"):
            tie = np.abs(0.1 / t1 - 0.1 / t2) < 1e-5
        stable &= ~np.where(np.isfinite(t2), tie, False)
        assert np.array_equal(ids[stable], ref[stable])
        hit = stable & (ref != BG)
        depth = out["depth_bits"][0, 0].view(np.float32)
        assert np.allclose(depth[hit], 0.1 / t1[hit], rtol=3e-3)
        checked += int(stable.sum())
        owned += int(hit.sum())
    assert checked > 0.9 * 6 * W * H and owned > 500


def test_mesh_triangle_ids_match_brute_force_ray_cast(orc):
    """Caller-supplied closed meshes (a non-convex torus, an icosphere, a tetrahedron) against the same ray cast."""
    W = H = 24
    tv, tt = wl.torus_mesh(0.3, 0.12, 8, 5)
    iv, it = wl.icosphere_mesh(0.2, 1)
    tet_v = np.array([[0.3, 0, -0.2], [-0.2, 0.3, -0.2], [-0.2, -0.3, -0.2], [0, 0, 0.35]], np.float32)
    tet_t = np.array([[0, 2, 1], [0, 1, 3], [1, 2, 3], [2, 0, 3]], np.uint32)
    bodies = [wl.mesh(tv, tt, RGB), wl.mesh(iv, it, RGB, scale=(1.0, 1.5, 0.8)), wl.mesh(tet_v, tet_t, RGB)]
    desc = wl.default_scene(W, H, bodies)
    desc["cam_offset"] = (-1.3, 0.0, 0.6)
    desc["ground_enabled"] = False
    s = orc.Scene(desc)
    mesh = s.mesh()
    tris = mesh["tris"].astype(np.int64)
    shapes = [b["shape"] for b in bodies]
    rng = np.random.default_rng(31)
    checked = owned = 0
    for _ in range(6):
        poses = np.zeros((3, 7), np.float32)
        poses[0] = pose_row((0, 0, 1), wl.random_quats(rng, ()))
        for b in (1, 2):
            poses[b] = pose_row((rng.uniform(-0.2, 0.3), rng.uniform(-0.5, 0.5), 1 + rng.uniform(-0.3, 0.3)),
                                wl.random_quats(rng, ()))
        out = s.render(poses[None, None], want_depth=True)
        ids = out["ids"][0, 0].astype(np.int64)
        world = world_positions(mesh, shapes, poses.astype(np.float64))
        ref, t1, t2 = _brute_force_ids(desc, world, tris, poses[0, :3])
        eps = 3.0 / 256.0
        stable = np.ones_like(ref, dtype=bool)
        for di, dj in [(-eps, 0), (eps, 0), (0, -eps), (0, eps), (-eps, -eps), (eps, eps), (-eps, eps), (eps, -eps)]:
            stable &= _brute_force_ids(desc, world, tris, poses[0, :3], di, dj)[0] == ref
        with np.errstate(divide="ignore", invalid="ignore"):
            tie = np.abs(0.1 / t1 - 0.1 / t2) < 1e-5
        stable &= ~np.where(np.isfinite(t2), tie, False)
        assert np.array_equal(ids[stable], ref[stable])
        hit = stable & (ref != BG)
        depth = out["depth_bits"][0, 0].view(np.float32)
        assert np.allclose(depth[hit], 0.1 / t1[hit], rtol=3e-3)
        checked += int(stable.sum())
        owned += int(hit.sum())
    assert checked > 0.85 * 6 * W * H and owned > 400


# ---------------------------------------------------------------- ground plane

def test_horizon_row_and_checker_parity(orc):
    W, H = 40, 48
    desc = one_body_scene(wl.sphere(0.1, RGB, 8, 4), W, H)
    s = orc.Scene(desc)
    cam = s.camera()
    poses = pose_row((0.3, -0.2, 1.0))[None, None, None]
    shapes = np.zeros((1, 1, 4), np.float32)  # collapse the body to a point: only ground and sky remain
    out = s.render(poses, shapes)
    ids, fr = out["ids"][0, 0], out["frames"][0, 0]
    Rv, f = look_at(desc)
    eye = np.array([0.3, -0.2, 1.0]) + np.array(desc["cam_offset"])
    assert abs(Rv[0][2]) < 1e-12  # no roll: the horizon is a pixel row
    j = np.arange(H)
    ndz = Rv[1][2] * (j + 0.5 - H / 2) / f - Rv[2][2]
    is_ground = (ndz > 0) & (eye[2] / np.where(ndz > 0, ndz, 1) <= desc["z_far"])
    j_h = int(np.argmax(is_ground))
    assert 0 < j_h < H and is_ground[j_h:].all()
    assert np.all(ids[:j_h] == BG) and np.all(ids[j_h:] == GROUND)
    bg_u8 = np.floor(255.0 * np.array(desc["background_rgb"], np.float32) + 0.5).astype(np.uint8)
    assert np.all(fr[:j_h] == bg_u8)
    # analytic hit point of every ground pixel -> checker parity -> grey level
    eye_d, dirs = _pixel_rays(desc, (0.3, -0.2, 1.0))
    t = eye_d[2] / -dirs[..., 2]
    wx, wy = eye_d[0] + t * dirs[..., 0], eye_d[1] + t * dirs[..., 1]
    par = (np.floor(wx).astype(np.int64) + np.floor(wy).astype(np.int64)) & 1
    margin = np.minimum(np.abs(wx - np.round(wx)), np.abs(wy - np.round(wy)))
    safe = (margin > 1e-3 * np.maximum(1.0, t)) & (np.arange(H)[:, None] >= j_h)
    grey = np.floor(255.0 * cam["gs"].astype(np.float64)[par] + 0.5).astype(np.uint8)
    assert safe.sum() > 0.9 * (H - j_h) * W
    assert np.all(fr[..., 0][safe] == grey[safe])
    assert np.all(fr[j_h:, :, 1] == fr[j_h:, :, 0]) and np.all(fr[j_h:, :, 2] == fr[j_h:, :, 0])
    assert len(np.unique(par[safe])) == 2
    # ground off, or camera below the plane: sky only
    off = dict(desc, ground_enabled=False)
    assert np.all(orc.Scene(off).render(poses, shapes)["ids"] == BG)
    low = pose_row((0.3, -0.2, -1.5))[None, None, None]
    assert np.all(s.render(low, shapes)["ids"] == BG)


def test_capsule_through_ground_boundary_row(orc):
    """A vertical capsule dipping below z=0 meets the ground where similar triangles say it should."""
    W = H = 64
    r, h = 0.15, 0.4
    desc = one_body_scene(wl.capsule(r, h, RGB, 24, 6), W, H)
    s = orc.Scene(desc)
    root = np.array([0.0, 0.0, 0.1])
    out = s.render(pose_row(root)[None, None, None])
    ids = out["ids"][0, 0]
    Rv, f = look_at(desc)
    eye = root + np.array(desc["cam_offset"])
    contact = np.array([-r, 0.0, 0.0])  # the camera sits at -x: nearest generator of the cylinder meets z=0 here
    pv = Rv @ (contact - eye)
    row = H / 2 - f * pv[1] / pv[2]
    col = ids[:, W // 2]
    is_tri = col < GROUND
    last = int(np.nonzero(is_tri)[0].max())
    assert abs((last + 1) - row) <= 1.0
    assert np.all(col[last + 1:] == GROUND)
    assert is_tri[int(row) - 5:last + 1].all()


# ---------------------------------------------------------------- shading

def _box_front_face_scene(light_dir):
    body = wl.box(0.4, 0.4, 0.4, (0.6, 0.4, 0.8), 2)
    return one_body_scene(body, 32, 32, cam_offset=(-2.0, 0.0, 0.0), light_dir=light_dir, ground_enabled=False)


def test_shade_extremes(orc):
    rgb = np.array([0.6, 0.4, 0.8], np.float32)
    # light shining straight onto the camera-facing (-x) face: full intensity, ambient + diffuse = 1
    s = orc.Scene(_box_front_face_scene((-1.0, 0.0, 0.0)))
    out = s.render(pose_row((0, 0, 1))[None, None, None])
    ids, fr = out["ids"][0, 0], out["frames"][0, 0]
    mesh = s.mesh()
    vis = ids != BG
    assert vis.sum() > 100
    assert np.all(mesh["normals"][ids[vis]] == np.array([-1.0, 0.0, 0.0], np.float32))
    mul = mesh["mul"][ids[vis]]
    assert set(np.unique(mul)) == {0.5, 1.0}
    expect = np.floor(255.0 * (rgb[None, :] * mul[:, None]) * np.float32(1.0) + 0.5).astype(np.uint8)
    assert np.array_equal(fr[vis], expect)
    # light from behind the face: ambient only
    s = orc.Scene(_box_front_face_scene((1.0, 0.0, 0.0)))
    out = s.render(pose_row((0, 0, 1))[None, None, None])
    fr2 = out["frames"][0, 0]
    expect2 = 255.0 * 0.3 * (rgb[None, :].astype(np.float64) * mul[:, None])
    assert np.all(np.abs(fr2[vis].astype(np.float64) - expect2) <= 0.5 + 1e-4)
    # grazing light (perpendicular to the normal): still ambient only, never negative
    s = orc.Scene(_box_front_face_scene((0.0, 0.0, 1.0)))
    fr3 = s.render(pose_row((0, 0, 1))[None, None, None])["frames"][0, 0]
    assert np.array_equal(fr3[vis], fr2[vis])


def test_lambert_follows_body_rotation(orc):
    """Rotating the body rotates its normals: intensity = max(0, n_world . l) with n_world = R n_body."""
    W = H = 48
    desc = one_body_scene(wl.box(0.3, 0.3, 0.3, (0.9, 0.9, 0.9), 1), W, H, cam_offset=(-1.5, 0.0, 0.5),
                          ground_enabled=False)
    s = orc.Scene(desc)
    mesh = s.mesh()
    l = np.array(desc["light_dir"]) / np.linalg.norm(desc["light_dir"])
    rng = np.random.default_rng(31)
    for _ in range(8):
        q = wl.random_quats(rng, ())
        out = s.render(pose_row((0, 0, 1), q)[None, None, None])
        ids, fr = out["ids"][0, 0], out["frames"][0, 0]
        vis = ids != BG
        n_world = mesh["normals"][ids[vis]].astype(np.float64) @ quat_to_mat(q).T
        inten = np.maximum(0.0, n_world @ l)
        expect = 255.0 * np.minimum(1.0, 0.9 * (0.3 + 0.7 * inten))
        assert np.all(np.abs(fr[vis][:, 0].astype(np.float64) - expect) <= 0.5 + 2e-3)
        assert vis.sum() > 50


def test_ground_grey_levels(orc):
    desc = one_body_scene(wl.sphere(0.1, RGB, 8, 4), 32, 32)
    s = orc.Scene(desc)
    out = s.render(pose_row((0, 0, 1))[None, None, None], np.zeros((1, 1, 4), np.float32))
    fr, ids = out["frames"][0, 0], out["ids"][0, 0]
    lz = 0.85 / np.linalg.norm(desc["light_dir"])
    levels = {int(np.floor(255 * g * (0.3 + 0.7 * lz) + 0.5)) for g in desc["ground_grey"]}
    assert set(np.unique(fr[ids == GROUND])) == levels


def test_ground_cell_index_beyond_int32_saturates(orc):
    """A camera billions of metres from the origin puts the checker's cell index outside int32.  The
    conversion is defined as saturating (NaN -> 0), so the x index is the same odd number for every such camera
    and the pattern is decided by y alone; it must not depend on how far beyond the range the camera is."""
    desc = one_body_scene(wl.sphere(0.1, RGB, 6, 3), 32, 24)
    s = orc.Scene(desc)

    def ground_rgb(x, y=0.3):
        o = s.render(pose_row((x, y, 1.0))[None, None, None])
        assert (o["ids"][0, 0] == GROUND).sum() > 100
        return np.where((o["ids"][0, 0] == GROUND)[..., None], o["frames"][0, 0], 0)

    far, farther, neg = ground_rgb(3.0e9), ground_rgb(7.5e9), ground_rgb(-6.0e9)
    assert np.array_equal(far, farther)
    # INT32_MAX is odd and INT32_MIN even: the two ends show complementary checkers
    greys = np.unique(far[far > 0])
    assert len(greys) == 2
    swapped = np.where(far == greys[0], greys[1], np.where(far == greys[1], greys[0], 0))
    assert np.array_equal(neg, swapped)
    # infinities and NaN are defined too (NaN counts as cell 0: the same parity as INT32_MIN)
    assert np.array_equal(ground_rgb(np.inf), far)
    assert np.array_equal(ground_rgb(np.nan), neg)
