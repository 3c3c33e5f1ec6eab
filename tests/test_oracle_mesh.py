"""Pins for the oracle's template meshes: counts, closedness, orientation, volume, radius, normals."""
import numpy as np
import pytest

from helpers import local_positions
from paper_2502_00021_amd import workloads as wl

RGB = (0.5, 0.5, 0.5)


def _scene(orc, body):
    return orc.Scene(wl.default_scene(32, 32, [body]))


def _weld(pos, tris):
    """Merge coincident vertices (box faces do not share theirs)."""
    key = np.round(pos * 1e6).astype(np.int64)
    _, inv = np.unique(key, axis=0, return_inverse=True)
    return inv.reshape(-1)[tris]


def _edge_check(tris):
    """Every directed edge appears once and its reverse appears once: closed, consistently oriented."""
    e = np.concatenate([tris[:, [0, 1]], tris[:, [1, 2]], tris[:, [2, 0]]]).astype(np.int64)
    fwd = {(a, b) for a, b in e}
    assert len(fwd) == len(e), "a directed edge is used twice"
    for a, b in e:
        assert (b, a) in fwd, "edge without an opposite partner: mesh not closed"
    return len(e) // 2


def _signed_volume(pos, tris):
    a, b, c = pos[tris[:, 0]], pos[tris[:, 1]], pos[tris[:, 2]]
    return float(np.einsum("ij,ij->i", a, np.cross(b, c)).sum() / 6.0)


@pytest.mark.parametrize("L,M", [(3, 1), (8, 4), (12, 6), (16, 8), (5, 3)])
def test_capsule_counts_closed_euler(orc, L, M):
    s = _scene(orc, wl.capsule(0.07, 0.2, RGB, L, M))
    assert s.V == 2 * L * M + 2
    assert s.T == 4 * L * M
    m = s.mesh()
    tris = m["tris"].astype(np.int64)
    assert tris.min() == 0 and tris.max() == s.V - 1
    E = _edge_check(tris)
    assert s.V - E + s.T == 2
    assert set(np.unique(m["uverts"][:, 3])) == {-1.0, 1.0}
    assert np.all(m["mul"] == 1.0)


@pytest.mark.parametrize("L,M", [(3, 1), (16, 8), (12, 6), (7, 2)])
def test_sphere_counts_closed_euler(orc, L, M):
    s = _scene(orc, wl.sphere(0.25, RGB, L, M))
    assert s.V == (2 * M - 1) * L + 2
    assert s.T == 2 * L * (2 * M - 1)
    m = s.mesh()
    E = _edge_check(m["tris"].astype(np.int64))
    assert s.V - E + s.T == 2
    assert np.all(m["uverts"][:, 3] == 0.0)
    # the equator ring lies exactly in the z = 0 plane
    assert np.count_nonzero(m["uverts"][:, 2] == 0.0) == L


@pytest.mark.parametrize("n", [1, 2, 4, 5])
def test_box_counts_closed_euler_checker(orc, n):
    s = _scene(orc, wl.box(0.3, 0.2, 0.1, RGB, n))
    assert s.V == 6 * (n + 1) ** 2
    assert s.T == 12 * n * n
    m = s.mesh()
    pos = local_positions(m, [(0.3, 0.2, 0.1, 0.0)])
    welded = _weld(pos, m["tris"].astype(np.int64))
    E = _edge_check(welded)
    assert len(np.unique(welded)) - E + s.T == 2
    assert np.abs(pos).max(axis=0).tolist() == pytest.approx([0.3, 0.2, 0.1])
    mul = m["mul"].reshape(6, n, n, 2)
    assert np.all(mul[..., 0] == mul[..., 1]), "both triangles of a cell share the multiplier"
    cu, cv = np.meshgrid(np.arange(n), np.arange(n))
    expect = np.where((cu + cv) % 2 == 0, 1.0, 0.5)
    for f in range(6):
        assert np.array_equal(mul[f, :, :, 0], expect)


def test_capsule_vertices_on_surface(orc):
    r, h = 0.07, 0.2
    s = _scene(orc, wl.capsule(r, h, RGB, 12, 6))
    pos = local_positions(s.mesh(), [(r, r, r, h)])
    zc = np.clip(pos[:, 2], -h, h)
    dist = np.sqrt(pos[:, 0] ** 2 + pos[:, 1] ** 2 + (pos[:, 2] - zc) ** 2)
    assert np.allclose(dist, r, atol=1e-6)
    assert pos[:, 2].max() == pytest.approx(h + r, abs=1e-7)
    assert pos[:, 2].min() == pytest.approx(-h - r, abs=1e-7)
    # both equator rings sit exactly at z = +h and z = -h
    assert np.count_nonzero(np.abs(pos[:, 2] - h) < 1e-12) == 12
    assert np.count_nonzero(np.abs(pos[:, 2] + h) < 1e-12) == 12


def test_volume_positive_and_converges_from_below(orc):
    r, h = 0.07, 0.2
    exact = np.pi * r * r * (2 * h) + 4.0 / 3.0 * np.pi * r ** 3
    prev = 0.0
    for L, M in [(6, 3), (12, 6), (24, 12), (48, 24)]:
        s = _scene(orc, wl.capsule(r, h, RGB, L, M))
        m = s.mesh()
        vol = _signed_volume(local_positions(m, [(r, r, r, h)]), m["tris"].astype(np.int64))
        assert 0.0 < prev < vol < exact or (prev == 0.0 and 0.0 < vol < exact)
        prev = vol
    assert prev == pytest.approx(exact, rel=5e-3)
    s = _scene(orc, wl.sphere(0.25, RGB, 48, 24))
    m = s.mesh()
    vol = _signed_volume(local_positions(m, [(0.25, 0.25, 0.25, 0.0)]), m["tris"].astype(np.int64))
    assert 0.0 < vol < 4.0 / 3.0 * np.pi * 0.25 ** 3
    assert vol == pytest.approx(4.0 / 3.0 * np.pi * 0.25 ** 3, rel=5e-3)
    s = _scene(orc, wl.box(0.3, 0.2, 0.1, RGB, 4))
    m = s.mesh()
    vol = _signed_volume(local_positions(m, [(0.3, 0.2, 0.1, 0.0)]), m["tris"].astype(np.int64))
    assert vol == pytest.approx(8 * 0.3 * 0.2 * 0.1, rel=1e-6)


@pytest.mark.parametrize("body,shape", [
    (wl.capsule(0.07, 0.2, RGB, 12, 6), (0.07, 0.07, 0.07, 0.2)),
    (wl.sphere(0.25, RGB, 16, 8), (0.25, 0.25, 0.25, 0.0)),
    (wl.box(0.3, 0.2, 0.1, RGB, 4), (0.3, 0.2, 0.1, 0.0)),
])
def test_normals_unit_outward_and_match_geometry(orc, body, shape):
    s = _scene(orc, body)
    m = s.mesh()
    n = m["normals"].astype(np.float64)
    assert np.allclose(np.linalg.norm(n, axis=1), 1.0, atol=1e-6)
    pos = local_positions(m, [shape])
    t = m["tris"].astype(np.int64)
    a, b, c = pos[t[:, 0]], pos[t[:, 1]], pos[t[:, 2]]
    geo = np.cross(b - a, c - a)
    geo /= np.linalg.norm(geo, axis=1, keepdims=True)
    # the stored normal is the geometric face normal of the posed triangle (isotropic shapes, box faces);
    # winding is outward-counter-clockwise, so the two agree in sign as well
    assert np.all(np.einsum("ij,ij->i", n, geo) > 0.999)
    centroid = (a + b + c) / 3.0
    if body["kind"] == "capsule":
        centroid[:, 2] -= np.clip(centroid[:, 2], -shape[3], shape[3])
    assert np.all(np.einsum("ij,ij->i", n, centroid) > 0.0)


def test_bodies_concatenate_in_descriptor_order(orc):
    bodies = [wl.capsule(0.05, 0.1, RGB, 8, 4), wl.sphere(0.2, RGB, 16, 8), wl.box(0.1, 0.1, 0.1, RGB, 4)]
    s = orc.Scene(wl.default_scene(32, 32, bodies))
    m = s.mesh()
    nv = [2 * 8 * 4 + 2, 15 * 16 + 2, 150]
    nt = [128, 480, 192]
    assert s.V == sum(nv) and s.T == sum(nt)
    assert np.array_equal(m["vert_body"], np.repeat(np.arange(3), nv))
    assert np.array_equal(m["tri_body"], np.repeat(np.arange(3), nt))
    vb = m["vert_body"][m["tris"].astype(np.int64)]
    assert np.all(vb == m["tri_body"][:, None]), "a triangle indexes another body's vertices"


# ---------------------------------------------------------------- caller-supplied triangle meshes

def _as_mesh_body(orc, prim, rgb):
    """The primitive's own template, handed back as a vertex / index buffer."""
    m = orc.Scene(wl.default_scene(16, 16, [prim])).mesh()
    assert np.all(m["uverts"][:, 3] == 0)  # no cap selector: boxes and spheres only
    return wl.mesh(m["uverts"][:, :3], m["tris"], rgb, scale=prim["shape"][:3], mul=m["mul"])


def test_mesh_body_reproduces_the_box_primitive(orc):
    """Same vertices, same triangle order, axis-aligned faces (cross products are exact): identical frames."""
    rgb = (0.7, 0.5, 0.3)
    box = wl.box(0.3, 0.2, 0.25, rgb, 3)
    rng = np.random.default_rng(3)
    poses = np.zeros((6, 1, 1, 7), np.float32)
    poses[:, 0, 0, :3] = (0, 0, 1)
    poses[:, 0, 0, 3:] = wl.random_quats(rng, (6,))
    a = orc.Scene(wl.default_scene(48, 40, [box])).render(poses)
    sm = orc.Scene(wl.default_scene(48, 40, [_as_mesh_body(orc, box, rgb)]))
    b = sm.render(poses)
    assert np.array_equal(a["ids"], b["ids"]) and np.array_equal(a["frames"], b["frames"])
    assert (a["ids"] < 0xFFFFFFFE).mean() > 0.02
    assert np.array_equal(sm.mesh()["normals"], orc.Scene(wl.default_scene(16, 16, [box])).mesh()["normals"])


def test_mesh_body_reproduces_the_sphere_up_to_normal_rounding(orc):
    """Same vertices and order: coverage identical; the normals are recomputed from the fp32 vertices, so
    shading may move by one quantisation step."""
    rgb = (0.4, 0.6, 0.8)
    sph = wl.sphere(0.3, rgb, 10, 4)
    rng = np.random.default_rng(4)
    poses = np.zeros((4, 1, 1, 7), np.float32)
    poses[:, 0, 0, :3] = (0, 0, 1)
    poses[:, 0, 0, 3:] = wl.random_quats(rng, (4,))
    a = orc.Scene(wl.default_scene(64, 64, [sph])).render(poses)
    sm = orc.Scene(wl.default_scene(64, 64, [_as_mesh_body(orc, sph, rgb)]))
    b = sm.render(poses)
    assert np.array_equal(a["ids"], b["ids"])
    assert np.abs(a["frames"].astype(int) - b["frames"].astype(int)).max() <= 1
    n = sm.mesh()["normals"].astype(np.float64)
    assert np.allclose(np.linalg.norm(n, axis=1), 1.0, atol=1e-6)
    assert np.abs(n - orc.Scene(wl.default_scene(16, 16, [sph])).mesh()["normals"]).max() < 1e-6


def test_mesh_normals_scale_multipliers_and_errors(orc):
    verts = np.array([[0, 0, 0], [1, 0, 0], [0, 1, 0], [0, 0, 1], [2, 0, 0]], np.float32)
    tris = np.array([[0, 1, 2], [0, 2, 1], [0, 3, 1], [0, 1, 4]], np.uint32)  # the last one has no area
    body = wl.mesh(verts, tris, (0.5, 0.5, 0.5), scale=(2.0, 3.0, 4.0), mul=[1.0, 0.5, 0.25, 1.0])
    s = orc.Scene(wl.default_scene(16, 16, [body]))
    m = s.mesh()
    assert (s.V, s.T) == (5, 4)
    assert np.array_equal(m["normals"], np.array([[0, 0, 1], [0, 0, -1], [0, 1, 0], [0, 0, 0]], np.float32))
    assert np.array_equal(m["mul"], np.array([1.0, 0.5, 0.25, 1.0], np.float32))
    assert np.array_equal(m["uverts"], np.concatenate([verts, np.zeros((5, 1), np.float32)], axis=1))
    # posed like any template: scaled per axis, then rotated and translated
    vs = s.vertex_stage(np.array([[0, 0, 1, 1, 0, 0, 0]], np.float32))
    ref = orc.Scene(wl.default_scene(16, 16, [wl.mesh(verts * np.array([2, 3, 4], np.float32), tris, (0.5,) * 3)]))
    vr = ref.vertex_stage(np.array([[0, 0, 1, 1, 0, 0, 0]], np.float32))
    assert np.array_equal(vs["X"], vr["X"]) and np.array_equal(vs["Y"], vr["Y"])
    bad = wl.mesh(verts, np.array([[0, 1, 5]], np.uint32), (0.5,) * 3)
    with pytest.raises(ValueError):
        orc.Scene(wl.default_scene(16, 16, [bad]))


def test_mesh_workload_structure(orc):
    w = wl.cfg_mesh(B=6)
    s = orc.Scene(w["desc"])
    tv, tt = wl.torus_mesh(0.3, 0.1, 20, 10)
    iv, it = wl.icosphere_mesh(0.2, 2)
    assert (s.V, s.T) == (2 * 12 * 6 + 2 + len(tv) + len(iv) + 13 * 13, 288 + len(tt) + len(it) + 288)
    assert (len(tv), len(tt), len(iv), len(it)) == (200, 400, 162, 320)
    # closed, consistently outward meshes: every edge is used once in each direction, volume matches the solid
    for v, t, vol in [(tv, tt, 2 * np.pi ** 2 * 0.3 * 0.1 ** 2), (iv, it, 4 / 3 * np.pi * 0.2 ** 3)]:
        edges = np.concatenate([t[:, [0, 1]], t[:, [1, 2]], t[:, [2, 0]]]).astype(np.int64)
        fwd = set(map(tuple, edges))
        assert len(fwd) == len(edges) and fwd == set(map(tuple, edges[:, ::-1]))
        v64 = v.astype(np.float64)
        got = np.einsum("ij,ij->i", v64[t[:, 0]], np.cross(v64[t[:, 1]], v64[t[:, 2]])).sum() / 6
        assert 0.8 * vol < got < vol
    out = s.render(w["poses"], distractor=w["distractor"])
    for lo, hi in [(0, 288), (288, 688), (688, 1008), (1008, 1296)]:  # every body is seen somewhere
        assert ((out["ids"] >= lo) & (out["ids"] < hi)).any()
