"""Pins for the oracle's coverage and depth rules on hand-built snapped triangle soups.

Coordinates are fixed point with 8 sub-pixel bits; pixel (i,j) has its centre
at (256 i + 128, 256 j + 128).  The renderer's screen order is (v0, v2, v1),
so a triangle listed counter-clockwise in the y-down raster frame (v0 -> v1 ->
v2 turning left on screen as drawn with y down = clockwise in integers' sign)
is front facing; `_front` below lists vertices so that they survive the cull.
"""
from fractions import Fraction
from math import ceil

import numpy as np
import pytest

BG = 0xFFFFFFFF


def _front(a, b, c):
    """Order three points so that the oracle keeps the triangle (positive area in its screen order)."""
    (ax, ay), (bx, by), (cx, cy) = a, b, c
    # screen order is (v0, v2, v1); area2 of that must be > 0
    area = (cx - ax) * (by - ay) - (cy - ay) * (bx - ax)
    return (a, b, c) if area > 0 else (a, c, b)


def _soup(tri_pts, depths=None):
    """Flatten a list of triangles (each 3 (x,y) points) into unshared vertex arrays."""
    X, Y, D, T = [], [], [], []
    for k, t in enumerate(tri_pts):
        for q, (x, y) in enumerate(t):
            X.append(int(x))
            Y.append(int(y))
            D.append(0.5 if depths is None else depths[k][q])
        T.append((3 * k, 3 * k + 1, 3 * k + 2))
    return np.array(X), np.array(Y), np.array(D, np.float32), np.array(T, np.uint32)


def _clampi(v, lo, hi):
    return max(lo, min(hi, v))


def _quad_count(x0, x1, y0, y1, W, H):
    """Pixel centres c with x0 <= c < x1 (left/top inclusive, right/bottom exclusive), clipped to the image."""
    nx = _clampi(ceil((x1 - 128) / 256), 0, W) - _clampi(ceil((x0 - 128) / 256), 0, W)
    ny = _clampi(ceil((y1 - 128) / 256), 0, H) - _clampi(ceil((y0 - 128) / 256), 0, H)
    return max(nx, 0) * max(ny, 0)


def test_axis_aligned_quad_pixel_count(orc):
    W, H = 24, 20
    rng = np.random.default_rng(5)
    for trial in range(400):
        if trial % 3 == 0:  # edges exactly on pixel centres
            x0, x1 = sorted(256 * rng.integers(-2, W + 2, 2) + 128)
            y0, y1 = sorted(256 * rng.integers(-2, H + 2, 2) + 128)
        else:
            x0, x1 = sorted(rng.integers(-600, 256 * W + 600, 2))
            y0, y1 = sorted(rng.integers(-600, 256 * H + 600, 2))
        if x0 == x1 or y0 == y1:
            continue
        p00, p10, p11, p01 = (x0, y0), (x1, y0), (x1, y1), (x0, y1)
        for tris in ([(p00, p10, p11), (p00, p11, p01)], [(p00, p10, p01), (p10, p11, p01)]):
            X, Y, D, T = _soup([_front(*t) for t in tris])
            ids, dep, cov = orc.raster(W, H, X, Y, D, T)
            assert cov.max() <= 1, "a pixel on the shared diagonal was covered twice"
            assert int(cov.sum()) == _quad_count(x0, x1, y0, y1, W, H)
            jj, ii = np.nonzero(cov)
            if len(ii):
                cxs, cys = 256 * ii + 128, 256 * jj + 128
                assert cxs.min() >= x0 and cxs.max() < x1 and cys.min() >= y0 and cys.max() < y1


def test_watertight_random_mesh(orc):
    """A jittered grid triangulation covers every interior pixel centre exactly once."""
    W, H = 32, 32
    rng = np.random.default_rng(9)
    for trial in range(20):
        n = int(rng.integers(3, 12))
        gx = np.linspace(-300, 256 * W + 300, n + 1)
        gy = np.linspace(-300, 256 * H + 300, n + 1)
        step = min(gx[1] - gx[0], gy[1] - gy[0])
        px = np.round(gx[None, :] + rng.uniform(-0.3, 0.3, (n + 1, n + 1)) * step).astype(np.int64)
        py = np.round(gy[:, None] + rng.uniform(-0.3, 0.3, (n + 1, n + 1)) * step).astype(np.int64)
        if trial % 2:  # snap many vertices onto pixel centres to force edges/vertices through them
            px = (px // 256) * 256 + 128
            py = (py // 256) * 256 + 128
        # keep the outer boundary outside the image so that every pixel is interior
        px[:, 0], px[:, -1], py[0, :], py[-1, :] = -300, 256 * W + 300, -300, 256 * H + 300
        tris = []
        for r in range(n):
            for c in range(n):
                p00, p10 = (px[r, c], py[r, c]), (px[r, c + 1], py[r, c + 1])
                p01, p11 = (px[r + 1, c], py[r + 1, c]), (px[r + 1, c + 1], py[r + 1, c + 1])
                if rng.random() < 0.5:
                    tris += [(p00, p10, p11), (p00, p11, p01)]
                else:
                    tris += [(p00, p10, p01), (p10, p11, p01)]
        kept = [_front(*t) for t in tris]
        X, Y, D, T = _soup(kept)
        ids, dep, cov = orc.raster(W, H, X, Y, D, T)
        assert cov.min() == 1 and cov.max() == 1


def _inside_exact(tri, px, py):
    """Strict rational point-in-triangle by solving P = a + u (b-a) + v (c-a); None when P is on an edge line."""
    (ax, ay), (bx, by), (cx, cy) = tri
    det = Fraction((bx - ax) * (cy - ay) - (by - ay) * (cx - ax))
    u = Fraction((px - ax) * (cy - ay) - (py - ay) * (cx - ax)) / det
    v = Fraction((bx - ax) * (py - ay) - (by - ay) * (px - ax)) / det
    w = 1 - u - v
    if u == 0 or v == 0 or w == 0:
        return None
    return u > 0 and v > 0 and w > 0


def test_coverage_matches_exact_rational_test(orc):
    W, H = 16, 12
    rng = np.random.default_rng(21)
    for _ in range(150):
        pts = [(int(rng.integers(-800, 256 * W + 800)), int(rng.integers(-800, 256 * H + 800))) for _ in range(3)]
        if (pts[1][0] - pts[0][0]) * (pts[2][1] - pts[0][1]) == (pts[1][1] - pts[0][1]) * (pts[2][0] - pts[0][0]):
            continue
        t = _front(*pts)
        X, Y, D, T = _soup([t])
        _, _, cov = orc.raster(W, H, X, Y, D, T)
        for j in range(H):
            for i in range(W):
                ins = _inside_exact(t, 256 * i + 128, 256 * j + 128)
                if ins is not None:
                    assert bool(cov[j, i]) == ins, (t, i, j)


def test_bbox_loop_equals_full_image_loop(orc):
    W, H = 20, 20
    rng = np.random.default_rng(33)
    tris = []
    for _ in range(300):
        c = rng.integers(-1000, 256 * W + 1000, 2)
        size = rng.choice([40, 200, 700, 4000])
        pts = [tuple(int(v) for v in c + rng.integers(-size, size + 1, 2)) for _ in range(3)]
        tris.append(_front(*pts))
    X, Y, D, T = _soup(tris, depths=[tuple(rng.uniform(0.1, 0.9, 3)) for _ in tris])
    a = orc.raster(W, H, X, Y, D, T, cull=0)
    b = orc.raster(W, H, X, Y, D, T, cull=2)
    for u, v in zip(a, b):
        assert np.array_equal(u, v)
    assert a[2].sum() > 0


def test_whole_pixel_translation_translates_coverage(orc):
    W, H = 40, 40
    rng = np.random.default_rng(41)
    tris = []
    for _ in range(60):
        c = rng.integers(256 * 10, 256 * 30, 2)
        pts = [tuple(int(v) for v in c + rng.integers(-900, 901, 2)) for _ in range(3)]
        tris.append(_front(*pts))
    X, Y, D, T = _soup(tris)
    _, _, cov0 = orc.raster(W, H, X, Y, D, T)
    for dx, dy in [(3, 0), (0, -4), (-5, 6)]:
        _, _, cov1 = orc.raster(W, H, X + 256 * dx, Y + 256 * dy, D, T)
        assert np.array_equal(np.roll(cov0, (dy, dx), axis=(0, 1)), cov1)
    _, _, cov2 = orc.raster(W, H, X + 100, Y, D, T)
    assert not np.array_equal(cov0, cov2)  # a sub-pixel shift is NOT a no-op: snapping matters


def test_cull_keeps_exactly_one_orientation(orc):
    t = _front((300, 300), (2500, 700), (900, 2600))
    X, Y, D, T = _soup([t, (t[0], t[2], t[1])])
    _, _, cov_f = orc.raster(16, 16, X, Y, D, T, cull=0)
    _, _, cov_b = orc.raster(16, 16, X, Y, D, T, cull=1)
    assert cov_f.max() == 1 and np.array_equal(cov_f, cov_b) and cov_f.sum() > 10
    ids, _, _ = orc.raster(16, 16, X, Y, D, T, cull=0)
    assert set(np.unique(ids)) == {0, BG}
    # degenerate (zero-area) triangles never cover anything
    X, Y, D, T = _soup([((128, 128), (1152, 1152), (2176, 2176))])
    assert orc.raster(16, 16, X, Y, D, T, cull=0)[2].sum() == 0
    assert orc.raster(16, 16, X, Y, D, T, cull=1)[2].sum() == 0


def test_rejected_vertex_drops_whole_triangle(orc):
    t = _front((300, 300), (2500, 700), (900, 2600))
    X, Y, D, T = _soup([t])
    for v in range(3):
        rej = np.zeros(3, np.uint8)
        rej[v] = 1
        ids, _, cov = orc.raster(16, 16, X, Y, D, T, rejected=rej)
        assert cov.sum() == 0 and np.all(ids == BG)


# ---------------------------------------------------------------- depth

def _quad(x0, x1, y0, y1, d00, d10, d11, d01):
    """Two front-facing triangles of an axis-aligned quad with per-corner depth (corner order 00,10,11,01)."""
    p = {"00": ((x0, y0), d00), "10": ((x1, y0), d10), "11": ((x1, y1), d11), "01": ((x0, y1), d01)}
    out_t, out_d = [], []
    for names in (("00", "10", "11"), ("00", "11", "01")):
        pts = [p[n][0] for n in names]
        dep = [p[n][1] for n in names]
        f = _front(*pts)
        out_t.append(f)
        out_d.append(tuple(dep[pts.index(q)] for q in f))
    return out_t, out_d


def test_nearer_parallel_quad_wins_everywhere(orc):
    W = H = 16
    ta, da = _quad(0, 4096, 0, 4096, 0.2, 0.2, 0.2, 0.2)
    tb, db = _quad(512, 3000, 700, 2500, 0.4, 0.4, 0.4, 0.4)
    X, Y, D, T = _soup(ta + tb, da + db)
    ids, dep, cov = orc.raster(W, H, X, Y, D, T)
    assert np.all((cov == 2) == np.isin(ids, [2, 3]))
    assert np.all(ids[cov == 1] < 2)
    assert np.all(dep[cov == 2] == np.float32(0.4).view(np.uint32))
    assert np.all(dep[cov == 0] == 0) and np.all(ids[cov == 0] == BG)
    # swap submission order and ids: same winners
    ids2, _, _ = orc.raster(W, H, X, Y, D, T, order=np.array([3, 2, 1, 0]))
    assert np.array_equal(ids, ids2)


def test_crossing_quads_switch_at_known_column(orc):
    """Quad A has depth rising left to right, quad B falling; they cross where the depths are equal."""
    W = H = 32
    x1 = 256 * W
    ta, da = _quad(0, x1, 0, x1, 0.1, 0.5, 0.5, 0.1)
    tb, db = _quad(0, x1, 0, x1, 0.4, 0.2, 0.2, 0.4)
    X, Y, D, T = _soup(ta + tb, da + db)
    ids, _, cov = orc.raster(W, H, X, Y, D, T)
    assert np.all(cov == 2)
    # 0.1 + 0.4 t = 0.4 - 0.2 t  =>  t = 0.5  => x = 16 px; centres at i + 0.5
    a_wins = ids < 2
    for j in range(H):
        cols = np.nonzero(a_wins[j])[0]
        assert len(cols) and cols.max() == W - 1 and np.all(np.diff(cols) == 1)
        assert abs(cols.min() - 16) <= 1
        assert not a_wins[j, :15].any()


def test_coincident_duplicates_resolve_to_lowest_id(orc):
    W = H = 16
    t = _front((100, 100), (3900, 500), (1800, 3800))
    d = (0.3, 0.6, 0.45)
    X, Y, D, T = _soup([t, t, t], [d, d, d])
    rng = np.random.default_rng(2)
    for _ in range(6):
        ids, _, cov = orc.raster(W, H, X, Y, D, T, order=rng.permutation(3))
        assert np.all(ids[cov > 0] == 0) and np.all(cov[cov > 0] == 3)


def test_permutation_invariance(orc):
    W = H = 24
    rng = np.random.default_rng(77)
    tris, deps = [], []
    for k in range(250):
        c = rng.integers(0, 256 * W, 2)
        size = rng.choice([60, 300, 1500])
        pts = [tuple(int(v) for v in c + rng.integers(-size, size + 1, 2)) for _ in range(3)]
        tris.append(_front(*pts))
        # few distinct depth levels => many exact ties between different triangles
        deps.append(tuple(np.float32(rng.choice([0.25, 0.5, 0.75])) for _ in range(3)) if k % 2 else
                    tuple(rng.uniform(0.1, 0.9, 3)))
    X, Y, D, T = _soup(tris, deps)
    ref = orc.raster(W, H, X, Y, D, T)
    assert (ref[2] > 1).sum() > 50
    for _ in range(100):
        out = orc.raster(W, H, X, Y, D, T, order=rng.permutation(len(tris)))
        assert np.array_equal(out[0], ref[0]) and np.array_equal(out[1], ref[1])


def test_depth_is_affine_interpolation(orc):
    """Reversed depth is affine in screen space: compare with exact rational interpolation."""
    W = H = 16
    rng = np.random.default_rng(13)
    for _ in range(40):
        pts = [(int(rng.integers(-500, 256 * W + 500)), int(rng.integers(-500, 256 * H + 500))) for _ in range(3)]
        if (pts[1][0] - pts[0][0]) * (pts[2][1] - pts[0][1]) == (pts[1][1] - pts[0][1]) * (pts[2][0] - pts[0][0]):
            continue
        d = [float(np.float32(v)) for v in rng.uniform(0.02, 0.9, 3)]
        order = _front(*pts)
        dd = [d[pts.index(p)] for p in order]
        X, Y, D, T = _soup([order], [tuple(dd)])
        ids, dep, cov = orc.raster(W, H, X, Y, D, T)
        (ax, ay), (bx, by), (cx, cy) = order
        det = Fraction((bx - ax) * (cy - ay) - (by - ay) * (cx - ax))
        for j, i in zip(*np.nonzero(cov)):
            px, py = 256 * int(i) + 128, 256 * int(j) + 128
            u = Fraction((px - ax) * (cy - ay) - (py - ay) * (cx - ax)) / det
            v = Fraction((bx - ax) * (py - ay) - (by - ay) * (px - ax)) / det
            exact = float(Fraction(dd[0]) + u * (Fraction(dd[1]) - Fraction(dd[0])) + v * (Fraction(dd[2]) - Fraction(dd[0])))
            got = float(dep[j, i:i + 1].view(np.float32)[0])
            assert got == pytest.approx(exact, rel=0, abs=4e-7)
