// orc.cpp — the CPU oracle (test infrastructure; see orc.h for what pins it).
//
// One frame = one (environment, step).  The paper (PixelBrax sections 1-2)
// states the job: body poses in, a small RGB observation out, optionally with
// a colour or a video distractor, reproducible from a seed.  Every convention
// below it (meshes, camera, fixed-point snap, fill rule, depth, shading) is
// this build's reading, stated once here in the order it is applied:
//
//   M  meshes      capsule / sphere / box templates on the unit shape
//   C  camera      fixed world-space offset from the root body, pinhole
//   V  vertices    pose -> view space -> perspective divide -> 8-bit snap
//   R  raster      int64 edge functions, top-left rule, reversed float depth,
//                  ties broken by the lower triangle id
//   G  ground      z=0 plane by per-pixel ray, 1 m checkerboard; background
//   S  shade       flat Lambert + ambient
//   X  distractor  colour jitter or video blend, then uint8 quantisation
//   F  kinematics  (optional producer stage) hinge angles -> body poses
//
// Build: g++ -O2 -ffp-contract=off -fno-fast-math.  `float` is IEEE binary32
// and every fp32 operation is rounded on its own unless written as fmaf().

#include "orc.h"

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>
#include <vector>

namespace {

const double kPi = 3.14159265358979323846;

struct Body {
    uint32_t kind;
    float shape[4];
    float rgb[3];
    uint32_t n_lon, n_lat;
    uint32_t vert_base, tri_base, n_verts, n_tris;
};

}  // namespace

struct orc_scene {
    uint32_t W, H, K, root;
    std::vector<Body> bodies;
    // template mesh (M)
    std::vector<float> uv;        // V*4: ux,uy,uz,s
    std::vector<uint32_t> tri;    // T*3 global vertex ids
    std::vector<float> nrm;       // T*3
    std::vector<float> mul;       // T
    std::vector<uint32_t> tbody;  // T
    std::vector<uint32_t> vbody;  // V
    // camera (C)
    float Rt[3], Up[3], Fw[3];
    float off[3];
    float f, halfW, halfH;
    std::vector<float> cx, cy;
    float z_near, z_far;
    // light / ground / background
    float l[3], ambient, diffuse;
    uint32_t ground_on;
    float cell, gs[2];
    float bg[3];
};

namespace {

inline float dot3(const float* a, float bx, float by, float bz) {
    return std::fmaf(a[0], bx, std::fmaf(a[1], by, a[2] * bz));
}

// ---------------------------------------------------------------- M: meshes
//
// Unit-shape vertices u = (ux,uy,uz) with a cap selector s in {+1,0,-1};
// the posed local position is (a*ux, b*uy, c*uz + s*h) for shape (a,b,c,h).
// Trigonometry in double, one rounding to fp32 at the end.

struct MeshOut {
    std::vector<float>& uv;
    std::vector<uint32_t>& tri;
    std::vector<float>& nrm;
    std::vector<float>& mul;
};

struct D3 { double x, y, z; };

D3 unit_normal(const D3& p0, const D3& p1, const D3& p2) {
    D3 e1{p1.x - p0.x, p1.y - p0.y, p1.z - p0.z};
    D3 e2{p2.x - p0.x, p2.y - p0.y, p2.z - p0.z};
    D3 n{e1.y * e2.z - e1.z * e2.y, e1.z * e2.x - e1.x * e2.z, e1.x * e2.y - e1.y * e2.x};
    double len = std::sqrt(n.x * n.x + n.y * n.y + n.z * n.z);
    return D3{n.x / len, n.y / len, n.z / len};
}

// A latitude ring of the unit sphere at polar angle theta (from +z).
// `exact_equator` forces sin=1, cos=0 so that equator rings have uz == 0.
void ring(std::vector<D3>& pts, uint32_t L, double theta, bool exact_equator) {
    double st = exact_equator ? 1.0 : std::sin(theta);
    double ct = exact_equator ? 0.0 : std::cos(theta);
    for (uint32_t j = 0; j < L; ++j) {
        double phi = ((2.0 * kPi) * (double)j) / (double)L;
        pts.push_back(D3{st * std::cos(phi), st * std::sin(phi), ct});
    }
}

// Capsule (with_band) or sphere (no band, single equator) with L longitudes
// and M latitude steps per hemisphere.  Vertex and triangle order:
//   pole(+z), rings from the top down, pole(-z);
//   top fan, then for each consecutive ring pair the quads (a,d,c),(a,c,b)
//   with a=U[j], b=U[j+1], c=Lw[j+1], d=Lw[j], then the bottom fan.
void build_round(MeshOut out, uint32_t base, uint32_t L, uint32_t M, bool with_band) {
    std::vector<D3> p;       // double positions on the unit sphere
    std::vector<float> sel;  // cap selector
    std::vector<int> ring_is_band_top;  // for each ring pair: 1 if it is the cylinder band
    p.push_back(D3{0.0, 0.0, 1.0});
    sel.push_back(with_band ? 1.0f : 0.0f);
    uint32_t n_rings;
    if (with_band) {
        for (uint32_t k = 1; k <= M; ++k) {
            ring(p, L, ((double)k * (kPi / 2.0)) / (double)M, k == M);
            for (uint32_t j = 0; j < L; ++j) sel.push_back(1.0f);
        }
        for (uint32_t m = 0; m < M; ++m) {
            ring(p, L, kPi / 2.0 + ((double)m * (kPi / 2.0)) / (double)M, m == 0);
            for (uint32_t j = 0; j < L; ++j) sel.push_back(-1.0f);
        }
        n_rings = 2 * M;
    } else {
        for (uint32_t k = 1; k <= 2 * M - 1; ++k) {
            ring(p, L, ((double)k * kPi) / (double)(2 * M), k == M);
            for (uint32_t j = 0; j < L; ++j) sel.push_back(0.0f);
        }
        n_rings = 2 * M - 1;
    }
    p.push_back(D3{0.0, 0.0, -1.0});
    sel.push_back(with_band ? -1.0f : 0.0f);

    for (size_t i = 0; i < p.size(); ++i) {
        out.uv.push_back((float)p[i].x);
        out.uv.push_back((float)p[i].y);
        out.uv.push_back((float)p[i].z);
        out.uv.push_back(sel[i]);
    }
    const uint32_t last = (uint32_t)p.size() - 1;
    auto rv = [&](uint32_t r, uint32_t j) { return 1 + r * L + (j % L); };  // ring r (0-based), longitude j
    auto emit = [&](uint32_t i0, uint32_t i1, uint32_t i2, const D3& n) {
        out.tri.push_back(base + i0);
        out.tri.push_back(base + i1);
        out.tri.push_back(base + i2);
        out.nrm.push_back((float)n.x);
        out.nrm.push_back((float)n.y);
        out.nrm.push_back((float)n.z);
        out.mul.push_back(1.0f);
    };
    for (uint32_t j = 0; j < L; ++j) {
        uint32_t i1 = rv(0, j), i2 = rv(0, j + 1);
        emit(0, i1, i2, unit_normal(p[0], p[i1], p[i2]));
    }
    for (uint32_t r = 0; r + 1 < n_rings; ++r) {
        bool band = with_band && (r == M - 1);  // top equator -> bottom equator
        for (uint32_t j = 0; j < L; ++j) {
            uint32_t a = rv(r, j), b = rv(r, j + 1), c = rv(r + 1, j + 1), d = rv(r + 1, j);
            if (band) {
                // both rings coincide on the unit sphere; the face normal is the
                // horizontal direction at the quad's mid-longitude
                double phi = ((2.0 * kPi) * ((double)j + 0.5)) / (double)L;
                D3 n{std::cos(phi), std::sin(phi), 0.0};
                emit(a, d, c, n);
                emit(a, c, b, n);
            } else {
                emit(a, d, c, unit_normal(p[a], p[d], p[c]));
                emit(a, c, b, unit_normal(p[a], p[c], p[b]));
            }
        }
    }
    for (uint32_t j = 0; j < L; ++j) {
        uint32_t i0 = rv(n_rings - 1, j), i2 = rv(n_rings - 1, j + 1);
        emit(i0, last, i2, unit_normal(p[i0], p[last], p[i2]));
    }
}

// Box with n x n cells per face; faces +x,-x,+y,-y,+z,-z; per face its own
// (n+1)^2 vertices; (u axis, v axis) chosen so that u x v is the outward normal;
// cell (cu,cv) -> (p00,p10,p11),(p00,p11,p01); checker multiplier 1 / 0.5.
void build_box(MeshOut out, uint32_t base, uint32_t n) {
    static const int axes[6][3] = {
        // normal axis (signed: +1..+3 / -1..-3 => x,y,z), u axis, v axis (0=x,1=y,2=z)
        {+1, 1, 2}, {-1, 2, 1}, {+2, 2, 0}, {-2, 0, 2}, {+3, 0, 1}, {-3, 1, 0}};
    for (int fidx = 0; fidx < 6; ++fidx) {
        int na = std::abs(axes[fidx][0]) - 1;
        double ns = axes[fidx][0] > 0 ? 1.0 : -1.0;
        int ua = axes[fidx][1], va = axes[fidx][2];
        uint32_t fbase = (uint32_t)fidx * (n + 1) * (n + 1);
        for (uint32_t iv = 0; iv <= n; ++iv)
            for (uint32_t iu = 0; iu <= n; ++iu) {
                double c[3];
                c[na] = ns;
                c[ua] = -1.0 + (2.0 * (double)iu) / (double)n;
                c[va] = -1.0 + (2.0 * (double)iv) / (double)n;
                out.uv.push_back((float)c[0]);
                out.uv.push_back((float)c[1]);
                out.uv.push_back((float)c[2]);
                out.uv.push_back(0.0f);
            }
        float nf[3] = {0.0f, 0.0f, 0.0f};
        nf[na] = (float)ns;
        for (uint32_t cv = 0; cv < n; ++cv)
            for (uint32_t cu = 0; cu < n; ++cu) {
                uint32_t p00 = fbase + cv * (n + 1) + cu, p10 = p00 + 1;
                uint32_t p01 = p00 + (n + 1), p11 = p01 + 1;
                float m = ((cu + cv) & 1u) ? 0.5f : 1.0f;
                const uint32_t t[2][3] = {{p00, p10, p11}, {p00, p11, p01}};
                for (int k = 0; k < 2; ++k) {
                    for (int q = 0; q < 3; ++q) out.tri.push_back(base + t[k][q]);
                    for (int q = 0; q < 3; ++q) out.nrm.push_back(nf[q]);
                    out.mul.push_back(m);
                }
            }
    }
}

// Arbitrary triangle mesh given by the caller: vertices are taken as they are (fp32, selector 0, scaled
// per axis by the body's shape like any other template), triangles keep their order, the normal of a
// triangle is the unit cross product (v1-v0) x (v2-v0) of its unscaled vertices in double (zero for a
// triangle without area), the colour multiplier is the caller's (1 if none).  Returns false on an index
// out of range.
bool build_mesh(MeshOut out, uint32_t base, uint32_t nv, const float* verts, uint32_t nt, const uint32_t* tris,
                const float* mul) {
    for (uint32_t v = 0; v < nv; ++v) {
        for (int c = 0; c < 3; ++c) out.uv.push_back(verts[(size_t)v * 3 + c]);
        out.uv.push_back(0.0f);
    }
    for (uint32_t t = 0; t < nt; ++t) {
        const uint32_t* ix = tris + (size_t)t * 3;
        if (ix[0] >= nv || ix[1] >= nv || ix[2] >= nv) return false;
        if (mul && !(mul[t] >= 0.0f)) return false;  // a colour multiplier cannot be negative
        D3 p[3];
        for (int q = 0; q < 3; ++q) p[q] = D3{verts[(size_t)ix[q] * 3], verts[(size_t)ix[q] * 3 + 1], verts[(size_t)ix[q] * 3 + 2]};
        D3 n = unit_normal(p[0], p[1], p[2]);
        if (!(std::isfinite(n.x) && std::isfinite(n.y) && std::isfinite(n.z))) n = D3{0.0, 0.0, 0.0};
        for (int q = 0; q < 3; ++q) out.tri.push_back(base + ix[q]);
        out.nrm.push_back((float)n.x);
        out.nrm.push_back((float)n.y);
        out.nrm.push_back((float)n.z);
        out.mul.push_back(mul ? mul[t] : 1.0f);
    }
    return true;
}

// ---------------------------------------------------------------- V: vertices

struct FrameXform {
    float eye[3];
    std::vector<float> M;   // K*9, row-major: view <- body rotation
    std::vector<float> t;   // K*3: body origin in view space
    std::vector<float> lb;  // K*3: light direction in the body frame
};

void body_transforms(const orc_scene* s, const float* poses, FrameXform& fx) {
    const uint32_t K = s->K;
    fx.M.resize(K * 9);
    fx.t.resize(K * 3);
    fx.lb.resize(K * 3);
    const float* pr = poses + (size_t)s->root * 7;
    for (int c = 0; c < 3; ++c) fx.eye[c] = pr[c] + s->off[c];
    const float* Rv[3] = {s->Rt, s->Up, s->Fw};
    for (uint32_t b = 0; b < K; ++b) {
        const float* p = poses + (size_t)b * 7;
        float w = p[3], x = p[4], y = p[5], z = p[6];
        float R[3][3];
        R[0][0] = 1.0f - 2.0f * (y * y + z * z);
        R[0][1] = 2.0f * (x * y - w * z);
        R[0][2] = 2.0f * (x * z + w * y);
        R[1][0] = 2.0f * (x * y + w * z);
        R[1][1] = 1.0f - 2.0f * (x * x + z * z);
        R[1][2] = 2.0f * (y * z - w * x);
        R[2][0] = 2.0f * (x * z - w * y);
        R[2][1] = 2.0f * (y * z + w * x);
        R[2][2] = 1.0f - 2.0f * (x * x + y * y);
        float d[3] = {p[0] - fx.eye[0], p[1] - fx.eye[1], p[2] - fx.eye[2]};
        for (int r = 0; r < 3; ++r) {
            for (int c = 0; c < 3; ++c) fx.M[b * 9 + r * 3 + c] = dot3(Rv[r], R[0][c], R[1][c], R[2][c]);
            fx.t[b * 3 + r] = dot3(Rv[r], d[0], d[1], d[2]);
        }
        for (int c = 0; c < 3; ++c) fx.lb[b * 3 + c] = dot3(s->l, R[0][c], R[1][c], R[2][c]);
    }
}

// rej[v]: 0 = projected and snapped; 2 = behind the near plane (pv.z < z_near): its triangles are clipped;
// 1 = unusable (outside the guard band, or a non-finite depth): its triangles are dropped.
// PV (optional) receives the view-space position of every vertex.
void vertex_stage(const orc_scene* s, const float* poses, const float* shapes, FrameXform& fx,
                  int32_t* X, int32_t* Y, float* D, uint8_t* rej, float* PV = nullptr) {
    body_transforms(s, poses, fx);
    const uint32_t V = (uint32_t)s->vbody.size();
    for (uint32_t v = 0; v < V; ++v) {
        uint32_t b = s->vbody[v];
        const float* sh = shapes ? shapes + (size_t)b * 4 : s->bodies[b].shape;
        const float* u = &s->uv[(size_t)v * 4];
        float lx = sh[0] * u[0];
        float ly = sh[1] * u[1];
        float lz = std::fmaf(sh[2], u[2], u[3] * sh[3]);
        const float* M = &fx.M[b * 9];
        const float* t = &fx.t[b * 3];
        float pv[3];
        for (int r = 0; r < 3; ++r)
            pv[r] = std::fmaf(M[r * 3 + 0], lx, std::fmaf(M[r * 3 + 1], ly, std::fmaf(M[r * 3 + 2], lz, t[r])));
        float inv = 1.0f / pv[2];
        float sx = std::fmaf(s->f, pv[0] * inv, s->halfW);
        float sy = std::fmaf(-s->f, pv[1] * inv, s->halfH);
        bool ok = (pv[2] >= s->z_near) && (std::fabs(sx) <= 16384.0f) && (std::fabs(sy) <= 16384.0f);
        if (PV) for (int r = 0; r < 3; ++r) PV[(size_t)v * 3 + r] = pv[r];
        if (ok) {
            X[v] = (int32_t)std::floor(std::fmaf(sx, 256.0f, 0.5f));
            Y[v] = (int32_t)std::floor(std::fmaf(sy, 256.0f, 0.5f));
            D[v] = s->z_near * inv;
            rej[v] = 0;
        } else {
            X[v] = 0;
            Y[v] = 0;
            D[v] = 0.0f;
            rej[v] = (pv[2] < s->z_near) ? 2 : 1;
        }
    }
}

// ---------------------------------------------------------------- R: raster

inline int64_t orient(int64_t px, int64_t py, int64_t qx, int64_t qy, int64_t rx, int64_t ry) {
    return (qx - px) * (ry - py) - (qy - py) * (rx - px);
}
inline bool top_left(int64_t px, int64_t py, int64_t qx, int64_t qy) {
    int64_t dx = qx - px, dy = qy - py;
    return dy < 0 || (dy == 0 && dx > 0);
}
// float -> int32 for a value that may lie outside the int32 range.  C++ leaves that conversion undefined and the
// paper says nothing of such inputs (a camera 3e9 m from the origin); defined here as saturating, NaN -> 0.
inline int32_t to_int_saturating(float x) {
    if (x != x) return 0;
    if (x >= 2147483648.0f) return INT32_MAX;
    if (x <= -2147483648.0f) return INT32_MIN;
    return (int32_t)x;
}

inline int64_t floor_div(int64_t a, int64_t b) {  // b > 0
    int64_t q = a / b, r = a % b;
    return (r < 0) ? q - 1 : q;
}
inline int64_t ceil_div(int64_t a, int64_t b) { return -floor_div(-a, b); }
inline uint32_t fbits(float x) {
    uint32_t u;
    std::memcpy(&u, &x, 4);
    return u;
}

struct ZBuf {
    std::vector<float> depth;
    std::vector<uint32_t> id;
    void reset(size_t n) {
        depth.assign(n, 0.0f);
        id.assign(n, ORC_ID_BG);
    }
    // z-test: nearer (larger reversed depth) wins; equal depth -> lower id.
    inline void test(size_t pix, float d, uint32_t g) {
        if (d > depth[pix] || (d == depth[pix] && g < id[pix])) {
            depth[pix] = d;
            id[pix] = g;
        }
    }
};

void raster_triangle(uint32_t W, uint32_t H, const int32_t* X, const int32_t* Y, const float* D,
                     const uint8_t* rej, const uint32_t* tri, uint32_t g, uint32_t cull, ZBuf* zb,
                     uint32_t* cover) {
    uint32_t v0 = tri[0], v1 = tri[1], v2 = tri[2];
    if (rej[v0] || rej[v1] || rej[v2]) return;  // an unusable corner (or, for a bare soup, one behind the near plane)
    // screen order: swapping two vertices turns world-CCW front faces into
    // positive orientation in the y-down raster frame
    uint32_t ia = v0, ib = v2, ic = v1;
    if (cull == 1) { ib = v1; ic = v2; }  // keep back faces instead
    int64_t ax = X[ia], ay = Y[ia], bx = X[ib], by = Y[ib], cx = X[ic], cy = Y[ic];
    int64_t A2 = orient(ax, ay, bx, by, cx, cy);
    if (A2 <= 0) return;
    int64_t i0, i1, j0, j1;
    if (cull == 2) {
        i0 = 0; i1 = (int64_t)W - 1; j0 = 0; j1 = (int64_t)H - 1;
    } else {
        int64_t minx = std::min(ax, std::min(bx, cx)), maxx = std::max(ax, std::max(bx, cx));
        int64_t miny = std::min(ay, std::min(by, cy)), maxy = std::max(ay, std::max(by, cy));
        i0 = std::max<int64_t>(0, ceil_div(minx - 128, 256));
        i1 = std::min<int64_t>((int64_t)W - 1, floor_div(maxx - 128, 256));
        j0 = std::max<int64_t>(0, ceil_div(miny - 128, 256));
        j1 = std::min<int64_t>((int64_t)H - 1, floor_div(maxy - 128, 256));
    }
    bool tl_ab = top_left(ax, ay, bx, by), tl_bc = top_left(bx, by, cx, cy), tl_ca = top_left(cx, cy, ax, ay);
    float invA = 1.0f / (float)A2;
    float Da = D[ia], dDb = D[ib] - D[ia], dDc = D[ic] - D[ia];
    for (int64_t j = j0; j <= j1; ++j)
        for (int64_t i = i0; i <= i1; ++i) {
            int64_t px = 256 * i + 128, py = 256 * j + 128;
            int64_t e_ab = orient(ax, ay, bx, by, px, py);
            int64_t e_bc = orient(bx, by, cx, cy, px, py);
            int64_t e_ca = orient(cx, cy, ax, ay, px, py);
            bool in = (e_ab > 0 || (e_ab == 0 && tl_ab)) && (e_bc > 0 || (e_bc == 0 && tl_bc)) &&
                      (e_ca > 0 || (e_ca == 0 && tl_ca));
            if (!in) continue;
            size_t pix = (size_t)j * W + (size_t)i;
            if (cover) cover[pix] += 1;
            if (zb) {
                float beta = (float)e_ca * invA;   // weight of b
                float gamma = (float)e_ab * invA;  // weight of c
                float dp = std::fmaf(beta, dDb, std::fmaf(gamma, dDc, Da));
                zb->test(pix, dp, g);
            }
        }
}

// Near-plane clipping of one triangle whose vertices are partly behind z_near (view space).
// Walk the edges v0->v1, v1->v2, v2->v0 (Sutherland-Hodgman against the single plane z = z_near): a
// vertex in front is kept; an edge that crosses the plane adds its intersection, always computed from
// the endpoint in front (P) towards the one behind (Q), so two triangles sharing the edge get the same
// point:  t = (z_near - P.z) / (Q.z - P.z),  I = (fma(t, Q.x - P.x, P.x), fma(t, Q.y - P.y, P.y), z_near).
// The 3 or 4 resulting corners w0.. keep the winding; they are projected and snapped exactly like
// template vertices (a corner outside the guard band is unusable) and rastered as (w0,w1,w2) and
// (w0,w2,w3) under the parent's id by the ordinary rule.
void clip_and_raster(const orc_scene* s, const float* PV, const int32_t* X, const int32_t* Y, const float* D,
                     const uint8_t* rej, const uint32_t* tri, uint32_t g, ZBuf* zb) {
    float wx[4], wy[4], wz[4];
    int from_vertex[4];  // index 0..2 of the original corner, or -1 for an intersection
    int n = 0;
    for (int e = 0; e < 3; ++e) {
        const uint32_t vs = tri[e], ve = tri[(e + 1) % 3];
        const bool s_in = rej[vs] != 2, e_in = rej[ve] != 2;
        if (s_in) {
            from_vertex[n] = e;
            wx[n] = wy[n] = wz[n] = 0.0f;
            ++n;
        }
        if (s_in != e_in) {
            const float* P = PV + (size_t)(s_in ? vs : ve) * 3;
            const float* Q = PV + (size_t)(s_in ? ve : vs) * 3;
            const float t = (s->z_near - P[2]) / (Q[2] - P[2]);
            from_vertex[n] = -1;
            wx[n] = std::fmaf(t, Q[0] - P[0], P[0]);
            wy[n] = std::fmaf(t, Q[1] - P[1], P[1]);
            wz[n] = s->z_near;
            ++n;
        }
    }
    if (n < 3) return;  // nothing in front
    int32_t cX[4], cY[4];
    float cD[4];
    uint8_t cr[4];
    for (int k = 0; k < n; ++k) {
        if (from_vertex[k] >= 0) {
            const uint32_t v = tri[from_vertex[k]];
            cX[k] = X[v]; cY[k] = Y[v]; cD[k] = D[v]; cr[k] = rej[v];
            continue;
        }
        const float inv = 1.0f / wz[k];
        const float sx = std::fmaf(s->f, wx[k] * inv, s->halfW);
        const float sy = std::fmaf(-s->f, wy[k] * inv, s->halfH);
        const bool ok = (std::fabs(sx) <= 16384.0f) && (std::fabs(sy) <= 16384.0f);
        cr[k] = ok ? 0 : 1;
        cX[k] = ok ? (int32_t)std::floor(std::fmaf(sx, 256.0f, 0.5f)) : 0;
        cY[k] = ok ? (int32_t)std::floor(std::fmaf(sy, 256.0f, 0.5f)) : 0;
        cD[k] = s->z_near * inv;
    }
    const uint32_t first[3] = {0, 1, 2}, second[3] = {0, 2, 3};
    raster_triangle(s->W, s->H, cX, cY, cD, cr, first, g, 0, zb, nullptr);
    if (n == 4) raster_triangle(s->W, s->H, cX, cY, cD, cr, second, g, 0, zb, nullptr);
}

// ---------------------------------------------------------------- X: generator

inline void mulhilo(uint32_t a, uint32_t b, uint32_t& hi, uint32_t& lo) {
    uint64_t p = (uint64_t)a * (uint64_t)b;
    hi = (uint32_t)(p >> 32);
    lo = (uint32_t)p;
}

void philox(uint64_t seed, uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t out[4]) {
    uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
    for (int round = 0; round < 10; ++round) {
        if (round > 0) {
            k0 += 0x9E3779B9u;
            k1 += 0xBB67AE85u;
        }
        uint32_t hi0, lo0, hi1, lo1;
        mulhilo(0xD2511F53u, c0, hi0, lo0);
        mulhilo(0xCD9E8D57u, c2, hi1, lo1);
        uint32_t n0 = hi1 ^ c1 ^ k0, n1 = lo1, n2 = hi0 ^ c3 ^ k1, n3 = lo0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

inline float u01(uint32_t x) { return (float)(x >> 8) * 5.9604644775390625e-08f; }  // 2^-24

}  // namespace

// ================================================================ C interface

extern "C" {

orc_scene* orc_scene_create(uint32_t width, uint32_t height, uint32_t n_bodies, uint32_t root_body,
                            const uint32_t* kinds, const float* shapes, const float* rgbs,
                            const uint32_t* n_lon, const uint32_t* n_lat, const float* cam,
                            const float* light, const float* ground, const float* bg) {
    return orc_scene_create_meshes(width, height, n_bodies, root_body, kinds, shapes, rgbs, n_lon, n_lat, cam, light,
                                   ground, bg, nullptr, nullptr, nullptr, nullptr, nullptr);
}

orc_scene* orc_scene_create_meshes(uint32_t width, uint32_t height, uint32_t n_bodies, uint32_t root_body,
                                   const uint32_t* kinds, const float* shapes, const float* rgbs,
                                   const uint32_t* n_lon, const uint32_t* n_lat, const float* cam,
                                   const float* light, const float* ground, const float* bg,
                                   const uint32_t* mesh_nv, const uint32_t* mesh_nt, const float* mesh_verts,
                                   const uint32_t* mesh_tris, const float* mesh_mul) {
    size_t mesh_v0 = 0, mesh_t0 = 0;  // running offsets into the concatenated mesh arrays
    if (!kinds || !shapes || !rgbs || !n_lon || !n_lat || !cam || !light || !ground || !bg) return nullptr;
    if (width < 1 || height < 1 || n_bodies < 1 || root_body >= n_bodies) return nullptr;
    // colours are fractions of full intensity: base colours outside [0,1] are invalid input
    auto unit = [](float v) { return v >= 0.0f && v <= 1.0f; };
    for (uint32_t i = 0; i < n_bodies * 3; ++i)
        if (!unit(rgbs[i])) return nullptr;
    if (!unit(ground[2]) || !unit(ground[3]) || !unit(bg[0]) || !unit(bg[1]) || !unit(bg[2])) return nullptr;
    orc_scene* s = new orc_scene();
    s->W = width; s->H = height; s->K = n_bodies; s->root = root_body;
    MeshOut out{s->uv, s->tri, s->nrm, s->mul};
    for (uint32_t b = 0; b < n_bodies; ++b) {
        Body bd;
        bd.kind = kinds[b];
        for (int i = 0; i < 4; ++i) bd.shape[i] = shapes[b * 4 + i];
        for (int i = 0; i < 3; ++i) bd.rgb[i] = rgbs[b * 3 + i];
        bd.n_lon = n_lon[b]; bd.n_lat = n_lat[b];
        bd.vert_base = (uint32_t)(s->uv.size() / 4);
        bd.tri_base = (uint32_t)(s->tri.size() / 3);
        bool ok = true;
        if (bd.kind == ORC_CAPSULE && bd.n_lon >= 3 && bd.n_lat >= 1) build_round(out, bd.vert_base, bd.n_lon, bd.n_lat, true);
        else if (bd.kind == ORC_SPHERE && bd.n_lon >= 3 && bd.n_lat >= 1) build_round(out, bd.vert_base, bd.n_lon, bd.n_lat, false);
        else if (bd.kind == ORC_BOX && bd.n_lon >= 1) build_box(out, bd.vert_base, bd.n_lon);
        else if (bd.kind == ORC_MESH && mesh_nv && mesh_nt && mesh_verts && mesh_tris && mesh_nv[b] >= 1 && mesh_nt[b] >= 1) {
            ok = build_mesh(out, bd.vert_base, mesh_nv[b], mesh_verts + mesh_v0 * 3, mesh_nt[b], mesh_tris + mesh_t0 * 3,
                            mesh_mul ? mesh_mul + mesh_t0 : nullptr);
            mesh_v0 += mesh_nv[b];
            mesh_t0 += mesh_nt[b];
        }
        else ok = false;
        if (!ok) { delete s; return nullptr; }
        bd.n_verts = (uint32_t)(s->uv.size() / 4) - bd.vert_base;
        bd.n_tris = (uint32_t)(s->tri.size() / 3) - bd.tri_base;
        for (uint32_t i = 0; i < bd.n_verts; ++i) s->vbody.push_back(b);
        for (uint32_t i = 0; i < bd.n_tris; ++i) s->tbody.push_back(b);
        s->bodies.push_back(bd);
    }
    // C: camera.  Forward = -offset/|offset| (the camera looks at the root),
    // right = normalize(forward x up), up' = right x forward; double -> fp32.
    double fov = (double)cam[0];
    double off[3] = {cam[1], cam[2], cam[3]}, up[3] = {cam[4], cam[5], cam[6]};
    double on = std::sqrt(off[0] * off[0] + off[1] * off[1] + off[2] * off[2]);
    double Fw[3] = {-off[0] / on, -off[1] / on, -off[2] / on};
    double Rt[3] = {Fw[1] * up[2] - Fw[2] * up[1], Fw[2] * up[0] - Fw[0] * up[2], Fw[0] * up[1] - Fw[1] * up[0]};
    double rn = std::sqrt(Rt[0] * Rt[0] + Rt[1] * Rt[1] + Rt[2] * Rt[2]);
    if (!(on > 0.0) || !(rn > 0.0)) { delete s; return nullptr; }
    for (int i = 0; i < 3; ++i) Rt[i] /= rn;
    double Up[3] = {Rt[1] * Fw[2] - Rt[2] * Fw[1], Rt[2] * Fw[0] - Rt[0] * Fw[2], Rt[0] * Fw[1] - Rt[1] * Fw[0]};
    for (int i = 0; i < 3; ++i) {
        s->Rt[i] = (float)Rt[i]; s->Up[i] = (float)Up[i]; s->Fw[i] = (float)Fw[i];
        s->off[i] = cam[1 + i];
    }
    double fd = ((double)height / 2.0) / std::tan((fov * kPi / 180.0) / 2.0);
    s->f = (float)fd;
    s->halfW = (float)((double)width / 2.0);
    s->halfH = (float)((double)height / 2.0);
    s->cx.resize(width);
    s->cy.resize(height);
    for (uint32_t i = 0; i < width; ++i) s->cx[i] = (float)((((double)i + 0.5) - (double)width / 2.0) / fd);
    for (uint32_t j = 0; j < height; ++j) s->cy[j] = (float)(-(((double)j + 0.5) - (double)height / 2.0) / fd);
    s->z_near = cam[7];
    s->z_far = cam[8];
    double ld[3] = {light[0], light[1], light[2]};
    double ln = std::sqrt(ld[0] * ld[0] + ld[1] * ld[1] + ld[2] * ld[2]);
    if (!(ln > 0.0)) { delete s; return nullptr; }
    for (int i = 0; i < 3; ++i) s->l[i] = (float)(ld[i] / ln);
    s->ambient = light[3];
    s->diffuse = light[4];
    s->ground_on = ground[0] != 0.0f;
    s->cell = ground[1];
    double lz = ld[2] / ln;
    double lit = (double)light[3] + (double)light[4] * (lz > 0.0 ? lz : 0.0);
    // (like a shaded triangle, the lit ground never exceeds full intensity)
    s->gs[0] = std::min(1.0f, (float)((double)ground[2] * lit));
    s->gs[1] = std::min(1.0f, (float)((double)ground[3] * lit));
    for (int i = 0; i < 3; ++i) s->bg[i] = bg[i];
    return s;
}

void orc_scene_destroy(orc_scene* s) { delete s; }

void orc_scene_counts(const orc_scene* s, uint32_t* n_verts, uint32_t* n_tris) {
    if (n_verts) *n_verts = (uint32_t)s->vbody.size();
    if (n_tris) *n_tris = (uint32_t)s->tbody.size();
}

void orc_scene_mesh(const orc_scene* s, float* uverts, uint32_t* tris, float* normals, float* mul,
                    uint32_t* tri_body, uint32_t* vert_body) {
    if (uverts) std::memcpy(uverts, s->uv.data(), s->uv.size() * 4);
    if (tris) std::memcpy(tris, s->tri.data(), s->tri.size() * 4);
    if (normals) std::memcpy(normals, s->nrm.data(), s->nrm.size() * 4);
    if (mul) std::memcpy(mul, s->mul.data(), s->mul.size() * 4);
    if (tri_body) std::memcpy(tri_body, s->tbody.data(), s->tbody.size() * 4);
    if (vert_body) std::memcpy(vert_body, s->vbody.data(), s->vbody.size() * 4);
}

void orc_scene_camera(const orc_scene* s, float* Rv, float* f, float* cx, float* cy, float* gs, float* l) {
    if (Rv) for (int i = 0; i < 3; ++i) { Rv[i] = s->Rt[i]; Rv[3 + i] = s->Up[i]; Rv[6 + i] = s->Fw[i]; }
    if (f) *f = s->f;
    if (cx) std::memcpy(cx, s->cx.data(), s->cx.size() * 4);
    if (cy) std::memcpy(cy, s->cy.data(), s->cy.size() * 4);
    if (gs) { gs[0] = s->gs[0]; gs[1] = s->gs[1]; }
    if (l) for (int i = 0; i < 3; ++i) l[i] = s->l[i];
}

void orc_vertex_stage(const orc_scene* s, const float* poses, const float* shapes, int32_t* X, int32_t* Y,
                      float* D, uint8_t* rejected, float* eye) {
    FrameXform fx;
    vertex_stage(s, poses, shapes, fx, X, Y, D, rejected);
    if (eye) for (int i = 0; i < 3; ++i) eye[i] = fx.eye[i];
}

void orc_raster(uint32_t width, uint32_t height, uint32_t n_verts, const int32_t* X, const int32_t* Y,
                const float* D, const uint8_t* rejected, uint32_t n_tris, const uint32_t* tris,
                const uint32_t* order, uint32_t cull, uint32_t* ids, uint32_t* depth_bits, uint32_t* cover) {
    (void)n_verts;
    size_t n = (size_t)width * height;
    ZBuf zb;
    zb.reset(n);
    if (cover) std::memset(cover, 0, n * 4);
    for (uint32_t k = 0; k < n_tris; ++k) {
        uint32_t g = order ? order[k] : k;
        raster_triangle(width, height, X, Y, D, rejected, tris + (size_t)g * 3, g, cull, &zb, cover);
    }
    if (ids) std::memcpy(ids, zb.id.data(), n * 4);
    if (depth_bits) for (size_t i = 0; i < n; ++i) depth_bits[i] = fbits(zb.depth[i]);
}

int orc_render(const orc_scene* s, const float* poses, const float* shapes, uint32_t B, uint32_t S,
               uint32_t step0, uint32_t env0, const orc_distractor* dis, const uint32_t* order,
               uint8_t* frames, uint32_t* ids, uint32_t* depth_bits) {
    if (!s || !poses || !frames) return 1;
    const uint32_t W = s->W, H = s->H, K = s->K;
    const uint32_t V = (uint32_t)s->vbody.size(), T = (uint32_t)s->tbody.size();
    const size_t npix = (size_t)W * H;
    const uint32_t mode = dis ? dis->mode : ORC_DIS_NONE;
    if (mode == ORC_DIS_VIDEO && (!dis->video || dis->n_frames == 0)) return 1;
    std::vector<int32_t> X(V), Y(V);
    std::vector<float> D(V);
    std::vector<uint8_t> rej(V);
    std::vector<float> PV((size_t)V * 3);
    FrameXform fx;
    ZBuf zb;
    for (uint32_t e = 0; e < B; ++e) {
        const uint32_t env = env0 + e;
        const float* shp = shapes ? shapes + (size_t)e * K * 4 : nullptr;
        for (uint32_t st = 0; st < S; ++st) {
            const uint32_t step = step0 + st;
            const size_t frame = (size_t)e * S + st;
            const float* pose = poses + frame * K * 7;
            // V
            vertex_stage(s, pose, shp, fx, X.data(), Y.data(), D.data(), rej.data(), PV.data());
            // R (triangles reaching behind the near plane are clipped first)
            zb.reset(npix);
            for (uint32_t k = 0; k < T; ++k) {
                uint32_t g = order ? order[k] : k;
                const uint32_t* tri = &s->tri[(size_t)g * 3];
                const uint8_t r0 = rej[tri[0]], r1 = rej[tri[1]], r2 = rej[tri[2]];
                if (r0 != 1 && r1 != 1 && r2 != 1 && (r0 | r1 | r2) == 2)
                    clip_and_raster(s, PV.data(), X.data(), Y.data(), D.data(), rej.data(), tri, g, &zb);
                else
                    raster_triangle(W, H, X.data(), Y.data(), D.data(), rej.data(), tri, g, 0, &zb, nullptr);
            }
            // X: per-frame draws
            float scale[3] = {1.0f, 1.0f, 1.0f}, offs[3] = {0.0f, 0.0f, 0.0f};
            const uint8_t* vframe = nullptr;
            if (mode == ORC_DIS_COLOR) {
                uint32_t r[4];
                philox(dis->seed, env, step, 0u, 0u, r);
                for (int c = 0; c < 3; ++c) scale[c] = std::fmaf(u01(r[c]), dis->scale_hi - dis->scale_lo, dis->scale_lo);
                philox(dis->seed, env, step, 1u, 0u, r);
                for (int c = 0; c < 3; ++c) offs[c] = std::fmaf(u01(r[c]), dis->offset_hi - dis->offset_lo, dis->offset_lo);
            } else if (mode == ORC_DIS_VIDEO) {
                uint32_t eo;
                if (dis->env_offset) eo = dis->env_offset[e];
                else {
                    uint32_t r[4];
                    philox(dis->seed, env, 0xFFFFFFFFu, 2u, 0u, r);
                    eo = r[0] % dis->n_frames;
                }
                uint32_t fi = (uint32_t)(((uint64_t)eo + (uint64_t)step) % dis->n_frames);
                // which clip: each environment plays one clip of the set, drawn at random (paper section 2)
                uint32_t clip = 0;
                if (dis->n_videos > 1) {
                    if (dis->env_video) clip = dis->env_video[e] % dis->n_videos;
                    else {
                        uint32_t r[4];
                        philox(dis->seed, env, 0xFFFFFFFFu, 3u, 0u, r);
                        clip = r[0] % dis->n_videos;
                    }
                }
                vframe = dis->video + ((size_t)clip * dis->n_frames + fi) * npix * 3;
            }
            // G + S + X per pixel
            const float inv_ez = 1.0f / fx.eye[2];
            uint8_t* out = frames + frame * npix * 3;
            for (uint32_t j = 0; j < H; ++j)
                for (uint32_t i = 0; i < W; ++i) {
                    const size_t pix = (size_t)j * W + i;
                    float cxi = s->cx[i], cyj = s->cy[j];
                    float dwx = std::fmaf(s->Rt[0], cxi, std::fmaf(s->Up[0], cyj, s->Fw[0]));
                    float dwy = std::fmaf(s->Rt[1], cxi, std::fmaf(s->Up[1], cyj, s->Fw[1]));
                    float dwz = std::fmaf(s->Rt[2], cxi, std::fmaf(s->Up[2], cyj, s->Fw[2]));
                    float ndz = -dwz;
                    float tg = 0.0f;
                    if (s->ground_on && fx.eye[2] > 0.0f && ndz > 0.0f) {
                        tg = fx.eye[2] / ndz;
                        if (tg >= s->z_near && tg <= s->z_far) {
                            float dg = (s->z_near * ndz) * inv_ez;
                            zb.test(pix, dg, ORC_ID_GROUND);
                        }
                    }
                    const uint32_t g = zb.id[pix];
                    float c[3];
                    if (g == ORC_ID_BG) {
                        for (int ch = 0; ch < 3; ++ch) c[ch] = s->bg[ch];
                    } else if (g == ORC_ID_GROUND) {
                        float wx = std::fmaf(tg, dwx, fx.eye[0]);
                        float wy = std::fmaf(tg, dwy, fx.eye[1]);
                        // (the sum wraps: only its parity is used)
                        int par = (int)(((uint32_t)to_int_saturating(std::floor(wx / s->cell)) +
                                         (uint32_t)to_int_saturating(std::floor(wy / s->cell))) & 1u);
                        for (int ch = 0; ch < 3; ++ch) c[ch] = s->gs[par];
                    } else {
                        const uint32_t b = s->tbody[g];
                        const float* n = &s->nrm[(size_t)g * 3];
                        const float* lb = &fx.lb[b * 3];
                        float I = std::fmaf(n[0], lb[0], std::fmaf(n[1], lb[1], n[2] * lb[2]));
                        I = I > 0.0f ? I : 0.0f;
                        float sh = std::fmaf(s->diffuse, I, s->ambient);
                        for (int ch = 0; ch < 3; ++ch) {
                            float v = (s->bodies[b].rgb[ch] * s->mul[g]) * sh;
                            c[ch] = v < 1.0f ? v : 1.0f;
                        }
                    }
                    if (mode == ORC_DIS_COLOR) {
                        for (int ch = 0; ch < 3; ++ch) {
                            float v = std::fmaf(c[ch], scale[ch], offs[ch]);
                            v = v > 0.0f ? v : 0.0f;
                            c[ch] = v < 1.0f ? v : 1.0f;
                        }
                    } else if (mode == ORC_DIS_VIDEO && (g == ORC_ID_BG || g == ORC_ID_GROUND)) {
                        for (int ch = 0; ch < 3; ++ch) {
                            float vf = (float)vframe[pix * 3 + ch] * (1.0f / 255.0f);
                            c[ch] = std::fmaf(dis->alpha, vf - c[ch], c[ch]);
                        }
                    }
                    for (int ch = 0; ch < 3; ++ch)
                        out[pix * 3 + ch] = (uint8_t)(uint32_t)to_int_saturating(std::floor(std::fmaf(c[ch], 255.0f, 0.5f)));
                }
            if (ids) std::memcpy(ids + frame * npix, zb.id.data(), npix * 4);
            if (depth_bits) for (size_t p = 0; p < npix; ++p) depth_bits[frame * npix + p] = fbits(zb.depth[p]);
        }
    }
    return 0;
}

// ---------------------------------------------------------------- F: forward kinematics
//
// sin(theta/2), cos(theta/2) by their definition: the C library's double-precision routines on the exact
// half angle, each result rounded once to fp32.  Hinge angles beyond +-65536 rad (and non-finite ones) are
// outside the stage's domain: both come out as NaN, so the body and everything hanging on it vanish from
// the frame (a NaN vertex drops its triangles).
namespace {
void sincos_half(float theta, float* s_out, float* c_out) {
    if (!(std::fabs(theta) <= 65536.0f)) {
        *s_out = *c_out = std::numeric_limits<float>::quiet_NaN();
        return;
    }
    const double h = 0.5 * (double)theta;
    *s_out = (float)std::sin(h);
    *c_out = (float)std::cos(h);
}
}  // namespace

namespace {
void quat_matrix(const float* q, float R[3][3]) {  // same formulas as the vertex stage (V)
    const float w = q[0], x = q[1], y = q[2], z = q[3];
    R[0][0] = 1.0f - 2.0f * (y * y + z * z);
    R[0][1] = 2.0f * (x * y - w * z);
    R[0][2] = 2.0f * (x * z + w * y);
    R[1][0] = 2.0f * (x * y + w * z);
    R[1][1] = 1.0f - 2.0f * (x * x + z * z);
    R[1][2] = 2.0f * (y * z - w * x);
    R[2][0] = 2.0f * (x * z - w * y);
    R[2][1] = 2.0f * (y * z + w * x);
    R[2][2] = 1.0f - 2.0f * (x * x + y * y);
}
}  // namespace

int orc_fk(uint32_t n_bodies, const int32_t* parent, const int32_t* slot, const float* anchor, const float* axis,
           const float* offset, const float* free_poses, const float* angles, float* out) {
    for (uint32_t k = 0; k < n_bodies; ++k) {
        float* o = out + (size_t)k * 7;
        if (parent[k] < 0) {
            if (slot[k] < 0) return 1;
            for (int i = 0; i < 7; ++i) o[i] = free_poses[(size_t)slot[k] * 7 + i];
            continue;
        }
        if ((uint32_t)parent[k] >= k) return 1;
        const float* pp = out + (size_t)parent[k] * 7;
        const float* pq = pp + 3;
        const float theta = slot[k] >= 0 ? angles[slot[k]] : 0.0f;
        float sn, cs;
        sincos_half(theta, &sn, &cs);
        const float* u = axis + (size_t)k * 3;
        const float jw = cs, jx = sn * u[0], jy = sn * u[1], jz = sn * u[2];
        const float pw = pq[0], px = pq[1], py = pq[2], pz = pq[3];
        // Hamilton product parent (x) joint
        float q[4];
        q[0] = std::fmaf(-pz, jz, std::fmaf(-py, jy, std::fmaf(-px, jx, pw * jw)));
        q[1] = std::fmaf(py, jz, std::fmaf(-pz, jy, std::fmaf(px, jw, pw * jx)));
        q[2] = std::fmaf(pz, jx, std::fmaf(-px, jz, std::fmaf(py, jw, pw * jy)));
        q[3] = std::fmaf(px, jy, std::fmaf(-py, jx, std::fmaf(pz, jw, pw * jz)));
        float Rp[3][3], Rk[3][3];
        quat_matrix(pq, Rp);
        quat_matrix(q, Rk);
        const float* a = anchor + (size_t)k * 3;
        const float* c = offset + (size_t)k * 3;
        for (int r = 0; r < 3; ++r) {
            const float t1 = dot3(Rp[r], a[0], a[1], a[2]);
            const float t2 = dot3(Rk[r], c[0], c[1], c[2]);
            o[r] = (pp[r] + t1) + t2;
        }
        for (int i = 0; i < 4; ++i) o[3 + i] = q[i];
    }
    return 0;
}

void orc_philox(uint64_t seed, uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t* out) {
    philox(seed, c0, c1, c2, c3, out);
}

float orc_u01(uint32_t x) { return u01(x); }

}  // extern "C"
