// Host-side scene builder of libpxr: validation, tessellation of the unit
// primitives, camera / light / ground constants.  Runs once per scene, never
// on the hot path.  (The paper leaves geometry, camera and shading
// conventions open; the conventions here are this library's definition of a
// "scene of posed primitives" and are documented with the C ABI.)
//
// Numerical contract: every table is evaluated in double from the float
// inputs with libm, each entry rounded to fp32 exactly once.

#include <algorithm>
#include <cmath>
#include <cstring>

#include "pxr_internal.h"

namespace pxr {
namespace {

constexpr double kPi = 3.14159265358979323846;

struct Vec3d {
    double x, y, z;
};

inline Vec3d sub(const Vec3d& a, const Vec3d& b) { return {a.x - b.x, a.y - b.y, a.z - b.z}; }
inline Vec3d cross(const Vec3d& a, const Vec3d& b) {
    return {a.y * b.z - a.z * b.y, a.z * b.x - a.x * b.z, a.x * b.y - a.y * b.x};
}
inline double norm(const Vec3d& a) { return std::sqrt(a.x * a.x + a.y * a.y + a.z * a.z); }

inline float as_float(uint32_t u) {
    float f;
    std::memcpy(&f, &u, 4);
    return f;
}

// Collects one body's mesh in body-local numbering; flushed into the scene
// tables with the body's vertex base added.
struct BodyMesh {
    std::vector<Vec3d> pos;     // unit-shape positions (double)
    std::vector<int> cap;       // cap selector s in {+1,0,-1}
    std::vector<uint32_t> idx;  // 3 per triangle, local
    std::vector<Vec3d> nrm;     // per triangle
    std::vector<float> mul;     // per triangle

    void tri(uint32_t a, uint32_t b, uint32_t c, const Vec3d& n, float m = 1.0f) {
        idx.push_back(a);
        idx.push_back(b);
        idx.push_back(c);
        nrm.push_back(n);
        mul.push_back(m);
    }
    Vec3d face_normal(uint32_t a, uint32_t b, uint32_t c) const {
        Vec3d n = cross(sub(pos[b], pos[a]), sub(pos[c], pos[a]));
        double len = norm(n);
        return {n.x / len, n.y / len, n.z / len};
    }
};

// Latitude rings of a capsule or sphere, top to bottom.
struct RingSpec {
    double theta;
    bool equator;  // sin = 1, cos = 0 exactly
    int cap;
};

// Capsule: poles + 2*M rings (the two equators coincide on the unit sphere and
// are pulled apart by the cap selector).  Sphere: poles + 2*M-1 rings.
void tessellate_round(BodyMesh& m, uint32_t L, uint32_t M, bool capsule) {
    std::vector<RingSpec> rings;
    if (capsule) {
        for (uint32_t k = 1; k <= M; ++k) rings.push_back({((double)k * (kPi / 2.0)) / (double)M, k == M, +1});
        for (uint32_t k = 0; k < M; ++k) rings.push_back({kPi / 2.0 + ((double)k * (kPi / 2.0)) / (double)M, k == 0, -1});
    } else {
        for (uint32_t k = 1; k < 2 * M; ++k) rings.push_back({((double)k * kPi) / (double)(2 * M), k == M, 0});
    }
    const uint32_t R = (uint32_t)rings.size();
    const uint32_t n_verts = R * L + 2;
    m.pos.resize(n_verts);
    m.cap.resize(n_verts);
    m.pos[0] = {0.0, 0.0, 1.0};
    m.cap[0] = capsule ? +1 : 0;
    m.pos[n_verts - 1] = {0.0, 0.0, -1.0};
    m.cap[n_verts - 1] = capsule ? -1 : 0;
    for (uint32_t r = 0; r < R; ++r) {
        const double s = rings[r].equator ? 1.0 : std::sin(rings[r].theta);
        const double c = rings[r].equator ? 0.0 : std::cos(rings[r].theta);
        for (uint32_t j = 0; j < L; ++j) {
            const double phi = ((2.0 * kPi) * (double)j) / (double)L;
            m.pos[1 + r * L + j] = {s * std::cos(phi), s * std::sin(phi), c};
            m.cap[1 + r * L + j] = rings[r].cap;
        }
    }
    auto at = [L](uint32_t r, uint32_t j) { return 1 + r * L + (j == L ? 0 : j); };
    // top fan
    for (uint32_t j = 0; j < L; ++j) m.tri(0, at(0, j), at(0, j + 1), m.face_normal(0, at(0, j), at(0, j + 1)));
    // bands between consecutive rings: upper-left, lower-left, lower-right / upper-left, lower-right, upper-right
    for (uint32_t r = 0; r + 1 < R; ++r) {
        const bool cylinder = capsule && rings[r].cap != rings[r + 1].cap;
        for (uint32_t j = 0; j < L; ++j) {
            const uint32_t ul = at(r, j), ur = at(r, j + 1), ll = at(r + 1, j), lr = at(r + 1, j + 1);
            if (cylinder) {
                const double phi = ((2.0 * kPi) * ((double)j + 0.5)) / (double)L;
                const Vec3d n{std::cos(phi), std::sin(phi), 0.0};
                m.tri(ul, ll, lr, n);
                m.tri(ul, lr, ur, n);
            } else {
                m.tri(ul, ll, lr, m.face_normal(ul, ll, lr));
                m.tri(ul, lr, ur, m.face_normal(ul, lr, ur));
            }
        }
    }
    // bottom fan
    const uint32_t south = n_verts - 1;
    for (uint32_t j = 0; j < L; ++j)
        m.tri(at(R - 1, j), south, at(R - 1, j + 1), m.face_normal(at(R - 1, j), south, at(R - 1, j + 1)));
}

// Box faces +x,-x,+y,-y,+z,-z with (u,v) axes such that u x v = outward normal.
void tessellate_box(BodyMesh& m, uint32_t n) {
    struct Face {
        int axis;
        double sign;
        int u, v;
    };
    const Face faces[6] = {{0, +1.0, 1, 2}, {0, -1.0, 2, 1}, {1, +1.0, 2, 0}, {1, -1.0, 0, 2}, {2, +1.0, 0, 1}, {2, -1.0, 1, 0}};
    const uint32_t side = n + 1;
    for (int f = 0; f < 6; ++f) {
        const uint32_t base = (uint32_t)m.pos.size();
        for (uint32_t iv = 0; iv < side; ++iv)
            for (uint32_t iu = 0; iu < side; ++iu) {
                double p[3];
                p[faces[f].axis] = faces[f].sign;
                p[faces[f].u] = -1.0 + (2.0 * (double)iu) / (double)n;
                p[faces[f].v] = -1.0 + (2.0 * (double)iv) / (double)n;
                m.pos.push_back({p[0], p[1], p[2]});
                m.cap.push_back(0);
            }
        double nn[3] = {0.0, 0.0, 0.0};
        nn[faces[f].axis] = faces[f].sign;
        const Vec3d normal{nn[0], nn[1], nn[2]};
        for (uint32_t cv = 0; cv < n; ++cv)
            for (uint32_t cu = 0; cu < n; ++cu) {
                const uint32_t p00 = base + cv * side + cu;
                const uint32_t p10 = p00 + 1, p01 = p00 + side, p11 = p01 + 1;
                const float checker = ((cu ^ cv) & 1u) ? 0.5f : 1.0f;
                m.tri(p00, p10, p11, normal, checker);
                m.tri(p00, p11, p01, normal, checker);
            }
    }
}

// Binning works on pairs of triangles that share an edge (a quad of a band, a
// box cell, two neighbouring fan triangles): one box test over four vertices
// settles both.  Consecutive triangles t, t+1 of a body are paired when t+1
// runs along one of t's edges in the opposite direction; the entry is
// (q0,q1,q2,q3) with t = {q0,q1,q2}, t+1 = {q0,q2,q3} as vertex sets.  A
// triangle without such a neighbour stands alone (q3 = q2).
void pair_triangles(const BodyMesh& m, uint32_t vbase, uint32_t tbase, std::vector<uint32_t>& tbl) {
    const uint32_t nt = (uint32_t)m.mul.size();
    uint32_t t = 0;
    while (t < nt) {
        const uint32_t* A = &m.idx[3 * t];
        bool paired = false;
        if (t + 1 < nt) {
            const uint32_t* B = &m.idx[3 * (t + 1)];
            for (int eb = 0; eb < 3 && !paired; ++eb) {
                const uint32_t x = B[eb], y = B[(eb + 1) % 3], b3 = B[(eb + 2) % 3];
                for (int ea = 0; ea < 3; ++ea) {
                    if (A[ea] == y && A[(ea + 1) % 3] == x) {
                        const uint32_t a3 = A[(ea + 2) % 3];
                        tbl.push_back((vbase + x) | ((vbase + a3) << 16));
                        tbl.push_back((vbase + y) | ((vbase + b3) << 16));
                        tbl.push_back((tbase + t) | ((tbase + t + 1) << 16));
                        tbl.push_back(0u);  // pad to one 16-byte load
                        paired = true;
                        break;
                    }
                }
            }
        }
        if (paired) {
            t += 2;
        } else {
            tbl.push_back((vbase + A[0]) | ((vbase + A[1]) << 16));
            tbl.push_back((vbase + A[2]) | ((vbase + A[2]) << 16));
            tbl.push_back((tbase + t) | (kNoTriangle << 16));
            tbl.push_back(0u);
            t += 1;
        }
    }
}

// A caller-supplied mesh: vertices and triangle order are kept; normals from the unscaled vertices.
void tessellate_mesh(BodyMesh& m, const pxr_body_desc& bd) {
    for (uint32_t v = 0; v < bd.n_mesh_verts; ++v) {
        m.pos.push_back({(double)bd.mesh_verts[3 * v], (double)bd.mesh_verts[3 * v + 1], (double)bd.mesh_verts[3 * v + 2]});
        m.cap.push_back(0);
    }
    for (uint32_t t = 0; t < bd.n_mesh_tris; ++t) {
        const uint32_t a = bd.mesh_tris[3 * t], b = bd.mesh_tris[3 * t + 1], c = bd.mesh_tris[3 * t + 2];
        const Vec3d n = cross(sub(m.pos[b], m.pos[a]), sub(m.pos[c], m.pos[a]));
        const double len = norm(n);
        Vec3d unit{n.x / len, n.y / len, n.z / len};
        if (!(std::isfinite(unit.x) && std::isfinite(unit.y) && std::isfinite(unit.z))) unit = {0.0, 0.0, 0.0};
        m.tri(a, b, c, unit, bd.mesh_tri_mul ? bd.mesh_tri_mul[t] : 1.0f);
    }
}

// Pairing for meshes of unknown structure: every triangle is matched greedily with a not yet matched
// triangle that shares one of its edges (any orientation; the binning test only looks at the two
// vertex sets).  Same table format as pair_triangles.
void pair_triangles_general(const BodyMesh& m, uint32_t vbase, uint32_t tbase, std::vector<uint32_t>& tbl) {
    const uint32_t nt = (uint32_t)m.mul.size();
    auto key = [](uint32_t a, uint32_t b) { return ((uint64_t)std::min(a, b) << 32) | std::max(a, b); };
    std::vector<std::pair<uint64_t, uint32_t>> edges;  // (edge, triangle), sorted: neighbours sit together
    edges.reserve((size_t)nt * 3);
    for (uint32_t t = 0; t < nt; ++t)
        for (int e = 0; e < 3; ++e) edges.push_back({key(m.idx[3 * t + e], m.idx[3 * t + (e + 1) % 3]), t});
    std::sort(edges.begin(), edges.end());
    std::vector<uint32_t> mate(nt, kNoTriangle);
    for (uint32_t t = 0; t < nt; ++t) {
        if (mate[t] != kNoTriangle) continue;
        for (int e = 0; e < 3 && mate[t] == kNoTriangle; ++e) {
            const uint32_t x = m.idx[3 * t + e], y = m.idx[3 * t + (e + 1) % 3];
            if (x == y) continue;
            const uint64_t k = key(x, y);
            for (auto it = std::lower_bound(edges.begin(), edges.end(), std::make_pair(k, 0u));
                 it != edges.end() && it->first == k; ++it) {
                const uint32_t u = it->second;
                if (u != t && mate[u] == kNoTriangle) {
                    mate[t] = u;
                    mate[u] = t;
                    // q0, q2 = the shared edge; q1, q3 = the two remaining corners
                    const uint32_t a3 = m.idx[3 * t + (e + 2) % 3];
                    uint32_t b3 = x;
                    for (int q = 0; q < 3; ++q)
                        if (m.idx[3 * u + q] != x && m.idx[3 * u + q] != y) b3 = m.idx[3 * u + q];
                    tbl.push_back((vbase + x) | ((vbase + a3) << 16));
                    tbl.push_back((vbase + y) | ((vbase + b3) << 16));
                    tbl.push_back((tbase + t) | ((tbase + u) << 16));
                    tbl.push_back(0u);
                    break;
                }
            }
        }
        if (mate[t] == kNoTriangle) {
            mate[t] = t;
            tbl.push_back((vbase + m.idx[3 * t]) | ((vbase + m.idx[3 * t + 1]) << 16));
            tbl.push_back((vbase + m.idx[3 * t + 2]) | ((vbase + m.idx[3 * t + 2]) << 16));
            tbl.push_back((tbase + t) | (kNoTriangle << 16));
            tbl.push_back(0u);
        }
    }
}

bool finite_all(const float* p, int n) {
    for (int i = 0; i < n; ++i)
        if (!std::isfinite(p[i])) return false;
    return true;
}

bool unit_all(const float* p, int n) {  // colours: fractions of full intensity
    for (int i = 0; i < n; ++i)
        if (!(p[i] >= 0.0f && p[i] <= 1.0f)) return false;
    return true;
}

}  // namespace

int build_host_scene(const pxr_scene_desc& d, HostScene& hs, std::string& err) {
    SceneConsts& c = hs.c;
    if (d.width < 8 || d.width > 512 || d.height < 8 || d.height > 512) {
        err = "width and height must lie in [8,512]";
        return PXR_ERR_UNSUPPORTED;
    }
    if (d.n_bodies < 1 || d.n_bodies > 64) {
        err = "n_bodies must lie in [1,64]";
        return PXR_ERR_UNSUPPORTED;
    }
    if (!d.bodies) {
        err = "bodies is null";
        return PXR_ERR_INVALID_ARG;
    }
    if (d.root_body >= d.n_bodies) {
        err = "root_body out of range";
        return PXR_ERR_INVALID_ARG;
    }
    if (!std::isfinite(d.fov_y_deg) || !(d.fov_y_deg > 0.0f) || !(d.fov_y_deg < 180.0f) || !finite_all(d.cam_offset, 3) ||
        !finite_all(d.cam_up, 3) || !std::isfinite(d.z_near) || !std::isfinite(d.z_far) || !(d.z_near > 0.0f) ||
        !(d.z_far > d.z_near)) {
        err = "camera parameters must be finite with 0 < fov < 180 and 0 < z_near < z_far";
        return PXR_ERR_INVALID_ARG;
    }
    if (!finite_all(d.light_dir, 3) || !std::isfinite(d.ambient) || !std::isfinite(d.diffuse) || d.ambient < 0.0f ||
        d.diffuse < 0.0f) {
        err = "light parameters must be finite and non-negative";
        return PXR_ERR_INVALID_ARG;
    }
    if (!std::isfinite(d.ground_cell) || !(d.ground_cell > 0.0f) || !finite_all(d.ground_grey, 2) ||
        !finite_all(d.background_rgb, 3)) {
        err = "ground / background parameters must be finite, ground_cell > 0";
        return PXR_ERR_INVALID_ARG;
    }
    if (!unit_all(d.ground_grey, 2) || !unit_all(d.background_rgb, 3)) {
        err = "ground_grey and background_rgb must lie in [0,1]";
        return PXR_ERR_INVALID_ARG;
    }

    c.W = d.width;
    c.H = d.height;
    c.npix = d.width * d.height;
    c.K = d.n_bodies;
    c.root = d.root_body;
    c.magicW = (uint32_t)((0x100000000ull + d.width - 1) / d.width);

    // ---- meshes
    uint32_t vbase = 0, tbase = 0;
    hs.body_const.assign((size_t)d.n_bodies * 8, 0.0f);
    for (uint32_t b = 0; b < d.n_bodies; ++b) {
        const pxr_body_desc& bd = d.bodies[b];
        if (!finite_all(bd.shape, 4) || !finite_all(bd.rgb, 3)) {
            err = "body " + std::to_string(b) + ": non-finite shape or colour";
            return PXR_ERR_INVALID_ARG;
        }
        if (!unit_all(bd.rgb, 3)) {
            err = "body " + std::to_string(b) + ": rgb must lie in [0,1]";
            return PXR_ERR_INVALID_ARG;
        }
        BodyMesh m;
        if (bd.type == PXR_CAPSULE || bd.type == PXR_SPHERE) {
            if (bd.n_lon < 3 || bd.n_lon > 64 || bd.n_lat < 1 || bd.n_lat > 32) {
                err = "body " + std::to_string(b) + ": n_lon must lie in [3,64] and n_lat in [1,32]";
                return PXR_ERR_UNSUPPORTED;
            }
            tessellate_round(m, bd.n_lon, bd.n_lat, bd.type == PXR_CAPSULE);
        } else if (bd.type == PXR_BOX) {
            if (bd.n_lon < 1 || bd.n_lon > 16) {
                err = "body " + std::to_string(b) + ": box cells per edge must lie in [1,16]";
                return PXR_ERR_UNSUPPORTED;
            }
            tessellate_box(m, bd.n_lon);
        } else if (bd.type == PXR_MESH) {
            if (!bd.mesh_verts || !bd.mesh_tris || bd.n_mesh_verts == 0 || bd.n_mesh_tris == 0) {
                err = "body " + std::to_string(b) + ": a mesh needs vertices and triangles";
                return PXR_ERR_INVALID_ARG;
            }
            if (bd.n_mesh_verts > 65535u || bd.n_mesh_tris >= kNoTriangle) {
                err = "scene exceeds 65535 vertices or triangles";
                return PXR_ERR_UNSUPPORTED;
            }
            if (!finite_all(bd.mesh_verts, (int)bd.n_mesh_verts * 3) ||
                (bd.mesh_tri_mul && !finite_all(bd.mesh_tri_mul, (int)bd.n_mesh_tris))) {
                err = "body " + std::to_string(b) + ": non-finite mesh vertex or multiplier";
                return PXR_ERR_INVALID_ARG;
            }
            for (uint32_t t = 0; bd.mesh_tri_mul && t < bd.n_mesh_tris; ++t)
                if (bd.mesh_tri_mul[t] < 0.0f) {
                    err = "body " + std::to_string(b) + ": negative colour multiplier";
                    return PXR_ERR_INVALID_ARG;
                }
            for (uint32_t i = 0; i < bd.n_mesh_tris * 3; ++i)
                if (bd.mesh_tris[i] >= bd.n_mesh_verts) {
                    err = "body " + std::to_string(b) + ": mesh index out of range";
                    return PXR_ERR_INVALID_ARG;
                }
            tessellate_mesh(m, bd);
        } else {
            err = "body " + std::to_string(b) + ": unknown primitive type";
            return PXR_ERR_INVALID_ARG;
        }
        const uint32_t nv = (uint32_t)m.pos.size(), nt = (uint32_t)m.mul.size();
        if (vbase + nv > 65535u || tbase + nt >= kNoTriangle) {
            err = "scene exceeds 65535 vertices or triangles";
            return PXR_ERR_UNSUPPORTED;
        }
        for (uint32_t v = 0; v < nv; ++v) {
            hs.vtmpl.push_back((float)m.pos[v].x);
            hs.vtmpl.push_back((float)m.pos[v].y);
            hs.vtmpl.push_back((float)m.pos[v].z);
            hs.vtmpl.push_back(as_float((b << 2) | (uint32_t)(m.cap[v] + 1)));
        }
        for (uint32_t t = 0; t < nt; ++t) {
            const uint32_t v0 = vbase + m.idx[3 * t], v1 = vbase + m.idx[3 * t + 1], v2 = vbase + m.idx[3 * t + 2];
            hs.tri_idx.push_back(v0 | (v1 << 16));
            hs.tri_idx.push_back(v2 | (b << 16));
            hs.tri_shade.push_back((float)m.nrm[t].x);
            hs.tri_shade.push_back((float)m.nrm[t].y);
            hs.tri_shade.push_back((float)m.nrm[t].z);
            hs.tri_shade.push_back(m.mul[t]);
        }
        if (bd.type == PXR_MESH)
            pair_triangles_general(m, vbase, tbase, hs.pair_tbl);
        else
            pair_triangles(m, vbase, tbase, hs.pair_tbl);
        for (int i = 0; i < 4; ++i) hs.body_const[(size_t)b * 8 + i] = bd.shape[i];
        for (int i = 0; i < 3; ++i) hs.body_const[(size_t)b * 8 + 4 + i] = bd.rgb[i];
        vbase += nv;
        tbase += nt;
    }
    c.V = vbase;
    c.T = tbase;
    c.P = (uint32_t)(hs.pair_tbl.size() / 4);

    // ---- camera: forward looks from the eye to the root, right = forward x up
    const Vec3d off{d.cam_offset[0], d.cam_offset[1], d.cam_offset[2]};
    const Vec3d up{d.cam_up[0], d.cam_up[1], d.cam_up[2]};
    const double off_len = norm(off);
    if (!(off_len > 0.0)) {
        err = "cam_offset must be non-zero";
        return PXR_ERR_INVALID_ARG;
    }
    const Vec3d fw{-off.x / off_len, -off.y / off_len, -off.z / off_len};
    Vec3d rt = cross(fw, up);
    const double rt_len = norm(rt);
    if (!(rt_len > 1e-6 * norm(up))) {
        err = "cam_up is zero or parallel to the viewing direction";
        return PXR_ERR_INVALID_ARG;
    }
    rt = {rt.x / rt_len, rt.y / rt_len, rt.z / rt_len};
    const Vec3d upv = cross(rt, fw);
    const double rtv[3] = {rt.x, rt.y, rt.z}, upa[3] = {upv.x, upv.y, upv.z}, fwa[3] = {fw.x, fw.y, fw.z};
    for (int i = 0; i < 3; ++i) {
        c.Rt[i] = (float)rtv[i];
        c.Up[i] = (float)upa[i];
        c.Fw[i] = (float)fwa[i];
        c.off[i] = d.cam_offset[i];
    }
    const double half_w = (double)d.width / 2.0, half_h = (double)d.height / 2.0;
    const double focal = half_h / std::tan(((double)d.fov_y_deg * kPi / 180.0) / 2.0);
    c.f = (float)focal;
    c.halfW = (float)half_w;
    c.halfH = (float)half_h;
    c.z_near = d.z_near;
    c.z_far = d.z_far;
    hs.cxcy.resize(d.width + d.height);
    for (uint32_t i = 0; i < d.width; ++i) hs.cxcy[i] = (float)((((double)i + 0.5) - half_w) / focal);
    for (uint32_t j = 0; j < d.height; ++j) hs.cxcy[d.width + j] = (float)(-(((double)j + 0.5) - half_h) / focal);

    // ---- light, ground, background
    const Vec3d ld{d.light_dir[0], d.light_dir[1], d.light_dir[2]};
    const double ld_len = norm(ld);
    if (!(ld_len > 0.0)) {
        err = "light_dir must be non-zero";
        return PXR_ERR_INVALID_ARG;
    }
    c.l[0] = (float)(ld.x / ld_len);
    c.l[1] = (float)(ld.y / ld_len);
    c.l[2] = (float)(ld.z / ld_len);
    c.ambient = d.ambient;
    c.diffuse = d.diffuse;
    c.ground_on = d.ground_enabled ? 1u : 0u;
    c.cell = d.ground_cell;
    // A ground point is eye + t * direction with t <= z_far and |direction| < 2^30 (fov < 180 degrees as a float,
    // images up to 512 pixels): with z_far <= 2^64 the product is finite, and the sum is a NaN only if the eye is.
    c.checker_short_form = (d.ground_cell == 1.0f && d.z_far <= 0x1p64f) ? 1u : 0u;
    const double lz = ld.z / ld_len;
    const double lit = (double)d.ambient + (double)d.diffuse * (lz > 0.0 ? lz : 0.0);
    c.gs[0] = std::fmin(1.0f, (float)((double)d.ground_grey[0] * lit));  // (capped like a shaded triangle)
    c.gs[1] = std::fmin(1.0f, (float)((double)d.ground_grey[1] * lit));
    for (int i = 0; i < 3; ++i) c.bg[i] = d.background_rgb[i];

    // ---- LDS carve-up of one frame workgroup.  The pixel keys dominate for tall frames; they are
    // kept for `band_rows` rows at a time.  Prefer the fewest bands that let two workgroups share a
    // compute unit (80 KB each); failing that, the fewest bands that fit at all.
    auto align = [](uint32_t x, uint32_t a) { return (x + a - 1) / a * a; };
    auto layout = [&](uint32_t n_bands, bool whole_trips = false) {
        c.band_rows = (c.H + n_bands - 1) / n_bands;
        c.first_band_rows = c.band_rows;
        if (whole_trips) {
            // Two bands: the resolve loop of the 768-thread workgroups such frames run takes 768 x 4 pixels a trip.
            // A first band of whole trips (and a taller second one) saves the nearly empty trip that an even split
            // ends both bands with: 84 x 84 as 36 + 48 rows is three trips instead of four (+2.4 %).
            const uint32_t rows_per_trip = (768u * 4u) / c.W;
            const uint32_t first = rows_per_trip ? c.band_rows / rows_per_trip * rows_per_trip : 0u;
            if (n_bands != 2 || (c.W & 3u) || first == 0 || first == c.band_rows) return 0xFFFFFFFFu;  // nothing to gain
            c.first_band_rows = first;
            c.band_rows = c.H - first;
        }
        uint32_t o = 0;
        c.lds_keys = o;  // 16-byte aligned regions first
        o += align(std::max(c.band_rows * c.W * 8, c.V * 4 + 4 + c.T * 2), 16);  // (V codes, one word of code 0, T candidates)
        c.lds_cxcy = o;
        o += align((c.W + c.H) * 4, 16);
        c.lds_rows = o;  // float4 per image row
        o += c.H * 16;
        c.lds_misc = o;
        o += 64 * 4;
        c.lds_body = o;
        o += c.K * kBodyStride * 4;
        c.lds_vxy = o;  // (x, y) pairs: 8-byte aligned, as everything before it is a multiple of 16
        o += c.V * 8;
        c.lds_vd = o;
        o += c.V * 4;
        c.lds_list = o;
        o += align(c.T * 2, 4);
        c.lds_large = o;
        o += align(c.T * 2, 4);
        c.lds_blist = c.lds_blist2 = 0;
        if (n_bands >= kBandListsFrom) {  // a band round's lists
            c.lds_blist = o;
            o += kBandListEntries * 2;
            c.lds_blist2 = o;
            o += kBandListEntries * 2;
        }
        c.lds_total = align(o, 16);
        // Video distractor: blended byte by (colour under the clip, clip byte), nine tables of 256 bytes
        // (background r, g, b, and each of the two greys three times, so that "channel" is the same address offset
        // whatever lies under the clip).  Taken only where it costs no workgroup per compute unit.
        c.lds_vlut = 0;
        const uint32_t with_tables = c.lds_total + kVideoTableBytes;
        if (with_tables <= 160u * 1024u && (160u * 1024u) / with_tables == (160u * 1024u) / c.lds_total) {
            c.lds_vlut = c.lds_total;
            c.lds_total = with_tables;
        }
        return c.lds_total;
    };
    const uint32_t kHalf = 80u * 1024u, kAll = 160u * 1024u, kMaxBands = 128;
    uint32_t chosen = 0;
    bool whole_trips = false;
    for (uint32_t nb = 1; nb <= kMaxBands && !chosen; ++nb) {
        if (layout(nb) <= kHalf) chosen = nb;
        if (chosen == 2 && layout(2, true) <= kHalf) whole_trips = true;
    }
    // A frame that would need many bands at half a compute unit's LDS is better off with all of it: a third of the
    // bands (each costs a pass over the bins and three barriers) outweighs having no second workgroup to overlap
    // with (measured: 192x192 +19 %, 256x256 +25 %, 512x512 x2.1; 128x128 and smaller lose 8-15 %).
    if (chosen >= kBandListsFrom) chosen = 0;
    for (uint32_t nb = 1; nb <= kMaxBands && !chosen; ++nb)
        if (layout(nb) <= kAll) chosen = nb;
    if (!chosen) {
        err = "scene needs " + std::to_string(layout(kMaxBands)) + " bytes of LDS per frame; the limit is 163840";
        return PXR_ERR_UNSUPPORTED;
    }
    layout(chosen, whole_trips && chosen == 2);
    return PXR_OK;
}

}  // namespace pxr
