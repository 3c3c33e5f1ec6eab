// Driver for the sanitizer test of the library's host-side scene builder (csrc/scene.cpp is plain C++: no
// device call in it): scenes with every primitive kind and a caller's mesh, at several image sizes (unbanded,
// banded, many bands), and descriptions the builder must reject.  Built with -fsanitize=address,undefined by
// tests/test_host_sanitizers.py; prints "ok <n>" and exits 0 when every scene came out as expected.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <string>
#include <vector>

#include "../paper_2502_00021_amd/csrc/pxr_internal.h"

namespace {

pxr_body_desc body(uint32_t type, float a, float b, float c, float h, uint32_t lon, uint32_t lat) {
    pxr_body_desc d{};
    d.type = type;
    d.shape[0] = a; d.shape[1] = b; d.shape[2] = c; d.shape[3] = h;
    d.rgb[0] = 0.8f; d.rgb[1] = 0.4f; d.rgb[2] = 0.2f;
    d.n_lon = lon; d.n_lat = lat;
    return d;
}

pxr_scene_desc scene(uint32_t W, uint32_t H, const std::vector<pxr_body_desc>& bodies) {
    pxr_scene_desc s{};
    s.width = W; s.height = H; s.n_bodies = (uint32_t)bodies.size(); s.root_body = 0; s.bodies = bodies.data();
    s.fov_y_deg = 60.0f;
    s.cam_offset[0] = -2.5f; s.cam_offset[1] = 0.0f; s.cam_offset[2] = 1.0f;
    s.cam_up[0] = 0.0f; s.cam_up[1] = 0.0f; s.cam_up[2] = 1.0f;
    s.z_near = 0.1f; s.z_far = 50.0f;
    s.light_dir[0] = -0.4f; s.light_dir[1] = -0.3f; s.light_dir[2] = 0.85f;
    s.ambient = 0.3f; s.diffuse = 0.7f;
    s.ground_enabled = 1; s.ground_cell = 1.0f; s.ground_grey[0] = 0.35f; s.ground_grey[1] = 0.65f;
    s.background_rgb[0] = 0.55f; s.background_rgb[1] = 0.7f; s.background_rgb[2] = 0.9f;
    return s;
}

int expect(const pxr_scene_desc& d, bool ok, const char* what) {
    pxr::HostScene hs;
    std::string err;
    const int rc = pxr::build_host_scene(d, hs, err);
    if ((rc == PXR_OK) != ok) {
        std::fprintf(stderr, "%s: expected %s, got code %d (%s)\n", what, ok ? "success" : "an error", rc, err.c_str());
        return 1;
    }
    if (ok) {
        // every table has the size its counts say, every index stays inside its table
        if (hs.vtmpl.size() != (size_t)hs.c.V * 4 || hs.tri_idx.size() != (size_t)hs.c.T * 2 || hs.tri_shade.size() != (size_t)hs.c.T * 4 ||
            hs.pair_tbl.size() != (size_t)hs.c.P * 4 || hs.cxcy.size() != (size_t)hs.c.W + hs.c.H) {
            std::fprintf(stderr, "%s: table sizes do not match the counts\n", what);
            return 1;
        }
        for (uint32_t t = 0; t < hs.c.T; ++t) {
            const uint32_t a = hs.tri_idx[2 * t] & 0xFFFFu, b = hs.tri_idx[2 * t] >> 16, c = hs.tri_idx[2 * t + 1] & 0xFFFFu;
            if (a >= hs.c.V || b >= hs.c.V || c >= hs.c.V) {
                std::fprintf(stderr, "%s: triangle %u points outside the vertex table\n", what, t);
                return 1;
            }
        }
        if (hs.c.lds_total > 160u * 1024u || hs.c.band_rows == 0 || hs.c.band_rows > hs.c.H || hs.c.first_band_rows > hs.c.band_rows + hs.c.H) {
            std::fprintf(stderr, "%s: LDS layout out of range\n", what);
            return 1;
        }
    }
    return 0;
}

}  // namespace

int main() {
    int bad = 0, n = 0;
    std::vector<pxr_body_desc> mix = {body(PXR_SPHERE, 0.25f, 0.25f, 0.25f, 0.0f, 16, 8), body(PXR_CAPSULE, 0.1f, 0.1f, 0.1f, 0.3f, 12, 6),
                                      body(PXR_BOX, 0.3f, 0.2f, 0.1f, 0.0f, 4, 0), body(PXR_CAPSULE, 0.05f, 0.05f, 0.05f, 0.0f, 3, 1)};
    // a caller's mesh: a tetrahedron and a triangle without area
    const float mv[] = {0, 0, 0, 1, 0, 0, 0, 1, 0, 0, 0, 1, 2, 2, 2};
    const uint32_t mt[] = {0, 2, 1, 0, 1, 3, 1, 2, 3, 0, 3, 2, 4, 4, 4};
    const float mm[] = {1.0f, 0.5f, 0.25f, 1.0f, 0.0f};
    pxr_body_desc mesh = body(PXR_MESH, 1.0f, 1.0f, 1.0f, 0.0f, 0, 0);
    mesh.mesh_verts = mv; mesh.mesh_tris = mt; mesh.mesh_tri_mul = mm; mesh.n_mesh_verts = 5; mesh.n_mesh_tris = 5;
    std::vector<pxr_body_desc> with_mesh = mix;
    with_mesh.push_back(mesh);

    const uint32_t sizes[][2] = {{8, 8}, {33, 27}, {64, 64}, {84, 84}, {110, 100}, {128, 128}, {256, 256}, {500, 36}, {512, 512}, {9, 512}};
    for (const auto& wh : sizes) {
        bad += expect(scene(wh[0], wh[1], mix), true, "primitive mix"); ++n;
        bad += expect(scene(wh[0], wh[1], with_mesh), true, "primitive mix with a mesh"); ++n;
    }
    // a humanoid-sized scene and a 64-body one
    std::vector<pxr_body_desc> many;
    for (int i = 0; i < 14; ++i) many.push_back(body(PXR_CAPSULE, 0.06f, 0.06f, 0.06f, 0.2f, 12, 6));
    many.push_back(body(PXR_BOX, 0.3f, 0.3f, 0.3f, 0.0f, 4, 0));
    bad += expect(scene(64, 64, many), true, "humanoid and box"); ++n;
    bad += expect(scene(84, 84, many), true, "humanoid and box, banded"); ++n;
    std::vector<pxr_body_desc> sixty_four(64, body(PXR_SPHERE, 0.05f, 0.05f, 0.05f, 0.0f, 4, 2));
    bad += expect(scene(32, 32, sixty_four), true, "sixty-four bodies"); ++n;

    // descriptions the builder must turn down (with a message, without touching anything out of bounds)
    { auto d = scene(64, 64, mix); d.n_bodies = 0; bad += expect(d, false, "no bodies"); ++n; }
    { auto d = scene(64, 64, mix); d.root_body = 9; bad += expect(d, false, "root out of range"); ++n; }
    { auto d = scene(4, 64, mix); bad += expect(d, false, "image too small"); ++n; }
    { auto d = scene(64, 513, mix); bad += expect(d, false, "image too large"); ++n; }
    { auto d = scene(64, 64, mix); d.fov_y_deg = 180.0f; bad += expect(d, false, "field of view"); ++n; }
    { auto d = scene(64, 64, mix); d.z_near = 0.0f; bad += expect(d, false, "near plane"); ++n; }
    { auto d = scene(64, 64, mix); d.z_far = d.z_near; bad += expect(d, false, "far plane"); ++n; }
    { auto d = scene(64, 64, mix); d.cam_offset[0] = d.cam_offset[2] = 0.0f; bad += expect(d, false, "camera on the root"); ++n; }
    { auto d = scene(64, 64, mix); d.cam_up[0] = -2.5f; d.cam_up[1] = 0.0f; d.cam_up[2] = 1.0f; bad += expect(d, false, "up along the view"); ++n; }
    { auto d = scene(64, 64, mix); d.background_rgb[1] = 1.5f; bad += expect(d, false, "colour above one"); ++n; }
    { auto d = scene(64, 64, mix); d.ground_grey[0] = -0.1f; bad += expect(d, false, "negative grey"); ++n; }
    { auto d = scene(64, 64, mix); d.light_dir[0] = NAN; bad += expect(d, false, "non-finite light"); ++n; }
    { auto b = mix; b[1].n_lon = 2; bad += expect(scene(64, 64, b), false, "two longitudes"); ++n; }
    { auto b = mix; b[0].shape[0] = NAN; bad += expect(scene(64, 64, b), false, "non-finite radius"); ++n; }
    { auto b = mix; b[0].shape[0] = -0.25f; bad += expect(scene(64, 64, b), true, "mirrored body (shapes are scale factors)"); ++n; }
    { auto b = mix; b[2].type = 7; bad += expect(scene(64, 64, b), false, "unknown body type"); ++n; }
    { auto b = mix; b[0].rgb[2] = INFINITY; bad += expect(scene(64, 64, b), false, "non-finite colour"); ++n; }
    { auto b = with_mesh; b.back().mesh_verts = nullptr; bad += expect(scene(64, 64, b), false, "mesh without vertices"); ++n; }
    { auto b = with_mesh; const uint32_t wild[] = {0, 1, 9}; b.back().mesh_tris = wild; b.back().n_mesh_tris = 1;
      bad += expect(scene(64, 64, b), false, "mesh index out of range"); ++n; }
    { auto b = with_mesh; const float neg[] = {-1.0f}; b.back().mesh_tri_mul = neg; b.back().n_mesh_tris = 1;
      bad += expect(scene(64, 64, b), false, "negative multiplier"); ++n; }
    { std::vector<pxr_body_desc> heavy(40, body(PXR_SPHERE, 0.2f, 0.2f, 0.2f, 0.0f, 64, 32));
      bad += expect(scene(64, 64, heavy), false, "more geometry than LDS holds"); ++n; }
    if (bad) return 1;
    std::printf("ok %d\n", n);
    return 0;
}
