// Driver for the sanitizer test of the CPU oracle: a humanoid-sized scene with every primitive kind,
// degenerate and off-screen poses, both distractors.  Built with -fsanitize=address,undefined by
// tests/test_oracle_sanitizers.py; exits 0 when nothing was flagged.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <vector>

#include "../oracle/orc.h"

int main() {
    const uint32_t W = 40, H = 28, K = 4, B = 6, S = 2;
    const uint32_t kinds[K] = {ORC_SPHERE, ORC_CAPSULE, ORC_BOX, ORC_CAPSULE};
    const float shapes[K * 4] = {0.25f, 0.25f, 0.25f, 0.f, 0.1f, 0.1f, 0.1f, 0.3f, 0.3f, 0.2f, 0.1f, 0.f, 0.05f, 0.05f, 0.05f, 0.f};
    const float rgbs[K * 3] = {0.9f, 0.2f, 0.2f, 0.2f, 0.9f, 0.2f, 0.2f, 0.2f, 0.9f, 0.5f, 0.5f, 0.5f};
    const uint32_t nlon[K] = {16, 12, 4, 5}, nlat[K] = {8, 6, 0, 2};
    const float cam[9] = {60.f, -2.5f, 0.f, 1.f, 0.f, 0.f, 1.f, 0.1f, 50.f};
    const float light[5] = {-0.4f, -0.3f, 0.85f, 0.3f, 0.7f};
    const float ground[4] = {1.f, 0.7f, 0.35f, 0.65f};
    const float bg[3] = {0.55f, 0.7f, 0.9f};
    orc_scene* s = orc_scene_create(W, H, K, 0, kinds, shapes, rgbs, nlon, nlat, cam, light, ground, bg);
    if (!s) return 2;
    uint32_t V = 0, T = 0;
    orc_scene_counts(s, &V, &T);
    std::vector<float> poses((size_t)B * S * K * 7);
    uint32_t rng = 12345u;
    auto rnd = [&]() { rng = rng * 1664525u + 1013904223u; return (float)(rng >> 8) * (1.0f / 16777216.0f); };
    for (uint32_t f = 0; f < B * S; ++f)
        for (uint32_t b = 0; b < K; ++b) {
            float* p = &poses[((size_t)f * K + b) * 7];
            p[0] = rnd() - 0.5f; p[1] = rnd() - 0.5f; p[2] = 0.5f + rnd();
            float q[4] = {rnd() - 0.5f, rnd() - 0.5f, rnd() - 0.5f, rnd() - 0.5f};
            float n = std::sqrt(q[0] * q[0] + q[1] * q[1] + q[2] * q[2] + q[3] * q[3]) + 1e-6f;
            for (int i = 0; i < 4; ++i) p[3 + i] = q[i] / n;
        }
    // degenerate inputs: behind the camera, non-finite, straddling the near plane, huge coordinates
    poses[(1 * K + 1) * 7 + 0] = -6.0f;
    poses[(2 * K + 2) * 7 + 1] = NAN;
    poses[(3 * K + 3) * 7 + 0] = poses[(3 * K + 0) * 7 + 0] - 2.45f;
    poses[(3 * K + 3) * 7 + 2] = poses[(3 * K + 0) * 7 + 2] + 1.0f;
    poses[(4 * K + 1) * 7 + 1] = 1e9f;
    poses[(5 * K + 0) * 7 + 2] = -2.0f;
    std::vector<float> env_shapes((size_t)B * K * 4);
    for (uint32_t e = 0; e < B; ++e)
        for (uint32_t i = 0; i < K * 4; ++i) env_shapes[(size_t)e * K * 4 + i] = shapes[i] * (0.5f + rnd());
    std::vector<uint8_t> frames((size_t)B * S * W * H * 3), video((size_t)5 * W * H * 3);
    std::vector<uint32_t> ids((size_t)B * S * W * H), depth(ids.size()), order(T);
    for (auto& v : video) v = (uint8_t)(rnd() * 255.0f);
    for (uint32_t i = 0; i < T; ++i) order[i] = T - 1 - i;
    orc_distractor d{};
    if (orc_render(s, poses.data(), nullptr, B, S, 0, 0, nullptr, nullptr, frames.data(), ids.data(), depth.data())) return 3;
    d.mode = ORC_DIS_COLOR; d.seed = 0xDEADBEEFCAFEF00Dull; d.scale_lo = 0.5f; d.scale_hi = 1.5f; d.offset_lo = -0.2f; d.offset_hi = 0.2f;
    if (orc_render(s, poses.data(), env_shapes.data(), B, S, 0xFFFFFFF0u, 7, &d, order.data(), frames.data(), ids.data(), nullptr)) return 4;
    d.mode = ORC_DIS_VIDEO; d.video = video.data(); d.n_frames = 5; d.alpha = 0.5f;
    if (orc_render(s, poses.data(), env_shapes.data(), B, S, 3, 0xFFFFFFF0u, &d, nullptr, frames.data(), nullptr, depth.data())) return 5;
    std::vector<int32_t> X(V), Y(V);
    std::vector<float> D(V);
    std::vector<uint8_t> rej(V);
    std::vector<uint32_t> tris((size_t)T * 3), cover((size_t)W * H);
    orc_scene_mesh(s, nullptr, tris.data(), nullptr, nullptr, nullptr, nullptr);
    orc_vertex_stage(s, poses.data(), nullptr, X.data(), Y.data(), D.data(), rej.data(), nullptr);
    for (uint32_t cull = 0; cull < 3; ++cull)
        orc_raster(W, H, V, X.data(), Y.data(), D.data(), rej.data(), T, tris.data(), nullptr, cull, ids.data(), depth.data(), cover.data());
    uint32_t out[4];
    orc_philox(~0ull, ~0u, ~0u, ~0u, ~0u, out);
    unsigned long sum = 0;
    for (auto v : frames) sum += v;
    std::printf("ok %lu %u %u\n", sum, out[0], V + T);
    orc_scene_destroy(s);
    return 0;
}
