// C ABI of libpxr (declared in include/pxr.h): argument checking, scene
// lifetime, distractor binding and the launch of the render kernel.

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstring>
#include <mutex>
#include <new>

#include "pxr_internal.h"

struct pxr_scene {
    pxr::SceneConsts sc{};
    pxr::DistractConsts dc{};
    void* d_arena = nullptr;
    pxr::SkeletonConsts sk{};
    void* d_skeleton = nullptr;
    int device = 0;
    uint32_t block_threads = 0;
    uint32_t default_threads = 0;
};

namespace {

thread_local std::string g_last_error;

int fail(int code, const std::string& msg) {
    g_last_error = msg;
    return code;
}

}  // namespace

int pxr::set_error(int code, const std::string& msg) { return fail(code, msg); }

void pxr::scene_shape(const pxr_scene* s, uint32_t* K, uint32_t* H, uint32_t* W) {
    *K = s->sc.K;
    *H = s->sc.H;
    *W = s->sc.W;
}

int pxr::render_envs(pxr_scene* s, const float* d_poses, const float* d_shapes, uint32_t e0, uint32_t n, uint32_t S,
                     uint32_t step0, uint32_t env0, uint8_t* d_frames, uint32_t* d_ids, void* stream, std::string& err) {
    if (n == 0 || S == 0 || (uint64_t)n * S > 0x7FFFFFFFull) {
        err = "B*S must lie in [1, 2^31-1]";
        return PXR_ERR_INVALID_ARG;
    }
    if ((uint64_t)step0 + S > 0x100000000ull || (uint64_t)env0 + e0 + n > 0x100000000ull) {
        err = "step0 + S or env0 + B overflows 32 bits";
        return PXR_ERR_INVALID_ARG;
    }
    const size_t K = s->sc.K, npix = s->sc.npix;
    const float* poses = d_poses + (size_t)e0 * S * K * 7;
    const float* shapes = d_shapes ? d_shapes + (size_t)e0 * K * 4 : nullptr;
    uint8_t* frames = d_frames + (size_t)e0 * S * npix * 3;
    uint32_t* ids = d_ids ? d_ids + (size_t)e0 * S * npix : nullptr;
    if ((reinterpret_cast<uintptr_t>(poses) & 3u) || (reinterpret_cast<uintptr_t>(shapes) & 15u) ||
        (reinterpret_cast<uintptr_t>(frames) & 3u) || (reinterpret_cast<uintptr_t>(ids) & 15u)) {
        err = "poses/frames must be 4-byte and shapes/ids 16-byte aligned";
        return PXR_ERR_INVALID_ARG;
    }
    pxr::DistractConsts dc = s->dc;  // the per-environment arrays follow the environments
    if (dc.env_offset) dc.env_offset += e0;
    if (dc.env_video) dc.env_video += e0;
    return pxr::launch_render(s->sc, dc, poses, shapes, n * S, S, step0, env0 + e0, frames, ids, s->block_threads, stream, err);
}

namespace {

uint32_t pick_block_threads(const pxr::SceneConsts& sc) {
    // Fill the 32 wave slots of a compute unit: LDS decides how many frame
    // workgroups are resident, the workgroup size makes up the rest.  (The
    // 1024-thread variant is compiled for 64 VGPRs so that two of them fit.)
    const uint32_t groups_per_cu = (160u * 1024u) / (sc.lds_total ? sc.lds_total : 1u);
    if (groups_per_cu >= 8) return 256;
    if (groups_per_cu >= 3) return 512;
    // the banded kernel variants need more than 64 registers: two groups of 768 threads then
    if (groups_per_cu == 2 && sc.band_rows < sc.H) return 768;
    return 1024;
}

// The kernels' dynamic-LDS caps are raised once per device and process, by the first scene created there.
int prepare_device_once(int device, std::string& err) {
    static std::mutex mu;
    static bool done[64] = {};
    if (device < 0 || device >= 64) return pxr::prepare_kernels(err);
    std::lock_guard<std::mutex> lock(mu);
    if (done[device]) return PXR_OK;
    const int rc = pxr::prepare_kernels(err);
    if (rc == PXR_OK) done[device] = true;
    return rc;
}

}  // namespace

extern "C" {

const char* pxr_last_error(void) { return g_last_error.c_str(); }

int pxr_create_scene(const pxr_scene_desc* desc, pxr_scene** out) {
    if (!desc || !out) return fail(PXR_ERR_INVALID_ARG, "pxr_create_scene: null argument");
    pxr::HostScene hs;
    std::string err;
    int rc = pxr::build_host_scene(*desc, hs, err);
    if (rc != PXR_OK) return fail(rc, "pxr_create_scene: " + err);

    // one arena, 256-byte aligned sub-tables, one synchronous upload
    struct Part {
        const void* src;
        size_t bytes;
        size_t off;
    };
    // The device copy of the pair table holds, in place of the four vertex indices, the LDS byte addresses of
    // the vertices' cell codes (the kernel reads them without any address arithmetic): code v sits at
    // lds_keys + 4 v of the dynamic LDS segment, which starts at address 0 (prepare_kernels checks that the
    // kernels have no static LDS in front of it).
    // It is padded to a multiple of 64 entries (a wavefront reads 64 without a bounds test) with entries that
    // hold no triangle and point four times at the word after the last code, which the kernel sets to code 0.
    if ((uint64_t)hs.c.lds_keys + 4ull * (hs.c.V + 1ull) > 0x10000ull)
        return fail(PXR_ERR_UNSUPPORTED, "pxr_create_scene: too many vertices for 16-bit LDS addresses in the pair table");

    pxr_scene* s = new (std::nothrow) pxr_scene();
    if (!s) return fail(PXR_ERR_OOM, "pxr_create_scene: host allocation failed");
    s->sc = hs.c;
    if (hipGetDevice(&s->device) != hipSuccess) {
        delete s;
        return fail(PXR_ERR_DEVICE, "pxr_create_scene: no HIP device");
    }
    std::vector<uint32_t> pair_dev(hs.pair_tbl);
    for (size_t p = 0; p < pair_dev.size() / 4; ++p)
        for (int w = 0; w < 2; ++w) {
            const uint32_t q = hs.pair_tbl[p * 4 + w];
            pair_dev[p * 4 + w] = (hs.c.lds_keys + 4u * (q & 0xFFFFu)) | ((hs.c.lds_keys + 4u * (q >> 16)) << 16);
        }
    const uint32_t zero_code_at = hs.c.lds_keys + 4u * hs.c.V;
    while ((pair_dev.size() / 4) % 64 != 0) {
        pair_dev.push_back(zero_code_at | (zero_code_at << 16));
        pair_dev.push_back(zero_code_at | (zero_code_at << 16));
        pair_dev.push_back(pxr::kNoTriangle | (pxr::kNoTriangle << 16));
        pair_dev.push_back(0u);
    }
    // Likewise the device copy of the vertex templates: its fourth word holds the LDS byte address of the body's
    // record, shifted left by 2, and the cap selector as a 2-bit two's-complement number (-1, 0, +1) below it, in
    // place of body << 2 | (selector + 1).
    std::vector<float> vtmpl_dev(hs.vtmpl);
    for (size_t v = 0; v < vtmpl_dev.size() / 4; ++v) {
        uint32_t code;
        std::memcpy(&code, &hs.vtmpl[v * 4 + 3], 4);
        const uint32_t body_at = hs.c.lds_body + (code >> 2) * pxr::kBodyStride * 4u, sel = ((code & 3u) - 1u) & 3u;
        const uint32_t dev = (body_at << 2) | sel;
        std::memcpy(&vtmpl_dev[v * 4 + 3], &dev, 4);
    }
    // Behind the bodies' constants: the rows (right, up, forward) of the view rotation and the light direction, for
    // the lanes of the kernel's set-up phase that take one row each.
    std::vector<float> body_dev(hs.body_const);
    for (const float* row : {hs.c.Rt, hs.c.Up, hs.c.Fw, hs.c.l}) body_dev.insert(body_dev.end(), row, row + 3);
    Part parts[6] = {{vtmpl_dev.data(), vtmpl_dev.size() * 4, 0},
                     {hs.tri_idx.data(), hs.tri_idx.size() * 4, 0},
                     {hs.tri_shade.data(), hs.tri_shade.size() * 4, 0},
                     {body_dev.data(), body_dev.size() * 4, 0},
                     {hs.cxcy.data(), hs.cxcy.size() * 4, 0},
                     {pair_dev.data(), pair_dev.size() * 4, 0}};
    size_t total = 0;
    for (Part& p : parts) {
        p.off = total;
        total += (p.bytes + 255) / 256 * 256;
    }
    std::vector<unsigned char> staging(total, 0);
    for (const Part& p : parts) std::memcpy(staging.data() + p.off, p.src, p.bytes);
    hipError_t hrc = hipMalloc(&s->d_arena, total);
    if (hrc != hipSuccess) {
        delete s;
        return fail(hrc == hipErrorOutOfMemory ? PXR_ERR_OOM : PXR_ERR_DEVICE,
                    std::string("pxr_create_scene: hipMalloc failed: ") + hipGetErrorString(hrc));
    }
    hrc = hipMemcpy(s->d_arena, staging.data(), total, hipMemcpyHostToDevice);
    if (hrc != hipSuccess) {
        (void)hipFree(s->d_arena);
        delete s;
        return fail(PXR_ERR_DEVICE, std::string("pxr_create_scene: upload failed: ") + hipGetErrorString(hrc));
    }
    const unsigned char* base = static_cast<const unsigned char*>(s->d_arena);
    s->sc.vtmpl = reinterpret_cast<const float*>(base + parts[0].off);
    s->sc.tri_idx = reinterpret_cast<const uint32_t*>(base + parts[1].off);
    s->sc.tri_shade = reinterpret_cast<const float*>(base + parts[2].off);
    s->sc.body_const = reinterpret_cast<const float*>(base + parts[3].off);
    s->sc.cxcy = reinterpret_cast<const float*>(base + parts[4].off);
    s->sc.pair_tbl = reinterpret_cast<const uint32_t*>(base + parts[5].off);
    s->sc.P = (uint32_t)(pair_dev.size() / 4);  // (with the padding)

    rc = prepare_device_once(s->device, err);
    if (rc != PXR_OK) {
        (void)hipFree(s->d_arena);
        delete s;
        return fail(rc, "pxr_create_scene: " + err);
    }
    s->default_threads = s->block_threads = pick_block_threads(s->sc);
    s->dc.mode = PXR_DISTRACT_NONE;
    *out = s;
    return PXR_OK;
}

int pxr_destroy_scene(pxr_scene* s) {
    if (!s) return PXR_OK;
    hipError_t hrc = hipFree(s->d_arena);
    if (s->d_skeleton) {
        const hipError_t hrc2 = hipFree(s->d_skeleton);
        if (hrc == hipSuccess) hrc = hrc2;
    }
    delete s;
    if (hrc != hipSuccess) return fail(PXR_ERR_DEVICE, std::string("pxr_destroy_scene: hipFree failed: ") + hipGetErrorString(hrc));
    return PXR_OK;
}

int pxr_apply_distractor(pxr_scene* s, const pxr_distractor_desc* d) {
    if (!s) return fail(PXR_ERR_INVALID_ARG, "pxr_apply_distractor: null scene");
    pxr::DistractConsts dc{};
    dc.mode = PXR_DISTRACT_NONE;
    if (d && d->mode != PXR_DISTRACT_NONE) {
        dc.seed_lo = (uint32_t)d->seed;
        dc.seed_hi = (uint32_t)(d->seed >> 32);
        if (d->mode == PXR_DISTRACT_COLOR) {
            if (!std::isfinite(d->scale_lo) || !std::isfinite(d->scale_hi) || !std::isfinite(d->offset_lo) ||
                !std::isfinite(d->offset_hi))
                return fail(PXR_ERR_INVALID_ARG, "pxr_apply_distractor: non-finite colour range");
            dc.mode = PXR_DISTRACT_COLOR;
            dc.scale_lo = d->scale_lo;
            dc.scale_span = d->scale_hi - d->scale_lo;
            dc.offset_lo = d->offset_lo;
            dc.offset_span = d->offset_hi - d->offset_lo;
        } else if (d->mode == PXR_DISTRACT_VIDEO) {
            if (!d->d_video || d->n_frames == 0)
                return fail(PXR_ERR_INVALID_ARG, "pxr_apply_distractor: video mode needs d_video and n_frames > 0");
            if (!(d->alpha >= 0.0f && d->alpha <= 1.0f))
                return fail(PXR_ERR_INVALID_ARG, "pxr_apply_distractor: alpha must lie in [0,1]");
            if ((reinterpret_cast<uintptr_t>(d->d_video) & 3u) || (reinterpret_cast<uintptr_t>(d->d_env_offset) & 3u) ||
                (reinterpret_cast<uintptr_t>(d->d_env_video) & 3u))
                return fail(PXR_ERR_INVALID_ARG, "pxr_apply_distractor: d_video, d_env_offset and d_env_video must be 4-byte aligned");
            if ((uint64_t)(d->n_videos ? d->n_videos : 1u) * d->n_frames > 0xFFFFFFFFull)
                return fail(PXR_ERR_INVALID_ARG, "pxr_apply_distractor: n_videos * n_frames overflows 32 bits");
            dc.mode = PXR_DISTRACT_VIDEO;
            dc.video = d->d_video;
            dc.n_frames = d->n_frames;
            dc.alpha = d->alpha;
            dc.env_offset = d->d_env_offset;
            dc.n_videos = d->n_videos ? d->n_videos : 1u;
            dc.env_video = dc.n_videos > 1 ? d->d_env_video : nullptr;
        } else {
            return fail(PXR_ERR_INVALID_ARG, "pxr_apply_distractor: unknown mode");
        }
    }
    s->dc = dc;
    return PXR_OK;
}

int pxr_render_batch(pxr_scene* s, const float* d_poses, const float* d_shapes, uint32_t B, uint32_t S, uint32_t step0,
                     uint32_t env0, uint8_t* d_frames, uint32_t* d_ids, void* hip_stream) {
    if (!s || !d_poses || !d_frames) return fail(PXR_ERR_INVALID_ARG, "pxr_render_batch: null scene, poses or frames");
    std::string err;
    const int rc = pxr::render_envs(s, d_poses, d_shapes, 0, B, S, step0, env0, d_frames, d_ids, hip_stream, err);
    if (rc != PXR_OK) return fail(rc, "pxr_render_batch: " + err);
    return PXR_OK;
}

int pxr_set_skeleton(pxr_scene* s, const pxr_skeleton_desc* k) {
    if (!s) return fail(PXR_ERR_INVALID_ARG, "pxr_set_skeleton: null scene");
    if (!k) {
        if (s->d_skeleton) (void)hipFree(s->d_skeleton);
        s->d_skeleton = nullptr;
        s->sk = pxr::SkeletonConsts{};
        return PXR_OK;
    }
    if (!k->parent || !k->slot || !k->anchor || !k->axis || !k->offset)
        return fail(PXR_ERR_INVALID_ARG, "pxr_set_skeleton: null array");
    const uint32_t K = s->sc.K;
    if (k->n_bodies != K) return fail(PXR_ERR_INVALID_ARG, "pxr_set_skeleton: n_bodies differs from the scene's");
    for (uint32_t b = 0; b < K; ++b) {
        const int32_t p = k->parent[b], sl = k->slot[b];
        if (p < 0) {
            if (sl < 0 || (uint32_t)sl >= k->n_free)
                return fail(PXR_ERR_INVALID_ARG, "pxr_set_skeleton: a free body needs a slot in [0, n_free)");
        } else {
            if ((uint32_t)p >= b) return fail(PXR_ERR_INVALID_ARG, "pxr_set_skeleton: a parent must precede its child");
            if (sl < -1 || (sl >= 0 && (uint32_t)sl >= k->n_angles))
                return fail(PXR_ERR_INVALID_ARG, "pxr_set_skeleton: hinge slot outside [-1, n_angles)");
        }
        for (int c = 0; c < 3; ++c)
            if (!std::isfinite(k->anchor[b * 3 + c]) || !std::isfinite(k->axis[b * 3 + c]) ||
                !std::isfinite(k->offset[b * 3 + c]))
                return fail(PXR_ERR_INVALID_ARG, "pxr_set_skeleton: non-finite anchor, axis or offset");
    }
    pxr::SkeletonConsts sk{};
    sk.K = K;
    sk.J = k->n_angles;
    sk.F = k->n_free;
    if ((uint64_t)sk.J + 7ull * sk.F + 7ull * K > 630ull || pxr::fk_lds_bytes(sk) > 160u * 1024u)
        return fail(PXR_ERR_UNSUPPORTED, "pxr_set_skeleton: 64 frames of this skeleton do not fit 160 KB of LDS");
    // one allocation: parent[K], slot[K], hinge[K][9]
    std::vector<uint32_t> staging((size_t)K * 11);
    for (uint32_t b = 0; b < K; ++b) {
        staging[b] = (uint32_t)k->parent[b];
        staging[K + b] = (uint32_t)k->slot[b];
        float h[9];
        for (int c = 0; c < 3; ++c) {
            h[c] = k->anchor[b * 3 + c];
            h[3 + c] = k->axis[b * 3 + c];
            h[6 + c] = k->offset[b * 3 + c];
        }
        std::memcpy(&staging[2 * (size_t)K + (size_t)b * 9], h, sizeof(h));
    }
    std::string err;
    int rc = pxr::prepare_fk_kernel(err);
    if (rc != PXR_OK) return fail(rc, "pxr_set_skeleton: " + err);
    void* d = nullptr;
    hipError_t hrc = hipMalloc(&d, staging.size() * 4);
    if (hrc != hipSuccess)
        return fail(hrc == hipErrorOutOfMemory ? PXR_ERR_OOM : PXR_ERR_DEVICE,
                    std::string("pxr_set_skeleton: hipMalloc failed: ") + hipGetErrorString(hrc));
    hrc = hipMemcpy(d, staging.data(), staging.size() * 4, hipMemcpyHostToDevice);
    if (hrc != hipSuccess) {
        (void)hipFree(d);
        return fail(PXR_ERR_DEVICE, std::string("pxr_set_skeleton: upload failed: ") + hipGetErrorString(hrc));
    }
    {
        // set-up is the place to look up this device's copy of the static pose buffer (used by
        // pxr_render_batch_kinematic_static), so that the hot call finds it cached
        float* unused = nullptr;
        std::string e2;
        (void)pxr::static_pose_scratch(&unused, nullptr, e2);
    }
    if (s->d_skeleton) (void)hipFree(s->d_skeleton);
    s->d_skeleton = d;
    sk.parent = static_cast<const int32_t*>(d);
    sk.slot = sk.parent + K;
    sk.hinge = reinterpret_cast<const float*>(sk.slot + K);
    s->sk = sk;
    return PXR_OK;
}

int pxr_pose_batch(pxr_scene* s, const float* d_free_poses, const float* d_angles, uint32_t n_frames, float* d_poses,
                   void* hip_stream) {
    if (!s) return fail(PXR_ERR_INVALID_ARG, "pxr_pose_batch: null scene");
    if (!s->d_skeleton) return fail(PXR_ERR_INVALID_ARG, "pxr_pose_batch: no skeleton bound (pxr_set_skeleton)");
    if (n_frames == 0 || n_frames > 0x7FFFFFFFu) return fail(PXR_ERR_INVALID_ARG, "pxr_pose_batch: n_frames must lie in [1, 2^31-1]");
    if (!d_poses || (s->sk.F && !d_free_poses) || (s->sk.J && !d_angles))
        return fail(PXR_ERR_INVALID_ARG, "pxr_pose_batch: null buffer");
    if ((reinterpret_cast<uintptr_t>(d_free_poses) & 3u) || (reinterpret_cast<uintptr_t>(d_angles) & 3u) ||
        (reinterpret_cast<uintptr_t>(d_poses) & 3u))
        return fail(PXR_ERR_INVALID_ARG, "pxr_pose_batch: buffers must be 4-byte aligned");
    std::string err;
    const int rc = pxr::launch_fk(s->sk, d_free_poses, d_angles, n_frames, d_poses, hip_stream, err);
    if (rc != PXR_OK) return fail(rc, "pxr_pose_batch: " + err);
    return PXR_OK;
}

int pxr_render_batch_kinematic(pxr_scene* s, const float* d_free_poses, const float* d_angles, const float* d_shapes,
                               uint32_t B, uint32_t S, uint32_t step0, uint32_t env0, float* d_poses, uint8_t* d_frames,
                               uint32_t* d_ids, void* hip_stream) {
    if (B == 0 || S == 0 || (uint64_t)B * S > 0x7FFFFFFFull)
        return fail(PXR_ERR_INVALID_ARG, "pxr_render_batch_kinematic: B*S must lie in [1, 2^31-1]");
    if (!d_frames) return fail(PXR_ERR_INVALID_ARG, "pxr_render_batch_kinematic: null frames");
    int rc = pxr_pose_batch(s, d_free_poses, d_angles, B * S, d_poses, hip_stream);
    if (rc != PXR_OK) return rc;
    return pxr_render_batch(s, d_poses, d_shapes, B, S, step0, env0, d_frames, d_ids, hip_stream);
}

int pxr_render_batch_kinematic_static(pxr_scene* s, const float* d_free_poses, const float* d_angles,
                                      const float* d_shapes, uint32_t B, uint32_t S, uint32_t step0, uint32_t env0,
                                      uint8_t* d_frames, uint32_t* d_ids, void* hip_stream) {
    if (!s) return fail(PXR_ERR_INVALID_ARG, "pxr_render_batch_kinematic_static: null scene");
    if (B == 0 || S == 0 || (uint64_t)B * S > 0x7FFFFFFFull)
        return fail(PXR_ERR_INVALID_ARG, "pxr_render_batch_kinematic_static: B*S must lie in [1, 2^31-1]");
    if (!d_frames) return fail(PXR_ERR_INVALID_ARG, "pxr_render_batch_kinematic_static: null frames");
    float* d_poses = nullptr;
    size_t capacity = 0;
    std::string err;
    int device = -1;
    if (hipGetDevice(&device) != hipSuccess || device != s->device)
        return fail(PXR_ERR_INVALID_ARG, "pxr_render_batch_kinematic_static: the scene's device must be the current one");
    const int rc = pxr::static_pose_scratch(&d_poses, &capacity, err);
    if (rc != PXR_OK) return fail(rc, "pxr_render_batch_kinematic_static: " + err);
    const uint64_t need = (uint64_t)B * S * s->sc.K * 7ull * sizeof(float);
    if (need > capacity)
        return fail(PXR_ERR_UNSUPPORTED, "pxr_render_batch_kinematic_static: B*S*n_bodies*28 = " + std::to_string(need) +
                                             " bytes of poses exceed the library's " + std::to_string(capacity) +
                                             "-byte static buffer; use pxr_render_batch_kinematic with a buffer of your own");
    // (every pose the render kernel reads is written by the kinematics kernel in front of it on the same stream:
    // nothing of an earlier call's contents is used, so nothing needs clearing)
    return pxr_render_batch_kinematic(s, d_free_poses, d_angles, d_shapes, B, S, step0, env0, d_poses, d_frames, d_ids,
                                      hip_stream);
}

int pxr_scene_info(const pxr_scene* s, uint32_t* n_verts, uint32_t* n_tris, uint32_t* lds_bytes, uint32_t* block_threads) {
    if (!s) return fail(PXR_ERR_INVALID_ARG, "pxr_scene_info: null scene");
    if (n_verts) *n_verts = s->sc.V;
    if (n_tris) *n_tris = s->sc.T;
    if (lds_bytes) *lds_bytes = s->sc.lds_total;
    if (block_threads) *block_threads = s->block_threads;
    return PXR_OK;
}

int pxr_host_tables(const pxr_scene_desc* desc, uint32_t* n_verts, uint32_t* n_tris, float* vtmpl, uint32_t* tri_idx,
                    float* tri_shade, float* cxcy, float* consts, uint32_t* n_pairs, uint32_t* pair_tbl) {
    if (!desc) return fail(PXR_ERR_INVALID_ARG, "pxr_host_tables: null desc");
    pxr::HostScene hs;
    std::string err;
    const int rc = pxr::build_host_scene(*desc, hs, err);
    if (rc != PXR_OK) return fail(rc, "pxr_host_tables: " + err);
    if (n_verts) *n_verts = hs.c.V;
    if (n_tris) *n_tris = hs.c.T;
    if (vtmpl) std::memcpy(vtmpl, hs.vtmpl.data(), hs.vtmpl.size() * 4);
    if (tri_idx) std::memcpy(tri_idx, hs.tri_idx.data(), hs.tri_idx.size() * 4);
    if (tri_shade) std::memcpy(tri_shade, hs.tri_shade.data(), hs.tri_shade.size() * 4);
    if (cxcy) std::memcpy(cxcy, hs.cxcy.data(), hs.cxcy.size() * 4);
    if (n_pairs) *n_pairs = hs.c.P;
    if (pair_tbl)
        for (uint32_t p = 0; p < hs.c.P; ++p)
            for (int w = 0; w < 3; ++w) pair_tbl[p * 3 + w] = hs.pair_tbl[p * 4 + w];
    if (consts) {
        for (int i = 0; i < 3; ++i) {
            consts[i] = hs.c.Rt[i];
            consts[3 + i] = hs.c.Up[i];
            consts[6 + i] = hs.c.Fw[i];
            consts[12 + i] = hs.c.l[i];
        }
        consts[9] = hs.c.f;
        consts[10] = hs.c.gs[0];
        consts[11] = hs.c.gs[1];
        consts[15] = (float)hs.c.lds_total;
    }
    return PXR_OK;
}

int pxr_selftest_arithmetic(uint64_t* counts) {
    if (!counts) return fail(PXR_ERR_INVALID_ARG, "pxr_selftest_arithmetic: null output");
    std::string err;
    unsigned long long c[4] = {0, 0, 0, 0};
    const int rc = pxr::selftest_arithmetic(c, err);
    if (rc != PXR_OK) return fail(rc, "pxr_selftest_arithmetic: " + err);
    for (int i = 0; i < 4; ++i) counts[i] = c[i];
    return PXR_OK;
}

int pxr_measure_peaks(double* fma_tlaneops, double* imad_tlaneops, double* copy_gbs, double* read_gbs, double* write_gbs) {
    std::string err;
    const int rc = pxr::measure_peaks(fma_tlaneops, imad_tlaneops, copy_gbs, read_gbs, write_gbs, err);
    if (rc != PXR_OK) return fail(rc, "pxr_measure_peaks: " + err);
    return PXR_OK;
}

int pxr_set_block_threads(pxr_scene* s, uint32_t threads) {
    if (!s) return fail(PXR_ERR_INVALID_ARG, "pxr_set_block_threads: null scene");
    if (threads == 0) threads = s->default_threads;
    if (threads != 256 && threads != 512 && threads != 768 && threads != 1024)
        return fail(PXR_ERR_INVALID_ARG, "pxr_set_block_threads: must be 256, 512, 768 or 1024");
    s->block_threads = threads;
    return PXR_OK;
}

}  // extern "C"
