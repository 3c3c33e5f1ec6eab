// pxr_pipeline_*: renderer and frame consumer as one step, with the consumer of one part of the batch running
// beside the renderer of the next part.  The render kernel is bound by vector-ALU issue and hardly touches HBM;
// the conv layer is bound by HBM and leaves the vector units half idle: run back to back they leave each
// other's resource unused.  The batch is cut into chunks of environments; chunk c is rendered on the caller's
// stream, and as soon as it is done (an event) its conv layer is enqueued on a second stream of the same,
// default, priority, while the caller's stream goes on to render chunk c + 1.  Within one step nothing depends
// on anything but its own chunk, so the bytes are those of the serial order.

#include <hip/hip_runtime.h>

#include <new>

#include "pxr_internal.h"

struct pxr_pipeline {
    pxr_scene* scene = nullptr;
    pxr_conv* conv = nullptr;
    uint32_t n_chunks = 0;
    int device = 0;
    hipStream_t side = nullptr;
    hipEvent_t rendered[pxr::kMaxPipelineChunks] = {};
    hipEvent_t consumed = nullptr;
};

extern "C" {

int pxr_pipeline_create(pxr_scene* s, pxr_conv* c, uint32_t n_chunks, pxr_pipeline** out) {
    using pxr::set_error;
    if (!s || !c || !out) return set_error(PXR_ERR_INVALID_ARG, "pxr_pipeline_create: null argument");
    if (n_chunks < 1 || n_chunks > pxr::kMaxPipelineChunks)
        return set_error(PXR_ERR_INVALID_ARG, "pxr_pipeline_create: n_chunks must lie in [1,16]");
    uint32_t K, H, W, cH, cW, cS, Ho, Wo;
    pxr::scene_shape(s, &K, &H, &W);
    pxr::conv_shape(c, &cH, &cW, &cS, &Ho, &Wo);
    if (cH != H || cW != W) return set_error(PXR_ERR_INVALID_ARG, "pxr_pipeline_create: the layer's input size is not the scene's frame size");
    pxr_pipeline* p = new (std::nothrow) pxr_pipeline();
    if (!p) return set_error(PXR_ERR_OOM, "pxr_pipeline_create: host allocation failed");
    p->scene = s;
    p->conv = c;
    p->n_chunks = n_chunks;
    hipError_t rc = hipGetDevice(&p->device);
    // (default priority: streams of different priorities must not be mixed on these machines)
    if (rc == hipSuccess) rc = hipStreamCreateWithFlags(&p->side, hipStreamNonBlocking);
    for (uint32_t i = 0; rc == hipSuccess && i < n_chunks; ++i) rc = hipEventCreateWithFlags(&p->rendered[i], hipEventDisableTiming);
    if (rc == hipSuccess) rc = hipEventCreateWithFlags(&p->consumed, hipEventDisableTiming);
    if (rc != hipSuccess) {
        const std::string msg = std::string("pxr_pipeline_create: ") + hipGetErrorString(rc);
        (void)pxr_pipeline_destroy(p);
        return set_error(PXR_ERR_DEVICE, msg);
    }
    *out = p;
    return PXR_OK;
}

int pxr_pipeline_destroy(pxr_pipeline* p) {
    if (!p) return PXR_OK;
    hipError_t rc = hipSuccess;
    auto keep = [&rc](hipError_t r) {
        if (rc == hipSuccess) rc = r;
    };
    if (p->side) {
        keep(hipStreamSynchronize(p->side));
        keep(hipStreamDestroy(p->side));
    }
    for (hipEvent_t e : p->rendered)
        if (e) keep(hipEventDestroy(e));
    if (p->consumed) keep(hipEventDestroy(p->consumed));
    delete p;
    if (rc != hipSuccess) return pxr::set_error(PXR_ERR_DEVICE, std::string("pxr_pipeline_destroy: ") + hipGetErrorString(rc));
    return PXR_OK;
}

int pxr_pipeline_step(pxr_pipeline* p, const float* d_poses, const float* d_shapes, uint32_t B, uint32_t step0, uint32_t env0,
                      uint8_t* d_frames, uint16_t* d_features, void* hip_stream) {
    using pxr::set_error;
    if (!p || !d_poses || !d_frames || !d_features) return set_error(PXR_ERR_INVALID_ARG, "pxr_pipeline_step: null argument");
    if (B == 0) return set_error(PXR_ERR_INVALID_ARG, "pxr_pipeline_step: B must be positive");
    if ((uint64_t)env0 + B > 0x100000000ull) return set_error(PXR_ERR_INVALID_ARG, "pxr_pipeline_step: env0 + B overflows 32 bits");
    // (checked before anything is enqueued; chunks start at multiples of four environments and keep these alignments)
    if ((reinterpret_cast<uintptr_t>(d_poses) & 3u) || (reinterpret_cast<uintptr_t>(d_shapes) & 15u) ||
        (reinterpret_cast<uintptr_t>(d_frames) & 3u) || (reinterpret_cast<uintptr_t>(d_features) & 15u))
        return set_error(PXR_ERR_INVALID_ARG, "pxr_pipeline_step: poses/frames must be 4-byte and shapes/features 16-byte aligned");
    uint32_t K, H, W, cH, cW, S, Ho, Wo;
    pxr::scene_shape(p->scene, &K, &H, &W);
    pxr::conv_shape(p->conv, &cH, &cW, &S, &Ho, &Wo);
    hipStream_t main = reinterpret_cast<hipStream_t>(hip_stream);
    // chunks of whole multiples of four environments (every chunk's buffers keep the 16-byte alignment of the batch's)
    const uint32_t per = ((B + p->n_chunks - 1) / p->n_chunks + 3u) & ~3u;
    std::string err;
    uint32_t used = 0;
    for (uint32_t e0 = 0; e0 < B; e0 += per, ++used) {
        const uint32_t n = B - e0 < per ? B - e0 : per;
        int rc = pxr::render_envs(p->scene, d_poses, d_shapes, e0, n, S, step0, env0, d_frames, nullptr, main, err);
        if (rc != PXR_OK) return set_error(rc, "pxr_pipeline_step: " + err);
        hipError_t hrc = hipEventRecord(p->rendered[used], main);
        if (hrc == hipSuccess) hrc = hipStreamWaitEvent(p->side, p->rendered[used], 0);
        if (hrc != hipSuccess) return set_error(PXR_ERR_DEVICE, std::string("pxr_pipeline_step: ") + hipGetErrorString(hrc));
        rc = pxr::conv_envs(p->conv, d_frames, e0, n, d_features, p->side, err);
        if (rc != PXR_OK) return set_error(rc, "pxr_pipeline_step: " + err);
    }
    // join: whatever the caller enqueues next on its stream sees all features
    hipError_t hrc = hipEventRecord(p->consumed, p->side);
    if (hrc == hipSuccess) hrc = hipStreamWaitEvent(main, p->consumed, 0);
    if (hrc != hipSuccess) return set_error(PXR_ERR_DEVICE, std::string("pxr_pipeline_step: ") + hipGetErrorString(hrc));
    return PXR_OK;
}

}  // extern "C"
