// Measured-peak microbenchmarks of libpxr (pxr_measure_peaks): what this GPU
// sustains on dependent-free fp32 FMA, on 24-bit integer multiply-add and on a
// plain device-to-device copy, so that a roofline fraction can be quoted
// against the machine as it runs and not only against its data sheet.  Not on
// the hot path; nothing else in the library uses these kernels.

#include <hip/hip_runtime.h>

#include "pxr_internal.h"

namespace pxr {
namespace {

constexpr int kChains = 8;  // independent accumulators per lane: enough to cover the VALU latency

__global__ __launch_bounds__(256) void fma_rate_kernel(float* sink, uint32_t iters, float a, float b) {
    float x[kChains];
#pragma unroll
    for (int c = 0; c < kChains; ++c) x[c] = (float)(threadIdx.x + c);
    for (uint32_t i = 0; i < iters; ++i) {
#pragma unroll
        for (int c = 0; c < kChains; ++c) x[c] = __builtin_fmaf(x[c], a, b);
    }
    float s = 0.0f;
#pragma unroll
    for (int c = 0; c < kChains; ++c) s += x[c];
    if (s == 12345.678f) sink[0] = s;  // keeps the loop alive, never true in practice
}

__global__ __launch_bounds__(256) void imad_rate_kernel(uint32_t* sink, uint32_t iters, uint32_t a, uint32_t b) {
    uint32_t x[kChains];
#pragma unroll
    for (int c = 0; c < kChains; ++c) x[c] = threadIdx.x + c;
    for (uint32_t i = 0; i < iters; ++i) {
#pragma unroll
        for (int c = 0; c < kChains; ++c) x[c] = __umul24(x[c], a) + b;
    }
    uint32_t s = 0;
#pragma unroll
    for (int c = 0; c < kChains; ++c) s ^= x[c];
    if (s == 0xDEADBEEFu) sink[0] = s;
}

__global__ __launch_bounds__(256) void copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

// read-only and write-only streams: HBM does not give both directions the same rate
__global__ __launch_bounds__(256) void read_kernel(const uint4* __restrict__ src, uint4* __restrict__ sink, size_t n) {
    uint4 acc = make_uint4(0, 0, 0, 0);
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
        const uint4 v = src[i];
        acc.x ^= v.x;
        acc.y ^= v.y;
        acc.z ^= v.z;
        acc.w ^= v.w;
    }
    if (acc.x == 0x12345678u && acc.y == 0x9ABCDEF0u) sink[0] = acc;  // keeps the loads alive
}

__global__ __launch_bounds__(256) void write_kernel(uint4* __restrict__ dst, size_t n) {
    const uint4 v = make_uint4(threadIdx.x, 2u, 3u, 4u);
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) dst[i] = v;
}

template <typename F>
int timed(hipStream_t st, int reps, F launch, double& seconds, std::string& err) {
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) {
        err = "hipEventCreate failed";
        return PXR_ERR_DEVICE;
    }
    launch();  // warm-up
    (void)hipEventRecord(e0, st);
    for (int r = 0; r < reps; ++r) launch();
    (void)hipEventRecord(e1, st);
    hipError_t rc = hipEventSynchronize(e1);
    float ms = 0.0f;
    if (rc == hipSuccess) rc = hipEventElapsedTime(&ms, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc != hipSuccess || hipGetLastError() != hipSuccess) {
        err = std::string("timing failed: ") + hipGetErrorString(rc);
        return PXR_ERR_DEVICE;
    }
    seconds = 1e-3 * ms / reps;
    return PXR_OK;
}

}  // namespace

int measure_peaks(double* fma_tlaneops, double* imad_tlaneops, double* copy_gbs, double* read_gbs, double* write_gbs,
                  std::string& err) {
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) {
        err = "no HIP device";
        return PXR_ERR_DEVICE;
    }
    const uint32_t blocks = (uint32_t)prop.multiProcessorCount * 8u, iters = 4096;  // 32 waves per compute unit
    const size_t copy_bytes = (size_t)1 << 30;
    void* buf = nullptr;
    if (hipMalloc(&buf, 2 * copy_bytes) != hipSuccess) {
        err = "hipMalloc of the 2 GiB copy buffers failed";
        return PXR_ERR_OOM;
    }
    if (hipMemset(buf, 1, 2 * copy_bytes) != hipSuccess) {
        (void)hipFree(buf);
        err = "hipMemset failed";
        return PXR_ERR_DEVICE;
    }
    hipStream_t st = nullptr;
    double t = 0.0;
    int rc = timed(st, 5, [&] { hipLaunchKernelGGL(fma_rate_kernel, dim3(blocks), dim3(256), 0, st, (float*)buf, iters, 0.999f, 0.001f); }, t, err);
    const double lane_ops = (double)blocks * 256.0 * iters * kChains;
    if (rc == PXR_OK && fma_tlaneops) *fma_tlaneops = lane_ops / t / 1e12;
    if (rc == PXR_OK)
        rc = timed(st, 5, [&] { hipLaunchKernelGGL(imad_rate_kernel, dim3(blocks), dim3(256), 0, st, (uint32_t*)buf, iters, 3u, 7u); }, t, err);
    if (rc == PXR_OK && imad_tlaneops) *imad_tlaneops = lane_ops / t / 1e12;
    if (rc == PXR_OK)
        rc = timed(st, 5, [&] {
            hipLaunchKernelGGL(copy_kernel, dim3((uint32_t)prop.multiProcessorCount * 16u), dim3(256), 0, st, (const uint4*)buf,
                               (uint4*)((char*)buf + copy_bytes), copy_bytes / 16);
        }, t, err);
    if (rc == PXR_OK && copy_gbs) *copy_gbs = 2.0 * (double)copy_bytes / t / 1e9;  // bytes read + bytes written
    const uint32_t stream_blocks = (uint32_t)prop.multiProcessorCount * 8u;
    if (rc == PXR_OK)
        rc = timed(st, 5, [&] {
            hipLaunchKernelGGL(read_kernel, dim3(stream_blocks), dim3(256), 0, st, (const uint4*)buf, (uint4*)buf, 2 * copy_bytes / 16);
        }, t, err);
    if (rc == PXR_OK && read_gbs) *read_gbs = 2.0 * (double)copy_bytes / t / 1e9;
    if (rc == PXR_OK)
        rc = timed(st, 5, [&] { hipLaunchKernelGGL(write_kernel, dim3(stream_blocks), dim3(256), 0, st, (uint4*)buf, 2 * copy_bytes / 16); },
                   t, err);
    if (rc == PXR_OK && write_gbs) *write_gbs = 2.0 * (double)copy_bytes / t / 1e9;
    (void)hipFree(buf);
    return rc;
}

}  // namespace pxr
