// Producer stage of libpxr: joint angles -> rigid-body poses on the device, so
// that the renderer's input never has to come from the host (PixelBrax, arXiv
// 2502.00021, section 1: the whole loop, environment step included, stays on
// the accelerator).  gfx950 only.
//
// One lane per frame.  A frame's kinematic tree is a serial chain of
// dependent quaternion products, so the parallel axis is the batch: 64 frames
// per wavefront, every lane walking the same skeleton in lock-step (the
// skeleton tables are wave-uniform and arrive through scalar loads).  The
// poses of a workgroup's 64 frames live in LDS as pose[k][component][lane]
// (row stride 65 floats: conflict-free both for the per-lane walk and for the
// transposed, fully coalesced copy to HBM at the end).
//
// Arithmetic: fp32, explicit fmaf, no contraction.  sin and cos of half the
// hinge angle come from a two-constant Cody-Waite reduction by pi/2 and two
// Taylor polynomials (within 1.25 * 2^-24 of the true values for hinge angles
// up to +-65536 rad); an angle beyond that, or a non-finite one, gives NaN for
// both, so the body and its descendants drop out of the frame.

#include <hip/hip_runtime.h>

#include "pxr_internal.h"

namespace pxr {
namespace {

constexpr uint32_t kFkLanes = 64;            // frames per workgroup (one wavefront)
constexpr uint32_t kFkStride = kFkLanes + 1; // LDS row stride in floats
constexpr uint32_t kFkBatch = 16;            // memory requests a lane has in flight per array in the copy stages

constexpr float kMaxHingeAngle = 65536.0f;  // radians; the reduction below is accurate up to here

__device__ __forceinline__ void sincos_half(float theta, float& s, float& c) {
    const float h = 0.5f * theta;
    const float kf = __builtin_rintf(h * 0.636619772f);  // nearest multiple of pi/2, ties to even
    float r = __builtin_fmaf(kf, -1.57079625f, h);
    r = __builtin_fmaf(kf, -7.54978942e-08f, r);
    const float r2 = r * r;
    float ps = __builtin_fmaf(r2, 2.75573192e-06f, -1.98412698e-04f);
    ps = __builtin_fmaf(ps, r2, 8.33333333e-03f);
    ps = __builtin_fmaf(ps, r2, -1.66666667e-01f);
    const float sp = __builtin_fmaf(r * r2, ps, r);
    float pc = __builtin_fmaf(r2, -2.75573192e-07f, 2.48015873e-05f);
    pc = __builtin_fmaf(pc, r2, -1.38888889e-03f);
    pc = __builtin_fmaf(pc, r2, 4.16666667e-02f);
    pc = __builtin_fmaf(pc, r2, -0.5f);
    const float cp = __builtin_fmaf(pc, r2, 1.0f);
    const int q = (int)kf & 3;  // (|kf| < 2^15 inside the domain)
    s = q == 0 ? sp : (q == 1 ? cp : (q == 2 ? -sp : -cp));
    c = q == 0 ? cp : (q == 1 ? -sp : (q == 2 ? -cp : sp));
    if (!(__builtin_fabsf(theta) <= kMaxHingeAngle)) s = c = __builtin_nanf("");
}

// Row r of the rotation matrix of quaternion (w,x,y,z) applied to v, as
// fma(m0, v0, fma(m1, v1, m2 * v2)); same matrix formulas as the renderer's
// vertex stage.
__device__ __forceinline__ void rotate(float w, float x, float y, float z, float v0, float v1, float v2, float out[3]) {
    const float m00 = 1.0f - 2.0f * (y * y + z * z), m01 = 2.0f * (x * y - w * z), m02 = 2.0f * (x * z + w * y);
    const float m10 = 2.0f * (x * y + w * z), m11 = 1.0f - 2.0f * (x * x + z * z), m12 = 2.0f * (y * z - w * x);
    const float m20 = 2.0f * (x * z - w * y), m21 = 2.0f * (y * z + w * x), m22 = 1.0f - 2.0f * (x * x + y * y);
    out[0] = __builtin_fmaf(m00, v0, __builtin_fmaf(m01, v1, m02 * v2));
    out[1] = __builtin_fmaf(m10, v0, __builtin_fmaf(m11, v1, m12 * v2));
    out[2] = __builtin_fmaf(m20, v0, __builtin_fmaf(m21, v1, m22 * v2));
}

__global__ __launch_bounds__(kFkLanes) void fk_kernel(const SkeletonConsts sk, const float* __restrict__ free_poses,
                                                      const float* __restrict__ angles, uint32_t n_frames,
                                                      float* __restrict__ poses) {
    extern __shared__ __align__(16) unsigned char lds[];
    float* pose = reinterpret_cast<float*>(lds);              // [K*7][kFkStride]
    float* ang = pose + (size_t)sk.K * 7 * kFkStride;         // [J][kFkStride]
    float* fre = ang + (size_t)sk.J * kFkStride;              // [F*7][kFkStride]

    const uint32_t lane = threadIdx.x;
    const uint32_t f0 = blockIdx.x * kFkLanes;                // first frame of this workgroup
    const uint32_t nf = min(kFkLanes, n_frames - f0);         // frames it holds (ragged tail)

    // Coalesced loads of the workgroup's contiguous input chunks, transposed into LDS.  A batch of requests goes out
    // before the first answer is used: one request per trip, each waited for, made this stage a chain of two dozen
    // memory round trips, which was most of the kernel's time.  (Lanes past the end of a chunk ask for its last
    // element again and drop the answer; index / row length by multiplication: indices stay below 64 * row length,
    // far inside the exact range.)
    {
        const uint32_t row_f = sk.F * 7;
        const uint32_t n_a = nf * sk.J, n_f = nf * row_f;
        const float* src_a = angles + (size_t)f0 * sk.J;
        const float* src_f = free_poses + (size_t)f0 * row_f;
        const uint32_t magic_j = sk.J > 1u ? 0xFFFFFFFFu / sk.J + 1u : 0u;  // (ceil(2^32 / J); J == 1 needs none)
        const uint32_t magic_f = row_f ? 0xFFFFFFFFu / row_f + 1u : 0u;     // (rows are multiples of 7)
        for (uint32_t base = 0; base < max(n_a, n_f); base += kFkLanes * kFkBatch) {
            float ta[kFkBatch], tf[kFkBatch];
            if (base < n_a) {
#pragma unroll
                for (uint32_t u = 0; u < kFkBatch; ++u) ta[u] = src_a[min(base + u * kFkLanes + lane, n_a - 1u)];
            }
            if (base < n_f) {
#pragma unroll
                for (uint32_t u = 0; u < kFkBatch; ++u) tf[u] = src_f[min(base + u * kFkLanes + lane, n_f - 1u)];
            }
            if (base < n_a) {
#pragma unroll
                for (uint32_t u = 0; u < kFkBatch; ++u) {
                    const uint32_t i = base + u * kFkLanes + lane;
                    const uint32_t n = sk.J > 1u ? __umulhi(i, magic_j) : i, j = i - n * sk.J;
                    if (i < n_a) ang[j * kFkStride + n] = ta[u];
                }
            }
            if (base < n_f) {
#pragma unroll
                for (uint32_t u = 0; u < kFkBatch; ++u) {
                    const uint32_t i = base + u * kFkLanes + lane;
                    const uint32_t n = __umulhi(i, magic_f), j = i - n * row_f;
                    if (i < n_f) fre[j * kFkStride + n] = tf[u];
                }
            }
        }
    }
    __syncthreads();

    if (lane < nf) {
        for (uint32_t k = 0; k < sk.K; ++k) {
            const int parent = sk.parent[k], slot = sk.slot[k];   // wave-uniform
            float* o = pose + (size_t)k * 7 * kFkStride + lane;
            if (parent < 0) {
                const float* src = fre + (size_t)slot * 7 * kFkStride + lane;
#pragma unroll
                for (int c = 0; c < 7; ++c) o[c * kFkStride] = src[c * kFkStride];
                continue;
            }
            const float* pp = pose + (size_t)parent * 7 * kFkStride + lane;
            const float ppx = pp[0], ppy = pp[kFkStride], ppz = pp[2 * kFkStride];
            const float pw = pp[3 * kFkStride], px = pp[4 * kFkStride], py = pp[5 * kFkStride], pz = pp[6 * kFkStride];
            const float theta = slot >= 0 ? ang[(size_t)slot * kFkStride + lane] : 0.0f;
            float sn, cs;
            sincos_half(theta, sn, cs);
            const float* tb = sk.hinge + (size_t)k * 9;           // anchor, axis, offset
            const float jw = cs, jx = sn * tb[3], jy = sn * tb[4], jz = sn * tb[5];
            // body orientation = parent orientation (x) hinge rotation (Hamilton product)
            const float qw = __builtin_fmaf(-pz, jz, __builtin_fmaf(-py, jy, __builtin_fmaf(-px, jx, pw * jw)));
            const float qx = __builtin_fmaf(py, jz, __builtin_fmaf(-pz, jy, __builtin_fmaf(px, jw, pw * jx)));
            const float qy = __builtin_fmaf(pz, jx, __builtin_fmaf(-px, jz, __builtin_fmaf(py, jw, pw * jy)));
            const float qz = __builtin_fmaf(px, jy, __builtin_fmaf(-py, jx, __builtin_fmaf(pz, jw, pw * jz)));
            float t1[3], t2[3];
            rotate(pw, px, py, pz, tb[0], tb[1], tb[2], t1);      // hinge position, parent frame -> world
            rotate(qw, qx, qy, qz, tb[6], tb[7], tb[8], t2);      // body centre relative to the hinge
            o[0] = (ppx + t1[0]) + t2[0];
            o[kFkStride] = (ppy + t1[1]) + t2[1];
            o[2 * kFkStride] = (ppz + t1[2]) + t2[2];
            o[3 * kFkStride] = qw;
            o[4 * kFkStride] = qx;
            o[5 * kFkStride] = qy;
            o[6 * kFkStride] = qz;
        }
    }
    __syncthreads();

    // coalesced store of the workgroup's contiguous output chunk (a batch of LDS reads, then the batch's stores)
    {
        const uint32_t row = sk.K * 7, n_o = nf * row;
        const uint32_t magic = 0xFFFFFFFFu / row + 1u;
        float* dst = poses + (size_t)f0 * row;
        for (uint32_t base = 0; base < n_o; base += kFkLanes * kFkBatch) {
            float t[kFkBatch];
#pragma unroll
            for (uint32_t u = 0; u < kFkBatch; ++u) {
                const uint32_t i = min(base + u * kFkLanes + lane, n_o - 1u);
                const uint32_t n = __umulhi(i, magic), j = i - n * row;
                t[u] = pose[j * kFkStride + n];
            }
#pragma unroll
            for (uint32_t u = 0; u < kFkBatch; ++u) {
                const uint32_t i = base + u * kFkLanes + lane;
                if (i < n_o) dst[i] = t[u];
            }
        }
    }
}

}  // namespace

uint32_t fk_lds_bytes(const SkeletonConsts& sk) { return (sk.K * 7 + sk.J + sk.F * 7) * kFkStride * 4u; }

int prepare_fk_kernel(std::string& err) {
    const hipError_t rc = hipFuncSetAttribute(reinterpret_cast<const void*>(&fk_kernel),
                                              hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (rc != hipSuccess) {
        err = std::string("hipFuncSetAttribute(MaxDynamicSharedMemorySize) failed: ") + hipGetErrorString(rc);
        return PXR_ERR_DEVICE;
    }
    return PXR_OK;
}

int launch_fk(const SkeletonConsts& sk, const float* d_free_poses, const float* d_angles, uint32_t n_frames,
              float* d_poses, void* stream, std::string& err) {
    const uint32_t blocks = (n_frames + kFkLanes - 1) / kFkLanes;
    hipLaunchKernelGGL(fk_kernel, dim3(blocks), dim3(kFkLanes), fk_lds_bytes(sk), reinterpret_cast<hipStream_t>(stream), sk,
                       d_free_poses, d_angles, n_frames, d_poses);
    const hipError_t rc = hipGetLastError();
    if (rc != hipSuccess) {
        err = std::string("kernel launch failed: ") + hipGetErrorString(rc);
        return PXR_ERR_DEVICE;
    }
    return PXR_OK;
}

}  // namespace pxr
