// pxr_selftest_arithmetic: the render kernel's two instruction-level shortcuts (arith.h) against the plain
// forms they stand for, over every 32-bit pattern, on the current device.  Not on the hot path.

#include <hip/hip_runtime.h>

#include "arith.h"
#include "pxr_internal.h"

namespace pxr {
namespace {

// counts[0]: floats in [kRecipMin, kRecipMax] whose short reciprocal differs from 1.0f / x
// counts[1]: non-NaN floats whose one-instruction floor-and-convert differs from (int)floorf(x)
// counts[2], counts[3]: how many patterns each check looked at
__global__ __launch_bounds__(256) void arithmetic_check_kernel(unsigned long long* counts) {
    const unsigned long long stride = (unsigned long long)gridDim.x * 256ull;
    unsigned long long bad_recip = 0, bad_floor = 0, n_recip = 0, n_floor = 0;
    for (unsigned long long b = (unsigned long long)blockIdx.x * 256ull + threadIdx.x; b < (1ull << 32); b += stride) {
        const float x = __uint_as_float((uint32_t)b);
        if (x == x) {
            ++n_floor;
            if (floor_to_int(x) != (int)__builtin_floorf(x)) ++bad_floor;
        }
        if (x >= kRecipMin && x <= kRecipMax) {
            ++n_recip;
            if (__float_as_uint(recip_in_range(x)) != __float_as_uint(1.0f / x)) ++bad_recip;
        }
    }
    if (bad_recip) atomicAdd(&counts[0], bad_recip);
    if (bad_floor) atomicAdd(&counts[1], bad_floor);
    atomicAdd(&counts[2], n_recip);
    atomicAdd(&counts[3], n_floor);
}

}  // namespace

int selftest_arithmetic(unsigned long long counts[4], std::string& err) {
    unsigned long long* d = nullptr;
    hipError_t rc = hipMalloc(&d, 4 * sizeof(unsigned long long));
    if (rc != hipSuccess) {
        err = std::string("hipMalloc failed: ") + hipGetErrorString(rc);
        return PXR_ERR_OOM;
    }
    rc = hipMemset(d, 0, 4 * sizeof(unsigned long long));
    if (rc == hipSuccess) {
        hipLaunchKernelGGL(arithmetic_check_kernel, dim3(8192), dim3(256), 0, nullptr, d);
        rc = hipGetLastError();
    }
    if (rc == hipSuccess) rc = hipMemcpy(counts, d, 4 * sizeof(unsigned long long), hipMemcpyDeviceToHost);
    const hipError_t rc_free = hipFree(d);
    if (rc == hipSuccess) rc = rc_free;
    if (rc != hipSuccess) {
        err = std::string("device error: ") + hipGetErrorString(rc);
        return PXR_ERR_DEVICE;
    }
    return PXR_OK;
}

}  // namespace pxr
