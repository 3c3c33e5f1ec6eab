// Instruction-level shortcuts of the render kernel for two operations whose results decide integers
// (snapped coordinates, depth keys), so they must equal the plain forms bit for bit.  Each is compared with
// the plain form over its whole domain, on the device, by pxr_selftest_arithmetic (selftest.hip).
#ifndef PXR_ARITH_H
#define PXR_ARITH_H

#include <hip/hip_runtime.h>

namespace pxr {

// (int)floorf(x) in one instruction (rounds towards minus infinity while converting and saturates like the
// two-instruction form).  NOT for values that may be NaN: those give INT_MAX or INT_MIN by sign here and 0
// there.  Used where the argument is finite by construction (a snapped coordinate inside the guard band, a
// clamped colour); the checkerboard cell index, which a non-finite root pose reaches, keeps the long form.
__device__ __forceinline__ int floor_to_int(float x) {
    int r;
    asm("v_cvt_flr_i32_f32 %0, %1" : "=v"(r) : "v"(x));
    return r;
}

// 1 / x, correctly rounded, for 2^-100 <= x <= 2^100: the hardware's reciprocal estimate (1 ulp) and one
// Newton step whose residual is a single fused operation.  Equal to the IEEE division sequence for every
// float in that range (checked exhaustively on the device by pxr_selftest_arithmetic); outside it (zero,
// denormal, huge, infinite, NaN) it is not, and callers route such values around it.
constexpr float kRecipMax = 0x1p100f, kRecipMin = 0x1p-100f;
__device__ __forceinline__ float recip_in_range(float x) {
    const float y = __builtin_amdgcn_rcpf(x);
    return __builtin_fmaf(__builtin_fmaf(-x, y, 1.0f), y, y);
}

}  // namespace pxr

#endif
