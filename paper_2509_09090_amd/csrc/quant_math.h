// Device arithmetic of the per-row int4 quantizer, shared by the kernels that quantize a row they
// have just produced (quantize.hip, glue.hip).  Device code only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sqap {

// Correctly rounded binary32 quotient v / s for a divisor whose reciprocal r = RN(1/s)
// was formed once per row (IEEE division).  q0 = RN(v r) is within one ulp of v/s, the
// FMA gives the exact remainder, and the second FMA rounds q0 + rem * r to the
// correctly rounded quotient (Markstein's correction; it can fail only for divisors whose
// significand is all ones, which a half-precision scale widened to binary32 never is).
// Three instructions instead of the ~15 of a full IEEE division per element; every
// half / half pair is compared against the division operator by sqap_selftest_quotient.
__device__ __forceinline__ float quotient(float v, float s, float r)
{
    const float q0 = v * r;
    const float rem = fmaf(-q0, s, v);
    return fmaf(rem, r, q0);
}

// clamp(rint(q), -8, 7) as a 4-bit two's complement code.  Clamping first gives the same integer (both
// bounds are integers and rounding is monotone), and adding 1.5 * 2^23 rounds a value of that size to
// the nearest integer, ties to even like rint, and leaves it in the low mantissa bits: one addition
// instead of a rounding and a conversion.  A NaN quotient clamps to -8 either way.
__device__ __forceinline__ uint32_t code4(float q)
{
    const float c = fminf(fmaxf(q, -8.f), 7.f);
    return __float_as_uint(c + 12582912.0f) & 15u;
}

// scale = half(max|v| / 7), the smallest subnormal when that rounds to zero (an all-zero row)
__device__ __forceinline__ __half row_scale(float amax)
{
    __half sh = __float2half_rn(amax / 7.0f);
    if (__half_as_ushort(sh) == 0) sh = __ushort_as_half((unsigned short)1);
    return sh;
}

}  // namespace sqap
