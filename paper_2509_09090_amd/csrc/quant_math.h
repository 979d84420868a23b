// Device arithmetic of the per-row int4 quantizer, shared by the kernels that quantize a row they
// have just produced (quantize.hip, glue.hip).  Device code only.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
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

// Adds the squares of eight half values (held as floats), times 2^48, to the 128-bit integer hi:lo: exactly.
// A half is an integer m < 2^11 times 2^e, e >= -24, so x^2 * 2^48 is an integer below 2^80.
// Usual case: binary64.  With E the binary32 exponent field of an element (127 + e + 10 for a normal half; a
// subnormal half has a smaller field and a coarser unit than that suggests), every square is a multiple of
// 2^(2 (E_min - 137)) and the sum of eight is below 2^(2 E_max - 249): when the fields of the nonzero elements
// differ by at most 14 every partial sum has at most 53 significant bits, the binary64 additions are exact, and
// the sum's significand is shifted into place once.  Otherwise (a group that spans more than 2^14 in magnitude)
// every square is shifted and added on its own.
__device__ __forceinline__ void add_squares8(const float (&v)[8], unsigned long long &hi, unsigned long long &lo)
{
    unsigned ex_max = 0u, ex_min = 255u;
    double sum = 0.0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const unsigned ex = (__float_as_uint(v[e]) >> 23) & 255u;          // 0 for a zero only: halves are not that small
        ex_max = max(ex_max, ex);
        ex_min = ex != 0u ? min(ex_min, ex) : ex_min;
        const double x = (double)v[e];
        sum = fma(x, x, sum);
    }
    const bool narrow = ex_max <= ex_min + 14u;                            // (a group of zeros: 0 <= 269)
    if (__builtin_expect(narrow, 1)) {
        if (sum != 0.0) {
            const unsigned long long bits = (unsigned long long)__double_as_longlong(sum);
            const unsigned long long mant = (bits & 0xfffffffffffffull) | 0x10000000000000ull;
            const int s = (int)(bits >> 52) - 1023 - 52 + 48;      // sum * 2^48 = mant * 2^s, an integer
            unsigned long long add_lo, add_hi = 0ull;
            if (s >= 0) {
                add_lo = mant << s;                                // s <= 33 + 25 - 52 + 48 < 64
                if (s > 11) add_hi = mant >> (64 - s);
            } else {
                add_lo = mant >> (-s);                             // the bits shifted out are zero
            }
            lo += add_lo;
            hi += add_hi + (lo < add_lo ? 1ull : 0ull);
        }
        return;
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const unsigned bits = __half_as_ushort(__float2half_rn(v[e]));      // exact: v is a half value
        const unsigned exh = (bits >> 10) & 31u, man = bits & 1023u;
        const unsigned long long m = exh ? man + 1024u : man;
        const int sh = exh ? 2 * (int)exh - 2 : 0;                          // 2e + 48, at most 58
        const unsigned long long m2 = m * m;                                // below 2^22
        const unsigned long long add_lo = m2 << sh;
        const unsigned long long add_hi = sh > 42 ? m2 >> (64 - sh) : 0ull;
        lo += add_lo;
        hi += add_hi + (lo < add_lo ? 1ull : 0ull);
    }
}

// S / K in binary64.  For a power of two the quotient is S with a smaller exponent (S is zero or at least 2^-48,
// so nothing underflows): one instruction instead of the division's forty, the same bits.
__device__ __forceinline__ double mean_of(double S, int K)
{
    if ((K & (K - 1)) == 0) return ldexp(S, -__builtin_ctz((unsigned)K));
    return S / (double)K;
}

}  // namespace sqap
