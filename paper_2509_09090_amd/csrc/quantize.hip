// Per-row symmetric int4 quantizer (activations: one row per token; weights:
// one row per output channel), with the optional Hadamard rotation of Eq. 6,
// and the re-layout of canonical packed weights into the streaming layout.
#include "common.h"
#include "quant_math.h"

namespace sqap {

// A thread holds up to 8 groups of 8 elements of its row: K <= 16384 (checked by the callers).

// How the scale enters (Section 3.3):
//   kPerRow      one scale per row, from the row's own maximum (per token / per output channel)
//   kChannelwise static scale per input channel given by the caller; the per-row scale written is 1
//   kFolded      the row is first multiplied by the per-channel scales (the activation scales folded
//                into a weight), then quantized per row
enum QuantMode { kPerRow = 0, kChannelwise = 1, kFolded = 2 };

// Reads one row into registers: thread t owns groups t, t+256, ... of 8 consecutive elements.
template <int GPT>
__device__ __forceinline__ void load_halves(const uint4 *xrow, int K, float (&v)[GPT][8])
{
    const int t = threadIdx.x;
    const int groups = K >> 3;
#pragma unroll
    for (int gi = 0; gi < GPT; ++gi) {
        const int g = t + gi * 256;
        if (g < groups) {
            typedef unsigned int v4u __attribute__((ext_vector_type(4)));
            union { v4u v; uint4 u; } ld;
            ld.v = __builtin_nontemporal_load(reinterpret_cast<const v4u *>(xrow) + g);   // a row is read once
            uint4 raw = ld.u;
            const __half2 *h2 = reinterpret_cast<const __half2 *>(&raw);
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                float2 f = __half22float2(h2[p]);
                v[gi][2 * p] = f.x;
                v[gi][2 * p + 1] = f.y;
            }
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) v[gi][e] = 0.f;
        }
    }
}

// The rotation of Eq. 6 on a row held in registers: butterfly stages at distance 1, 2, 4 inside a
// group of 8 in registers, then passes over LDS that each apply up to three further stages (distance
// s, 2s, 4s) to sets of 8 elements {base + j s} owned by one thread, so a pass costs one read, one
// write and one barrier for three stages; then one multiply by (float)(1/sqrt(B)), B = K for a power
// of two.  The stages come in the order 1, 2, 4, ..., B/2 and every butterfly is (a, b) -> (a + b, a - b) with a the lower
// index, as the definition has it, so the result is the same bits whatever the pass structure.
// LDS index i lives at i + 8 (i / 64): with that padding the lanes of a wavefront hit distinct
// banks in every pass.  Contains barriers.
__device__ __forceinline__ int rot_at(int i) { return i + ((i >> 6) << 3); }
constexpr size_t rot_lds_bytes(int K) { return ((size_t)K + (size_t)K / 8) * sizeof(float); }

template <int W>
__device__ __forceinline__ void rotate_pass(float *rot, int K, int s)
{
    for (int o = threadIdx.x; o < K / W; o += 256) {
        const int base = (o / s) * (W * s) + (o % s);
        float x[W];
#pragma unroll
        for (int j = 0; j < W; ++j) x[j] = rot[rot_at(base + j * s)];
#pragma unroll
        for (int hh = 1; hh < W; hh <<= 1) {
#pragma unroll
            for (int j = 0; j < W; ++j) {
                if ((j & hh) == 0) {
                    const float a = x[j], b = x[j + hh];
                    x[j] = a + b;
                    x[j + hh] = a - b;
                }
            }
        }
#pragma unroll
        for (int j = 0; j < W; ++j) rot[rot_at(base + j * s)] = x[j];
    }
}

template <int GPT>
__device__ __forceinline__ void rotate_row(int K, float (&v)[GPT][8], float *rot)
{
    const int t = threadIdx.x;
    const int groups = K >> 3;
#pragma unroll
    for (int gi = 0; gi < GPT; ++gi) {
#pragma unroll
        for (int h = 1; h < 8; h <<= 1) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                if ((e & h) == 0) {
                    float a = v[gi][e], b = v[gi][e + h];
                    v[gi][e] = a + b;
                    v[gi][e + h] = a - b;
                }
            }
        }
        const int g = t + gi * 256;
        if (g < groups) {                      // a group of 8 never straddles a padded block of 64
            float4 *dst = reinterpret_cast<float4 *>(rot + rot_at(g * 8));
            dst[0] = make_float4(v[gi][0], v[gi][1], v[gi][2], v[gi][3]);
            dst[1] = make_float4(v[gi][4], v[gi][5], v[gi][6], v[gi][7]);
        }
    }
    __syncthreads();
    // a row whose length is not a power of two is rotated block by block: one matrix of order B per
    // aligned run of B channels, B the largest power of two dividing K (the stages simply stop at B/2)
    const int B = K & -K;
    for (int s = 8; s < B; s <<= 3) {
        if (s * 8 <= B) rotate_pass<8>(rot, K, s);
        else if (s * 4 <= B) rotate_pass<4>(rot, K, s);
        else rotate_pass<2>(rot, K, s);
        __syncthreads();
    }
    const float c = (float)(1.0 / sqrt((double)B));
#pragma unroll
    for (int gi = 0; gi < GPT; ++gi) {
        const int g = t + gi * 256;
        if (g < groups) {
            const float4 *src = reinterpret_cast<const float4 *>(rot + rot_at(g * 8));
            const float4 lo = src[0], hi = src[1];
            v[gi][0] = lo.x * c; v[gi][1] = lo.y * c; v[gi][2] = lo.z * c; v[gi][3] = lo.w * c;
            v[gi][4] = hi.x * c; v[gi][5] = hi.y * c; v[gi][6] = hi.z * c; v[gi][7] = hi.w * c;
        }
    }
}

template <bool ROTATE, int GPT>
__device__ __forceinline__ void load_row(const uint4 *xrow, int K, float (&v)[GPT][8], float *rot)
{
    load_halves<GPT>(xrow, K, v);
    if (ROTATE) rotate_row<GPT>(K, v, rot);
}

// ---- operations fused in front of the quantizer (the decoder's glue between two linears) ----

// The empty asm makes x exist as a binary32 value: otherwise the compiler folds the operation that
// produced it and the conversion into one mixed-precision instruction that rounds only once.
__device__ __forceinline__ float round_to_half(float x)
{
    asm volatile("" : "+v"(x));
    return __half2float(__float2half_rn(x));
}

__device__ __forceinline__ void unpack8(const uint4 raw, float (&f)[8])
{
    const __half2 *h2 = reinterpret_cast<const __half2 *>(&raw);
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const float2 x = __half22float2(h2[p]);
        f[2 * p] = x.x;
        f[2 * p + 1] = x.y;
    }
}

__device__ __forceinline__ uint4 pack8(const float (&f)[8])
{
    uint4 raw;
    __half2 *h2 = reinterpret_cast<__half2 *>(&raw);
#pragma unroll
    for (int p = 0; p < 4; ++p) h2[p] = __floats2half2_rn(f[2 * p], f[2 * p + 1]);
    return raw;
}

// RMSNorm of the row in v (Zhang & Sennrich 2019, as used in front of every linear group of a
// Llama decoder), after an optional residual update x' = half(x + delta):
//   S = sum x'^2 exactly;  r = (float)(1 / sqrt(S / K + eps)) in binary64;
//   v = half((x' * r) * gamma)
// The sum is exact and therefore independent of the order in which lanes add: a half is an
// integer m < 2^11 times 2^e, e >= -24, so x^2 * 2^48 is an integer below 2^80; every thread
// adds its elements into a 128-bit integer, wavefronts and the block add those.  The sum is
// rounded to binary64 once (top 64 bits with a sticky last bit, then the hardware's u64 -> f64
// conversion, which rounds to nearest even).  Rows are assumed finite.
template <int GPT>
__device__ __forceinline__ void norm_row(float (&v)[GPT][8], int row, int K, const PreArgs &pre,
                                         unsigned long long *wsum)
{
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6, groups = K >> 3;
    unsigned long long hi = 0, lo = 0;
#pragma unroll
    for (int gi = 0; gi < GPT; ++gi) {
        const int g = t + gi * 256;
        if (g < groups) {
            if (pre.delta) {
                float d[8];
                unpack8(reinterpret_cast<const uint4 *>(pre.delta + (size_t)row * K)[g], d);
#pragma unroll
                for (int e = 0; e < 8; ++e) v[gi][e] = round_to_half(v[gi][e] + d[e]);
            }
            if (pre.xsum_out) reinterpret_cast<uint4 *>(pre.xsum_out + (size_t)row * K)[g] = pack8(v[gi]);
            add_squares8(v[gi], hi, lo);
        }
    }
    wave_sum128(hi, lo);
    if (lane == 0) {
        wsum[2 * wave] = hi;
        wsum[2 * wave + 1] = lo;
    }
    __syncthreads();
    hi = wsum[0];
    lo = wsum[1];
#pragma unroll
    for (int w = 1; w < 4; ++w) {
        const unsigned long long olo = wsum[2 * w + 1];
        lo += olo;
        hi += wsum[2 * w] + (lo < olo ? 1ull : 0ull);
    }
    double Sd;
    if (hi == 0) {
        Sd = (double)lo;
    } else {
        const int lz = __clzll((long long)hi);
        unsigned long long top = lz ? (hi << lz) | (lo >> (64 - lz)) : hi;
        const unsigned long long rest = lz ? lo << lz : lo;
        top |= rest != 0 ? 1ull : 0ull;
        Sd = ldexp((double)top, 64 - lz);
    }
    Sd = ldexp(Sd, -48);
    const float r = (float)(1.0 / sqrt(mean_of(Sd, K) + (double)pre.eps));
#pragma unroll
    for (int gi = 0; gi < GPT; ++gi) {
        const int g = t + gi * 256;
        if (g < groups) {
            float gm[8];
            unpack8(reinterpret_cast<const uint4 *>(pre.gamma)[g], gm);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float xr = v[gi][e] * r;
                v[gi][e] = round_to_half(xr * gm[e]);
            }
            if (pre.y_out) reinterpret_cast<uint4 *>(pre.y_out + (size_t)row * K)[g] = pack8(v[gi]);
        }
    }
}

// SwiGLU (Shazeer 2020; the feed-forward of a Llama decoder): v holds the gate row g, pre.U the
// up row;  v = half(silu(g) * u),  silu(g) = (float)(g / (1 + exp(-g))) evaluated in binary64.
// silu is a function of a half value: a GPU test walks all 2^16 of them against the host's.
// (A per-device table of the 2^16 results was slower than computing: 13 against 10 us at 84 x 11008,
// 48 scattered 4-byte loads per thread.)
template <int GPT>
__device__ __forceinline__ void swiglu_row(float (&v)[GPT][8], int row, int K, const PreArgs &pre)
{
    const int t = threadIdx.x, groups = K >> 3;
#pragma unroll
    for (int gi = 0; gi < GPT; ++gi) {
        const int g = t + gi * 256;
        if (g < groups) {
            float u[8];
            unpack8(reinterpret_cast<const uint4 *>(pre.U + (size_t)row * pre.ldu)[g], u);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const double gd = (double)v[gi][e];
                const float s = (float)(gd / (1.0 + exp(-gd)));
                v[gi][e] = round_to_half(s * u[e]);
            }
            if (pre.y_out) reinterpret_cast<uint4 *>(pre.y_out + (size_t)row * K)[g] = pack8(v[gi]);
        }
    }
}

// The eight per-channel scales of group g as floats.
__device__ __forceinline__ void load_col_scales(const __half *col_scales, int g, float (&c)[8])
{
    const uint4 raw = reinterpret_cast<const uint4 *>(col_scales)[g];
    const __half2 *h2 = reinterpret_cast<const __half2 *>(&raw);
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const float2 f = __half22float2(h2[p]);
        c[2 * p] = f.x;
        c[2 * p + 1] = f.y;
    }
}

// One block per output row; the row stays in registers from its single read to the packed
// store.  Arithmetic (all binary32, IEEE, no contraction possible):
//   scale = half(max|v| / 7), 2^-24 if that is zero;  code = clamp(rint(v / scale), -8, 7)
// GPT = groups per thread the instance is compiled for (registers, hence occupancy).
// PRE selects an operation applied to the row between its read and the quantizer (see above).
template <bool ROTATE, int GPT, int MODE, int PRE>
__global__ __launch_bounds__(256) void quantize_rows_kernel(const __half *X, int64_t ldx,      // may alias pre.xsum_out
                                                            const int32_t *__restrict__ rows, int K,
                                                            const __half *__restrict__ col_scales,
                                                            uint8_t *__restrict__ Xq,
                                                            __half *__restrict__ scale_out, const PreArgs pre)
{
    extern __shared__ __attribute__((aligned(16))) float rot[];       // the padded row when ROTATE
    __shared__ float wave_max[4];
    __shared__ unsigned long long wave_sum[8];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int row = blockIdx.x;
    const int64_t src = rows ? (int64_t)rows[row] : (int64_t)row;
    const uint4 *xrow = reinterpret_cast<const uint4 *>(X + src * ldx);
    const int groups = K >> 3;

    float v[GPT][8];
    load_halves<GPT>(xrow, K, v);
    if (PRE == kPreNorm) norm_row<GPT>(v, row, K, pre, wave_sum);
    if (PRE == kPreSwiglu) swiglu_row<GPT>(v, row, K, pre);
    if (ROTATE) rotate_row<GPT>(K, v, rot);
    if (!Xq) return;                     // the caller wanted the half-precision result only (uniform)
    uint32_t *qrow = reinterpret_cast<uint32_t *>(Xq + (size_t)row * (K >> 1));

    if (MODE == kChannelwise) {
        if (t == 0) scale_out[row] = __ushort_as_half((unsigned short)0x3c00);      // 1.0
#pragma unroll
        for (int gi = 0; gi < GPT; ++gi) {
            const int g = t + gi * 256;
            if (g < groups) {
                float c[8];
                load_col_scales(col_scales, g, c);
                uint32_t packed = 0;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    packed |= code4(v[gi][e] / c[e]) << (4 * e);
                }
                qrow[g] = packed;
            }
        }
        return;
    }
    if (MODE == kFolded) {
#pragma unroll
        for (int gi = 0; gi < GPT; ++gi) {
            const int g = t + gi * 256;
            if (g < groups) {
                float c[8];
                load_col_scales(col_scales, g, c);
#pragma unroll
                for (int e = 0; e < 8; ++e) v[gi][e] = v[gi][e] * c[e];
            }
        }
    }

    float amax = 0.f;
#pragma unroll
    for (int gi = 0; gi < GPT; ++gi)
#pragma unroll
        for (int e = 0; e < 8; ++e) amax = fmaxf(amax, fabsf(v[gi][e]));
    amax = wavefront_max(amax);
    if (lane == 0) wave_max[wave] = amax;
    __syncthreads();
    amax = fmaxf(fmaxf(wave_max[0], wave_max[1]), fmaxf(wave_max[2], wave_max[3]));

    const __half sh = row_scale(amax);
    const float sf = __half2float(sh);
    if (t == 0) scale_out[row] = sh;

    // Inputs that were neither rotated nor multiplied by channel scales are half values, for
    // which the fast quotient is verified exhaustively; the others take the division operator.
    const float rcp = 1.0f / sf;
#pragma unroll
    for (int gi = 0; gi < GPT; ++gi) {
        const int g = t + gi * 256;
        if (g < groups) {
            uint32_t packed = 0;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                packed |= code4((ROTATE || MODE == kFolded) ? v[gi][e] / sf : quotient(v[gi][e], sf, rcp)) << (4 * e);
            }
            qrow[g] = packed;
        }
    }
}

// The plain quantizer (no rotation, no channel scales, nothing fused in front) for many rows: one block
// takes TWO rows and asks for both before it works on the first, so the second row's read is in flight
// during the first row's reduction and arithmetic, and 2368 rows of K = 11008 fit the device in one
// round of blocks instead of one and a sixth.  Same arithmetic, statement by statement, as the kernel above.
template <int GPT>
__global__ __launch_bounds__(256) void quantize_row_pairs_kernel(const __half *__restrict__ X, int64_t ldx,
                                                                 const int32_t *__restrict__ rows, int M, int K,
                                                                 uint8_t *__restrict__ Xq,
                                                                 __half *__restrict__ scale_out)
{
    __shared__ float wave_max[2][4];
    typedef unsigned int v4u __attribute__((ext_vector_type(4)));
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int groups = K >> 3;
    const int row0 = 2 * blockIdx.x;
    const int nrows = row0 + 1 < M ? 2 : 1;
    v4u raw[2][GPT];
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        const int row = min(row0 + r, M - 1);                       // (a missing second row re-reads the first)
        const int64_t src = rows ? (int64_t)rows[row] : (int64_t)row;
        const v4u *xrow = reinterpret_cast<const v4u *>(X + src * ldx);
#pragma unroll
        for (int gi = 0; gi < GPT; ++gi) {
            const int g = t + gi * 256;
            raw[r][gi] = g < groups ? __builtin_nontemporal_load(xrow + g) : v4u{0u, 0u, 0u, 0u};
        }
    }
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        if (r >= nrows) break;
        const int row = row0 + r;
        float v[GPT][8];
#pragma unroll
        for (int gi = 0; gi < GPT; ++gi) {
            union { v4u v; uint4 u; } ld;
            ld.v = raw[r][gi];
            unpack8(ld.u, v[gi]);
        }
        float amax = 0.f;
#pragma unroll
        for (int gi = 0; gi < GPT; ++gi)
#pragma unroll
            for (int e = 0; e < 8; ++e) amax = fmaxf(amax, fabsf(v[gi][e]));
        amax = wavefront_max(amax);
        if (lane == 0) wave_max[r][wave] = amax;
        __syncthreads();
        amax = fmaxf(fmaxf(wave_max[r][0], wave_max[r][1]), fmaxf(wave_max[r][2], wave_max[r][3]));

        const __half sh = row_scale(amax);
        const float sf = __half2float(sh);
        if (t == 0) scale_out[row] = sh;
        const float rcp = 1.0f / sf;
        uint32_t *qrow = reinterpret_cast<uint32_t *>(Xq + (size_t)row * (K >> 1));
#pragma unroll
        for (int gi = 0; gi < GPT; ++gi) {
            const int g = t + gi * 256;
            if (g < groups) {
                uint32_t packed = 0;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    packed |= code4(quotient(v[gi][e], sf, rcp)) << (4 * e);
                }
                qrow[g] = packed;
            }
        }
    }
}

// Static channel scales from calibration rows: each block walks rows blockIdx.x, + gridDim.x,
// ... keeping the running maximum of its threads' columns in registers (the column layout of
// load_row is the same for every row), then merges into amax[] with an integer atomic maximum
// on the bit pattern (non-negative floats order like their bits; a maximum is order independent).
template <bool ROTATE, int GPT>
__global__ __launch_bounds__(256) void channel_absmax_kernel(const __half *__restrict__ X, int64_t ldx,
                                                             const int32_t *__restrict__ rows, int M, int K,
                                                             float *__restrict__ amax)
{
    extern __shared__ __attribute__((aligned(16))) float rot[];
    const int t = threadIdx.x, groups = K >> 3;
    float best[GPT][8];
#pragma unroll
    for (int gi = 0; gi < GPT; ++gi)
#pragma unroll
        for (int e = 0; e < 8; ++e) best[gi][e] = 0.f;
    for (int row = blockIdx.x; row < M; row += gridDim.x) {
        const int64_t src = rows ? (int64_t)rows[row] : (int64_t)row;
        float v[GPT][8];
        load_row<ROTATE, GPT>(reinterpret_cast<const uint4 *>(X + src * ldx), K, v, rot);
#pragma unroll
        for (int gi = 0; gi < GPT; ++gi)
#pragma unroll
            for (int e = 0; e < 8; ++e) best[gi][e] = fmaxf(best[gi][e], fabsf(v[gi][e]));
        if (ROTATE) __syncthreads();          // the next row reuses rot[]
    }
#pragma unroll
    for (int gi = 0; gi < GPT; ++gi) {
        const int g = t + gi * 256;
        if (g < groups) {
#pragma unroll
            for (int e = 0; e < 8; ++e)
                atomicMax(reinterpret_cast<unsigned int *>(amax) + g * 8 + e, __float_as_uint(best[gi][e]));
        }
    }
}

__global__ __launch_bounds__(256) void fill_zero_kernel(float *p, int n)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = 0.f;
}

// c_k = half(amax_k / 7), 2^-24 if that is zero
__global__ __launch_bounds__(256) void channel_scales_kernel(const float *__restrict__ amax, int K,
                                                             __half *__restrict__ scales)
{
    const int k = blockIdx.x * 256 + threadIdx.x;
    if (k < K) {
        __half sh = __float2half_rn(amax[k] / 7.0f);
        if (__half_as_ushort(sh) == 0) sh = __ushort_as_half((unsigned short)1);
        scales[k] = sh;
    }
}

template <bool ROTATE, int GPT, int MODE, int PRE>
static void launch_quantize_inst(const __half *X, int64_t ldx, const int32_t *rows, int M, int K, size_t lds,
                                 const __half *col_scales, uint8_t *Xq, __half *sx, const PreArgs &pre,
                                 hipStream_t st)
{
    hipLaunchKernelGGL((quantize_rows_kernel<ROTATE, GPT, MODE, PRE>), dim3(M), dim3(256), lds, st, X, ldx, rows, K,
                       col_scales, Xq, sx, pre);
}

template <bool ROTATE, int MODE, int PRE>
static void launch_quantize_gpt(int gpt, const __half *X, int64_t ldx, const int32_t *rows, int M, int K,
                                size_t lds, const __half *col_scales, uint8_t *Xq, __half *sx, const PreArgs &pre,
                                hipStream_t st)
{
    if (gpt <= 1) launch_quantize_inst<ROTATE, 1, MODE, PRE>(X, ldx, rows, M, K, lds, col_scales, Xq, sx, pre, st);
    else if (gpt <= 2) launch_quantize_inst<ROTATE, 2, MODE, PRE>(X, ldx, rows, M, K, lds, col_scales, Xq, sx, pre, st);
    else if (gpt <= 4) launch_quantize_inst<ROTATE, 4, MODE, PRE>(X, ldx, rows, M, K, lds, col_scales, Xq, sx, pre, st);
    else if (gpt <= 6) launch_quantize_inst<ROTATE, 6, MODE, PRE>(X, ldx, rows, M, K, lds, col_scales, Xq, sx, pre, st);
    else launch_quantize_inst<ROTATE, 8, MODE, PRE>(X, ldx, rows, M, K, lds, col_scales, Xq, sx, pre, st);
}

// Rotation keeps the row in LDS: K floats plus padding, above the 64 KiB default for the widest rows.
template <class Kern>
static sqap_status allow_rotation_lds(Kern kernel, size_t lds)
{
    if (lds > 48 * 1024)
        SQAP_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)rot_lds_bytes(16384)));
    return SQAP_OK;
}

constexpr int kPairsMinRows = 1024;      // from here on the plain quantizer takes two rows per block

template <int MODE, int PRE>
static sqap_status launch_quantize_mode(const __half *X, int64_t ldx, const int32_t *rows, int M, int K,
                                        bool rotate, const __half *col_scales, uint8_t *Xq, __half *sx,
                                        const PreArgs &pre, hipStream_t st)
{
    const int gpt = (K / 8 + 255) / 256;
    if (rotate) {
        if constexpr (PRE == kPreSwiglu) {
            return fail(SQAP_EUNSUPPORTED, "rotation is not available behind the SwiGLU gate");
        } else {
            const size_t lds = rot_lds_bytes(K);
            sqap_status s = allow_rotation_lds(&quantize_rows_kernel<true, 8, MODE, PRE>, lds);
            if (s != SQAP_OK) return s;
            launch_quantize_gpt<true, MODE, PRE>(gpt, X, ldx, rows, M, K, lds, col_scales, Xq, sx, pre, st);
        }
    } else if (MODE == kPerRow && PRE == kPreNone && Xq && M >= kPairsMinRows) {
        const dim3 grid((M + 1) / 2), block(256);
        if (gpt <= 1) hipLaunchKernelGGL(quantize_row_pairs_kernel<1>, grid, block, 0, st, X, ldx, rows, M, K, Xq, sx);
        else if (gpt <= 2) hipLaunchKernelGGL(quantize_row_pairs_kernel<2>, grid, block, 0, st, X, ldx, rows, M, K, Xq, sx);
        else if (gpt <= 4) hipLaunchKernelGGL(quantize_row_pairs_kernel<4>, grid, block, 0, st, X, ldx, rows, M, K, Xq, sx);
        else if (gpt <= 6) hipLaunchKernelGGL(quantize_row_pairs_kernel<6>, grid, block, 0, st, X, ldx, rows, M, K, Xq, sx);
        else hipLaunchKernelGGL(quantize_row_pairs_kernel<8>, grid, block, 0, st, X, ldx, rows, M, K, Xq, sx);
    } else {
        launch_quantize_gpt<false, MODE, PRE>(gpt, X, ldx, rows, M, K, 0, col_scales, Xq, sx, pre, st);
    }
    SQAP_HIP_CHECK(hipGetLastError());
    return SQAP_OK;
}

sqap_status launch_quantize_rows(const __half *X, int64_t ldx, const int32_t *rows, int M, int K,
                                 bool rotate, uint8_t *Xq, __half *sx, hipStream_t st)
{
    return launch_quantize_mode<kPerRow, kPreNone>(X, ldx, rows, M, K, rotate, nullptr, Xq, sx, PreArgs{}, st);
}

sqap_status launch_quantize_rows_scaled(const __half *X, int64_t ldx, const int32_t *rows, int M, int K,
                                        bool rotate, bool folded, const __half *col_scales, uint8_t *Xq,
                                        __half *sx, hipStream_t st)
{
    if (folded)
        return launch_quantize_mode<kFolded, kPreNone>(X, ldx, rows, M, K, rotate, col_scales, Xq, sx, PreArgs{}, st);
    return launch_quantize_mode<kChannelwise, kPreNone>(X, ldx, rows, M, K, rotate, col_scales, Xq, sx, PreArgs{}, st);
}

sqap_status launch_fused_quantize(int pre_op, const __half *X, int64_t ldx, const int32_t *rows, int M, int K,
                                  bool rotate, const __half *col_scales, uint8_t *Xq, __half *sx,
                                  const PreArgs &pre, hipStream_t st)
{
    if (pre_op == kPreNorm) {
        if (col_scales)
            return launch_quantize_mode<kChannelwise, kPreNorm>(X, ldx, rows, M, K, rotate, col_scales, Xq, sx, pre, st);
        return launch_quantize_mode<kPerRow, kPreNorm>(X, ldx, rows, M, K, rotate, nullptr, Xq, sx, pre, st);
    }
    if (col_scales)
        return launch_quantize_mode<kChannelwise, kPreSwiglu>(X, ldx, rows, M, K, rotate, col_scales, Xq, sx, pre, st);
    return launch_quantize_mode<kPerRow, kPreSwiglu>(X, ldx, rows, M, K, rotate, nullptr, Xq, sx, pre, st);
}

template <bool ROTATE>
static void launch_absmax_gpt(int gpt, int grid, size_t lds, const __half *X, int64_t ldx, const int32_t *rows,
                              int M, int K, float *amax, hipStream_t st)
{
    if (gpt <= 2)
        hipLaunchKernelGGL((channel_absmax_kernel<ROTATE, 2>), dim3(grid), dim3(256), lds, st, X, ldx, rows, M, K, amax);
    else if (gpt <= 4)
        hipLaunchKernelGGL((channel_absmax_kernel<ROTATE, 4>), dim3(grid), dim3(256), lds, st, X, ldx, rows, M, K, amax);
    else
        hipLaunchKernelGGL((channel_absmax_kernel<ROTATE, 8>), dim3(grid), dim3(256), lds, st, X, ldx, rows, M, K, amax);
}

sqap_status launch_channel_scales(const __half *X, int64_t ldx, const int32_t *rows, int M, int K, bool rotate,
                                  float *amax, bool accumulate, __half *scales, hipStream_t st)
{
    const int kblocks = (K + 255) / 256;
    if (!accumulate) hipLaunchKernelGGL(fill_zero_kernel, dim3(kblocks), dim3(256), 0, st, amax, K);
    if (M > 0) {
        const int gpt = (K / 8 + 255) / 256;
        const int grid = M < 256 ? M : 256;
        if (rotate) {
            const size_t lds = rot_lds_bytes(K);
            sqap_status s = allow_rotation_lds(&channel_absmax_kernel<true, 8>, lds);
            if (s != SQAP_OK) return s;
            launch_absmax_gpt<true>(gpt, grid, lds, X, ldx, rows, M, K, amax, st);
        } else {
            launch_absmax_gpt<false>(gpt, grid, 0, X, ldx, rows, M, K, amax, st);
        }
    }
    hipLaunchKernelGGL(channel_scales_kernel, dim3(kblocks), dim3(256), 0, st, amax, K, scales);
    SQAP_HIP_CHECK(hipGetLastError());
    return SQAP_OK;
}

// Self-test: for every pair (v, s) of finite half values with s > 0, compares the fast
// quotient with the division operator, bit for bit.  Counts the differences.
__global__ __launch_bounds__(256) void quotient_selftest_kernel(unsigned long long *mismatches)
{
    const unsigned s_bits = blockIdx.x + 1;                    // 1 .. 0x7bff
    const float s = __half2float(__ushort_as_half((unsigned short)s_bits));
    const float r = 1.0f / s;
    unsigned bad = 0;
    for (unsigned v_bits = threadIdx.x; v_bits < 0x7c00u; v_bits += 256) {
        const float v = __half2float(__ushort_as_half((unsigned short)v_bits));
        const float a = v / s, b = quotient(v, s, r);
        const float an = (-v) / s, bn = quotient(-v, s, r);
        // (a zero quotient may differ in sign: -0 / s is -0, the corrected form gives +0;
        // both become code 0)
        bad += (__float_as_uint(a) != __float_as_uint(b) && !(a == 0.f && b == 0.f)) +
               (__float_as_uint(an) != __float_as_uint(bn) && !(an == 0.f && bn == 0.f));
    }
    if (bad) atomicAdd(mismatches, (unsigned long long)bad);
}

sqap_status launch_quotient_selftest(unsigned long long *mismatches, hipStream_t st)
{
    hipLaunchKernelGGL(quotient_selftest_kernel, dim3(0x7bff), dim3(256), 0, st, mismatches);
    SQAP_HIP_CHECK(hipGetLastError());
    return SQAP_OK;
}

// canonical [N, K/2] -> streaming layout (see Weight in common.h); one 16-byte
// piece per thread; rows past N and their scales are written as zero.
__global__ __launch_bounds__(256) void weight_pack_kernel(const uint8_t *__restrict__ Wq,
                                                          const __half *__restrict__ sw, int N, int chunks,
                                                          int n_groups, uint4 *__restrict__ data,
                                                          __half *__restrict__ scales)
{
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t total = (int64_t)n_groups * chunks * 32;
    if (gid < (int64_t)n_groups * 32) scales[gid] = gid < N ? sw[gid] : __ushort_as_half((unsigned short)0);
    if (gid >= total) return;
    const int r = (int)(gid & 31);
    const int64_t gc = gid >> 5;
    const int c = (int)(gc % chunks);
    const int64_t n = (gc / chunks) * 32 + r;
    uint4 val = make_uint4(0, 0, 0, 0);
    if (n < N) val = reinterpret_cast<const uint4 *>(Wq + n * ((int64_t)chunks * 16))[c];
    data[gid] = val;
}

sqap_status launch_weight_pack(const uint8_t *Wq, const __half *sw, const Weight &w, hipStream_t st)
{
    const int64_t total = (int64_t)w.n_groups * w.chunks * 32;
    const int64_t blocks = (total + 255) / 256;
    if (blocks > 0x7fffffff) return fail(SQAP_EUNSUPPORTED, "sqap_weight_pack: too large");
    hipLaunchKernelGGL(weight_pack_kernel, dim3((unsigned)blocks), dim3(256), 0, st, Wq, sw, w.N, w.chunks,
                       w.n_groups, reinterpret_cast<uint4 *>(w.data), w.scales);
    SQAP_HIP_CHECK(hipGetLastError());
    return SQAP_OK;
}

}  // namespace sqap
