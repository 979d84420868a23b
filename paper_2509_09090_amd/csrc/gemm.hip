// W4A4 linear: acc = Xq * Wq^T exactly in int32 on the int8 MFMA units, with
// the per-token x per-channel dequantisation fused into the epilogue.
//
// CDNA4 has no int4 MFMA, so both operands are widened on the fly.  A 16-byte
// piece of a packed row holds 32 codes; `(x << 4) & 0xF0F0F0F0` turns the 16
// low nibbles into 16 int8 values equal to 16 * code (the nibble's sign bit
// lands on the byte's sign bit) and `x & 0xF0F0F0F0` does the same for the high
// nibbles.  The low-nibble bytes feed lanes 0-31 of a 32x32x32 MFMA operand and
// the high-nibble bytes feed lanes 32-63; the activation rows are split the
// same way, so every product pairs codes of the same k.  The accumulator is
// then 256 * sum(x*w), |.| <= 256 * 64 * K < 2^31 for K <= 131071, and the
// epilogue shifts it back: the integer result is exact.
#include "common.h"

namespace sqap {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kBK = 128;            // codes of the reduction axis per main-loop step
constexpr int kChunksPerStep = 4;   // = kBK / 32, 16-byte packed pieces per row per step
constexpr int kMaxK = 131040;       // keeps 256 * 64 * K below 2^31

struct GemmParams {
    const uint8_t *Xq;     // [M, K/2] canonical
    const __half *sx;      // [M]
    const uint8_t *Wd;     // streaming layout
    const __half *sw;      // [n_groups * 32]
    __half *Y;
    int32_t *acc_out;      // nullable
    int64_t ldy;
    int M, N, K;
    int n_groups, chunks;
    int m_tiles, n_tiles;
};

__device__ __forceinline__ void widen(const uint4 &p, v4i &lo, v4i &hi)
{
    lo.x = (int)((p.x << 4) & 0xF0F0F0F0u);
    lo.y = (int)((p.y << 4) & 0xF0F0F0F0u);
    lo.z = (int)((p.z << 4) & 0xF0F0F0F0u);
    lo.w = (int)((p.w << 4) & 0xF0F0F0F0u);
    hi.x = (int)(p.x & 0xF0F0F0F0u);
    hi.y = (int)(p.y & 0xF0F0F0F0u);
    hi.z = (int)(p.z & 0xF0F0F0F0u);
    hi.w = (int)(p.w & 0xF0F0F0F0u);
}

// Y = half((float(acc) * sx) * sw): two binary32 products, then one rounding to
// half.  The empty asm keeps the compiler from folding the second product and
// the conversion into v_fma_mixlo_f16, which rounds the exact product once and
// so differs from the two-step definition in about one result in 2^13.
__device__ __forceinline__ __half dequant(int acc, float sx, float sw)
{
    float y = ((float)acc * sx) * sw;
    asm volatile("" : "+v"(y));
    return __float2half_rn(y);
}

// Block tile BM x BN, four wavefronts as 2 x 2, each owning (BM/2) x (BN/2) as
// 32x32 MFMA tiles.  LDS holds two stages of widened operands in "fragment
// order": for row group rg (32 rows) and k-step ks (32 codes) the 1 KiB at
// ((rg * 4 + ks) * 1024) is exactly what the 64 lanes of a wavefront read with
// one ds_read_b128 (lane l at l * 16): rows in lanes 0-31 (even codes), the
// same rows in lanes 32-63 (odd codes).
template <int BM, int BN>
__global__ __launch_bounds__(256, 1) void gemm_tiled_kernel(const GemmParams p)
{
    constexpr int WM = BM / 2, WN = BN / 2;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int A_BYTES = BM * kBK, B_BYTES = BN * kBK;      // per stage, widened
    constexpr int STAGE = A_BYTES + B_BYTES;
    constexpr int A_UNITS = BM * kChunksPerStep, B_UNITS = BN * kChunksPerStep;
    constexpr int A_LOADS = (A_UNITS + 255) / 256, B_LOADS = (B_UNITS + 255) / 256;
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    // Tile order: the hardware deals consecutive workgroups to the 8 XCDs in
    // turn; give each XCD a contiguous run of tiles (n-tile major, m-tile minor)
    // so that the tiles sharing a weight panel sit behind one L2.
    const int tiles = p.m_tiles * p.n_tiles;
    const int bid = blockIdx.x;
    const int xcd = bid & 7, j = bid >> 3;
    const int q = tiles >> 3, r = tiles & 7;
    const int tile = xcd * q + (xcd < r ? xcd : r) + j;
    const int nt = tile / p.m_tiles, mt = tile - nt * p.m_tiles;
    const int m0 = mt * BM, ng0 = nt * (BN / 32);
    const int Kh = p.K >> 1;

    // per-thread load slots
    const uint4 *a_src[A_LOADS];
    int a_dst[A_LOADS], a_chunk[A_LOADS];
    bool a_ok[A_LOADS];
#pragma unroll
    for (int i = 0; i < A_LOADS; ++i) {
        const int u = i * 256 + t;
        const int row = (u >> 6) * 16 + (u & 15), chunk = (u & 63) >> 4;
        a_ok[i] = (u < A_UNITS) && (m0 + row < p.M);
        a_chunk[i] = chunk;
        a_src[i] = reinterpret_cast<const uint4 *>(p.Xq + (size_t)(m0 + row) * Kh) + chunk;
        a_dst[i] = (((row >> 5) * 4 + chunk) << 10) + ((row & 31) << 4);
        if (u >= A_UNITS) a_dst[i] = -1;
    }
    const uint4 *b_src[B_LOADS];
    int b_dst[B_LOADS], b_chunk[B_LOADS];
    bool b_ok[B_LOADS];
#pragma unroll
    for (int i = 0; i < B_LOADS; ++i) {
        const int u = i * 256 + t;
        const int ngl = u >> 7, rem = u & 127;
        b_ok[i] = (u < B_UNITS) && (ng0 + ngl < p.n_groups);
        b_chunk[i] = rem >> 5;
        b_src[i] = reinterpret_cast<const uint4 *>(p.Wd + ((size_t)(ng0 + ngl) * p.chunks) * 512) + rem;
        b_dst[i] = A_BYTES + ((ngl * 4 + (rem >> 5)) << 10) + ((rem & 31) << 4);
        if (u >= B_UNITS) b_dst[i] = -1;
    }

    v16i acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int jn = 0; jn < TN; ++jn)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][jn][e] = 0;

    uint4 ga[A_LOADS], gb[B_LOADS];
    const uint4 zero4 = make_uint4(0, 0, 0, 0);
    const int steps = (p.chunks + kChunksPerStep - 1) / kChunksPerStep;   // a ragged last step reads zeros

    auto load_global = [&](int step) {
#pragma unroll
        for (int i = 0; i < A_LOADS; ++i)
            ga[i] = (a_ok[i] && step * kChunksPerStep + a_chunk[i] < p.chunks) ? a_src[i][step * kChunksPerStep]
                                                                              : zero4;
#pragma unroll
        for (int i = 0; i < B_LOADS; ++i)
            gb[i] = (b_ok[i] && step * kChunksPerStep + b_chunk[i] < p.chunks)
                        ? b_src[i][step * kChunksPerStep * 32]
                        : zero4;
    };
    auto store_lds = [&](int stage) {
        uint8_t *base = smem + stage * STAGE;
#pragma unroll
        for (int i = 0; i < A_LOADS; ++i) {
            if (a_dst[i] >= 0) {
                v4i lo, hi;
                widen(ga[i], lo, hi);
                *reinterpret_cast<v4i *>(base + a_dst[i]) = lo;
                *reinterpret_cast<v4i *>(base + a_dst[i] + 512) = hi;
            }
        }
#pragma unroll
        for (int i = 0; i < B_LOADS; ++i) {
            if (b_dst[i] >= 0) {
                v4i lo, hi;
                widen(gb[i], lo, hi);
                *reinterpret_cast<v4i *>(base + b_dst[i]) = lo;
                *reinterpret_cast<v4i *>(base + b_dst[i] + 512) = hi;
            }
        }
    };

    load_global(0);
    store_lds(0);
    if (steps > 1) load_global(1);
    __syncthreads();

    for (int it = 0; it < steps; ++it) {
        const int cur = it & 1;
        if (it + 1 < steps) store_lds(cur ^ 1);
        if (it + 2 < steps) load_global(it + 2);
        const uint8_t *sa = smem + cur * STAGE + ((wm * TM * 4) << 10) + (lane << 4);
        const uint8_t *sb = smem + cur * STAGE + A_BYTES + ((wn * TN * 4) << 10) + (lane << 4);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            v4i af[TM], bf[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) af[i] = *reinterpret_cast<const v4i *>(sa + ((i * 4 + ks) << 10));
#pragma unroll
            for (int jn = 0; jn < TN; ++jn) bf[jn] = *reinterpret_cast<const v4i *>(sb + ((jn * 4 + ks) << 10));
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int jn = 0; jn < TN; ++jn)
                    acc[i][jn] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[i], bf[jn], acc[i][jn], 0, 0, 0);
        }
        __syncthreads();
    }

    // Epilogue.  In a 32x32 accumulator tile lane l, register e holds
    // row 8*(e/4) + 4*(l/32) + (e%4), column l%32.
    const int col_in = lane & 31, row_half = (lane >> 5) * 4;
#pragma unroll
    for (int jn = 0; jn < TN; ++jn) {
        const int col = (ng0 << 5) + wn * WN + jn * 32 + col_in;
        const bool col_ok = col < p.N;
        const float swf = col_ok ? __half2float(p.sw[col]) : 0.f;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int row = m0 + wm * WM + i * 32 + ((e >> 2) << 3) + row_half + (e & 3);
                if (col_ok && row < p.M) {
                    const int a = acc[i][jn][e] >> 8;
                    const float sxf = __half2float(p.sx[row]);
                    p.Y[(size_t)row * p.ldy + col] = dequant(a, sxf, swf);
                    if (p.acc_out) p.acc_out[(size_t)row * p.N + col] = a;
                }
            }
        }
    }
}

size_t linear_workspace_bytes(int, int, int) { return 0; }

template <int BM, int BN>
static sqap_status launch_tiled(GemmParams &p, hipStream_t st)
{
    p.m_tiles = (p.M + BM - 1) / BM;
    p.n_tiles = (p.n_groups * 32 + BN - 1) / BN;
    const size_t lds = (size_t)2 * (BM + BN) * kBK;
    static bool configured = false;
    if (!configured) {
        SQAP_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_tiled_kernel<BM, BN>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        configured = true;
    }
    const int64_t blocks = (int64_t)p.m_tiles * p.n_tiles;
    if (blocks > 0x7fffffff) return fail(SQAP_EUNSUPPORTED, "sqap_w4a4_linear: too many tiles");
    hipLaunchKernelGGL((gemm_tiled_kernel<BM, BN>), dim3((unsigned)blocks), dim3(256), lds, st, p);
    SQAP_HIP_CHECK(hipGetLastError());
    return SQAP_OK;
}

sqap_status launch_w4a4_linear(const uint8_t *Xq, const __half *sx, int M, const Weight &w,
                               __half *Y, int64_t ldy, int32_t *acc_out, void *, hipStream_t st)
{
    if (w.K > kMaxK) return fail(SQAP_EUNSUPPORTED, "sqap_w4a4_linear: K = %d above %d", w.K, kMaxK);
    GemmParams p;
    p.Xq = Xq;
    p.sx = sx;
    p.Wd = w.data;
    p.sw = w.scales;
    p.Y = Y;
    p.acc_out = acc_out;
    p.ldy = ldy;
    p.M = M;
    p.N = w.N;
    p.K = w.K;
    p.n_groups = w.n_groups;
    p.chunks = w.chunks;
    if (M <= 64) return launch_tiled<64, 256>(p, st);
    if (M <= 128) return launch_tiled<128, 256>(p, st);
    return launch_tiled<256, 256>(p, st);
}

}  // namespace sqap
