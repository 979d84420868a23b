// W4A4 linear for a few hundred token rows (8 < M <= 640): every workgroup owns complete outputs.
//
// At these sizes the output is too small to fill the machine with whole 256 x 256 tiles, and splitting K
// between workgroups costs a chain of global round trips (partial store, flag, reduction) that is longer
// than the arithmetic.  Here nothing crosses a workgroup: a workgroup (one per compute unit, eight
// wavefronts, two per SIMD) owns a block of up to 160 token rows times a short run of 16-channel groups
// over the WHOLE reduction axis.  Wavefront w takes quarter w % 4 of K and half w / 4 of the block's token
// groups; the four wavefronts of a half add their accumulators through LDS at the end.  Two wavefronts per
// SIMD matter: one wavefront issues at most one instruction every four cycles, and the int4 -> int8 widening
// costs about 2.5 vector-ALU instructions per matrix instruction, so a lone wavefront leaves the matrix
// core idle half of the time; with two, one's widening issues beside the other's products.
// Inside a workgroup every token byte is used by exactly one wavefront and every weight byte by two, so
// the main loop has no workgroup barrier:
//   weights   come straight from global memory into registers: the packed layout already is the operand
//             order of v_mfma_i32_16x16x64_i8 (lane l: channel l % 16, 16-byte piece l / 16);
//   tokens    are read with coalesced loads (8 rows x 128 bytes per wavefront load), parked in a slab of
//             LDS that belongs to the wavefront, and read back in operand order (lane l: token l % 16,
//             piece l / 16).  A slab row has a pitch of 144 bytes, which keeps both the row-wise stores
//             and the column-wise reads free of bank conflicts.  The rows of a pair of 16-token groups are
//             overwritten with the next step's rows as soon as the pair's products are issued, and
//             the registers they came from are reloaded for the step after that.
// int4 -> int8 as in the large-M kernel: (x << 4) & 0xF0F0F0F0 and x & 0xF0F0F0F0 give 16 * code for the even
// and the odd codes; both operands are split the same way, so the accumulator is 256 * sum(x * w).
// The price is that every workgroup reads all its token rows for the whole K (they come from the L2,
// which the 32 workgroups of an XCD share).
#include "common.h"

namespace sqap {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int kRowsMaxAH = 5;          // 16-token groups per wavefront (a block of token rows has twice as many)
constexpr int kRowsMaxA = 2 * kRowsMaxAH;
constexpr int kRowsMaxB = 3;           // 16-channel groups per tile
constexpr int kRowsWaves = 8;
constexpr int kRowsStepCodes = 256;    // codes of K per main-loop step of a wavefront (two MFMA K-blocks of 128)
constexpr int kRowsPitch = 144;        // bytes per slab row: 128 of codes + 16 of padding
constexpr int kRowsSlabBytes = kRowsMaxAH * 16 * kRowsPitch;                           // 11520 per wavefront
constexpr int kRowsReduceBytes = kRowsWaves * kRowsMaxAH * kRowsMaxB * 1024;            // 8 wavefronts x 15 tiles x 1 KiB
constexpr int kRowsLdsBytes = kRowsReduceBytes > kRowsWaves * kRowsSlabBytes ? kRowsReduceBytes : kRowsWaves * kRowsSlabBytes;

struct RowsParams {
    const uint8_t *Xq;     // [M, K/2] canonical
    const __half *sx;      // [M]
    const uint8_t *Wd;     // streaming layout (see common.h)
    const __half *sw;      // padded to whole row groups
    __half *Y;
    int32_t *acc_out;      // nullable
    int64_t ldy;
    int M, N, K, chunks;
    int c16;               // 16-channel groups: ceil(N / 16)
    int tblocks;           // blocks of token rows (1, 2 or 4)
    int rows_per_block;    // multiple of 16, at most 16 * kRowsMaxA
    int per_xcd;           // workgroups of an XCD that share its channel groups, per token block
};

__device__ __forceinline__ void widen16(const v4i p, v4i &lo, v4i &hi)
{
    const v4i mask = {(int)0xF0F0F0F0, (int)0xF0F0F0F0, (int)0xF0F0F0F0, (int)0xF0F0F0F0};
    lo = (p << 4) & mask;
    hi = p & mask;
}

// same two-step rounding as the large-M epilogue: two binary32 products, then one rounding to half
typedef float v2f_r __attribute__((ext_vector_type(2)));
typedef _Float16 v2h_r __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t dequant_pair(int acc0, int acc1, float sx_over_256, float sw0, float sw1)
{
    float y0 = ((float)acc0 * sx_over_256) * sw0;
    float y1 = ((float)acc1 * sx_over_256) * sw1;
    asm volatile("" : "+v"(y0), "+v"(y1));
    const v2f_r y = {y0, y1};
    union { v2h_r h; uint32_t u; } r;
    r.h = __builtin_convertvector(y, v2h_r);
    return r.u;
}

// One tile: token rows [row0, row0 + 32 AH), channel groups [c0, c0 + B), all of K.  AH and B are
// compile-time constants: every main-loop iteration then issues the same loads and stores in the same
// order, which lets the compiler give each wait the exact count of younger loads that may stay in flight
// (with loads under run-time conditions it waits for all of them, i.e. for a full memory round trip per
// token group).  Token groups are taken two at a time so that consecutive products go to different
// accumulators, and the next pair's operands are read from LDS before the current pair is multiplied.
template <int AH, int B>
__device__ __forceinline__ void rows_tile(const RowsParams &p, uint8_t *smem, int row0, int row_end, int c0)
{
    static_assert(AH >= 1 && AH <= kRowsMaxAH && B >= 1 && B <= kRowsMaxB, "tile shape");
    constexpr int PAIRS = (AH + 1) / 2;
    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int kq = wave & 3, th = wave >> 2;
    const int Kh = p.K >> 1;
    const int steps = p.K / kRowsStepCodes;
    const int s_begin = steps * kq / 4, s_end = steps * (kq + 1) / 4;
    // The wavefront takes its steps in rotated order, starting at a step that depends on the workgroup: all
    // workgroups of an XCD read the same token rows, and walking K in step they would all ask the same one
    // or two L2 channels for the same lines at the same time.
    const int nst = s_end - s_begin, rot = (int)(blockIdx.x >> 3) % nst;
    auto step_of = [&](int i) {                                     // i-th step of this wavefront (i past the end: the last)
        int v = min(i, nst - 1) + rot;
        if (v >= nst) v -= nst;
        return s_begin + v;
    };
    uint8_t *slab = smem + wave * kRowsSlabBytes;
    const int wrow0 = row0 + th * AH * 16;                          // this wavefront's first token row

    // token rows: wavefront load i covers rows 8 i .. 8 i + 7 of the wavefront's rows, 128 bytes of each.  Byte
    // offset of this lane's piece in load i: (wrow0 + 8 i + lane / 8) * Kh + 16 * (lane % 8); rows past M - 1
    // re-read row M - 1 (never stored): one addition and one minimum per load instead of a pointer per load.
    const int lr = lane >> 3, piece = lane & 7;
    const uint32_t xoff0 = (uint32_t)(wrow0 + lr) * (uint32_t)Kh + piece * 16;
    const uint32_t xlimit = (uint32_t)(p.M - 1) * (uint32_t)Kh + piece * 16;
    const uint8_t *xbase = p.Xq;
    auto x_ptr = [&](int i, int step) {           // uniform base + 32-bit lane offset: no 64-bit lane arithmetic
        const uint32_t off = min(xoff0 + (uint32_t)(i * 8) * (uint32_t)Kh, xlimit);
        return reinterpret_cast<const v4i *>(xbase + (size_t)step * 128 + off);
    };
    const int xdst = lr * kRowsPitch + piece * 16;                 // + i * 8 * pitch
    // operand order: lane l reads token l % 16, piece l / 16 (+ 4 for the second K-block of a step)
    const int xfrag = (lane & 15) * kRowsPitch + (lane >> 4) * 16;
    // weights: 16-channel group g = 2 * row group + half; chunk c of a row group sits at (rg * chunks + c) * 512
    // (uniform base per group + one 32-bit lane offset)
    const uint8_t *wbase[B];
#pragma unroll
    for (int j = 0; j < B; ++j) {
        const int g = c0 + j;
        wbase[j] = p.Wd + (size_t)(g >> 1) * p.chunks * 512 + (g & 1) * 256;
    }
    const uint32_t woff = (uint32_t)(lane >> 4) * 512 + (lane & 15) * 16;

    v4i acc[AH][B];
#pragma unroll
    for (int i = 0; i < AH; ++i)
#pragma unroll
        for (int j = 0; j < B; ++j) acc[i][j] = v4i{0, 0, 0, 0};

    v4i xr[2 * AH];                   // token rows of step s + 1 in flight
    v4i wr[2][2][B];                  // weights: step s in set s & 1 (used now), step s + 1 in the other; [K-block][group]
    v4i xf[2];                        // operands of the token-group pair about to be multiplied

    auto load_x = [&](int step) {
#pragma unroll
        for (int i = 0; i < 2 * AH; ++i) xr[i] = *x_ptr(i, step);
    };
    auto load_w = [&](int step, auto set_c, auto q_c) {
        constexpr int set = decltype(set_c)::value, q = decltype(q_c)::value;
#pragma unroll
        for (int j = 0; j < B; ++j)
            wr[set][q][j] = *reinterpret_cast<const v4i *>(wbase[j] + (size_t)(step * 8 + q * 4) * 512 + woff);
    };
    auto read_pair = [&](int ip, int q, v4i (&dst)[2]) {
#pragma unroll
        for (int g = 0; g < 2; ++g)
            if (2 * ip + g < AH)
                dst[g] = *reinterpret_cast<const v4i *>(slab + (2 * ip + g) * 16 * kRowsPitch + xfrag + q * 64);
    };

    constexpr std::integral_constant<int, 0> c0_{};
    constexpr std::integral_constant<int, 1> c1_{};
    // prologue: step s_begin goes to the slab, step s_begin + 1 stays in the registers
    load_x(step_of(0));
    load_w(step_of(0), c0_, c0_);
    load_w(step_of(0), c0_, c1_);
    load_w(step_of(1), c1_, c0_);
    load_w(step_of(1), c1_, c1_);
#pragma unroll
    for (int i = 0; i < 2 * AH; ++i) *reinterpret_cast<v4i *>(slab + i * 8 * kRowsPitch + xdst) = xr[i];
    load_x(step_of(1));
    read_pair(0, 0, xf);

    // The i-th step of the wavefront; PAR = i & 1 names the register set that holds the step's weights.
    auto step_body = [&](int i, auto par_c) {
        constexpr int PAR = decltype(par_c)::value;
        constexpr std::integral_constant<int, PAR> cur{};
        const int s2 = step_of(i + 2);
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            v4i wl[B], wh[B];
#pragma unroll
            for (int j = 0; j < B; ++j) widen16(wr[PAR][q][j], wl[j], wh[j]);
            // the registers just consumed take the step after next
            if (q == 0) load_w(s2, cur, c0_);
            else load_w(s2, cur, c1_);
#pragma unroll
            for (int ip = 0; ip < PAIRS; ++ip) {
                v4i nx[2];
                if (ip + 1 < PAIRS) read_pair(ip + 1, q, nx);
                else if (q == 0) read_pair(0, 1, nx);
                v4i xl[2], xh[2];
#pragma unroll
                for (int g = 0; g < 2; ++g)
                    if (2 * ip + g < AH) widen16(xf[g], xl[g], xh[g]);
#pragma unroll
                for (int j = 0; j < B; ++j)
#pragma unroll
                    for (int g = 0; g < 2; ++g)
                        if (2 * ip + g < AH)
                            acc[2 * ip + g][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wl[j], xl[g], acc[2 * ip + g][j], 0, 0, 0);
#pragma unroll
                for (int j = 0; j < B; ++j)
#pragma unroll
                    for (int g = 0; g < 2; ++g)
                        if (2 * ip + g < AH)
                            acc[2 * ip + g][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wh[j], xh[g], acc[2 * ip + g][j], 0, 0, 0);
                if (q == 1) {
                    // both K-blocks of this pair's rows are consumed: the next step's rows take their place in
                    // the slab and the registers they came from are asked for the step after that
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (4 * ip + r < 2 * AH) {
                            *reinterpret_cast<v4i *>(slab + (4 * ip + r) * 8 * kRowsPitch + xdst) = xr[4 * ip + r];
                            xr[4 * ip + r] = *x_ptr(4 * ip + r, s2);
                        }
                }
                if (ip + 1 < PAIRS || q == 0) {
                    xf[0] = nx[0];
                    xf[1] = nx[1];
                }
            }
        }
        read_pair(0, 0, xf);                         // the next step's first pair (its rows were stored above)
    };
    int i = 0;
    for (; i + 1 < nst; i += 2) {
        step_body(i, c0_);
        step_body(i + 1, c1_);
    }
    if (i < nst) step_body(i, c0_);

    // add the accumulators of the four wavefronts that share a token half through LDS; wavefront (kq, th)
    // finishes tiles kq, kq + 4, ... of its half
    __syncthreads();                                   // every wavefront is done with its slab
    int *red = reinterpret_cast<int *>(smem);
#pragma unroll
    for (int i = 0; i < AH; ++i)
#pragma unroll
        for (int j = 0; j < B; ++j)
            *reinterpret_cast<v4i *>(red + ((wave * AH * B + i * B + j) * 64 + lane) * 4) = acc[i][j];
    __syncthreads();
    const int tok_in = lane & 15, ch4 = (lane >> 4) * 4;
    const bool y_vec = (p.ldy & 3) == 0 && (reinterpret_cast<uintptr_t>(p.Y) & 7u) == 0;
    const bool a_vec = (p.N & 3) == 0 && p.acc_out && (reinterpret_cast<uintptr_t>(p.acc_out) & 15u) == 0;
    for (int tt = kq; tt < AH * B; tt += 4) {
        const int i = tt / B, j = tt - i * B;
        v4i sum = {0, 0, 0, 0};
#pragma unroll
        for (int w = 0; w < 4; ++w)
            sum += *reinterpret_cast<const v4i *>(red + (((th * 4 + w) * AH * B + tt) * 64 + lane) * 4);
        const int row = wrow0 + i * 16 + tok_in, col = (c0 + j) * 16 + ch4;
        if (row < row_end && col < p.N) {
            const float sxf = __half2float(p.sx[row]) * 0.00390625f;
            const uint2 swr = *reinterpret_cast<const uint2 *>(p.sw + col);            // zero padded past N
            const __half2 *sw2 = reinterpret_cast<const __half2 *>(&swr);
            const float2 s01 = __half22float2(sw2[0]), s23 = __half22float2(sw2[1]);
            uint2 pk;
            pk.x = dequant_pair(sum.x, sum.y, sxf, s01.x, s01.y);
            pk.y = dequant_pair(sum.z, sum.w, sxf, s23.x, s23.y);
            __half *dst = p.Y + (size_t)row * p.ldy + col;
            if (y_vec && col + 4 <= p.N) {
                *reinterpret_cast<uint2 *>(dst) = pk;
            } else {
                const __half *h = reinterpret_cast<const __half *>(&pk);
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (col + e < p.N) dst[e] = h[e];
            }
            if (p.acc_out) {
                int32_t *ad = p.acc_out + (size_t)row * p.N + col;
                const v4i v = {sum.x >> 8, sum.y >> 8, sum.z >> 8, sum.w >> 8};
                if (a_vec && col + 4 <= p.N) {
                    *reinterpret_cast<v4i *>(ad) = v;
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (col + e < p.N) ad[e] = v[e];
                }
            }
        }
    }
    __syncthreads();                                   // LDS is free for the next tile
}

// Workgroup b runs on XCD b % 8 (the hardware deals consecutive workgroups to the XCDs in turn; nothing
// here depends on it for correctness, only for locality).  The 16-channel groups are dealt to the XCDs in
// contiguous runs, and inside an XCD to `per_xcd` workgroups per token block, so that the workgroups that
// read the same weights (one per token block) sit behind one L2.  AH = 16-token groups per wavefront: a
// block has 2 AH of them (rows past the block re-read other rows and are never stored).
template <int AH>
__global__ __launch_bounds__(64 * kRowsWaves, 1) void gemm_rows_kernel(const RowsParams p)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
    const int tb = j % p.tblocks, slot = j / p.tblocks;
    if (slot >= p.per_xcd) return;
    const int W = 8 * p.per_xcd, i = xcd * p.per_xcd + slot;
    const int g_begin = (int)((long long)p.c16 * i / W), g_end = (int)((long long)p.c16 * (i + 1) / W);
    const int row0 = tb * p.rows_per_block;
    if (row0 >= p.M) return;
    const int row_end = min(p.M, row0 + p.rows_per_block);      // rows past it belong to the next block (or to nobody)
    // tiles of at most kRowsMaxB groups, as even as possible (5 -> 3 + 2, 4 -> 2 + 2)
    const int n = g_end - g_begin, tiles = (n + kRowsMaxB - 1) / kRowsMaxB;
    for (int k = 0; k < tiles; ++k) {
        const int c0 = g_begin + n * k / tiles, b = g_begin + n * (k + 1) / tiles - c0;
        if (b == 3) rows_tile<AH, 3>(p, smem, row0, row_end, c0);
        else if (b == 2) rows_tile<AH, 2>(p, smem, row0, row_end, c0);
        else rows_tile<AH, 1>(p, smem, row0, row_end, c0);
    }
}

// Token blocks: as few as hold M, more when the channel groups are too few to give every workgroup a run
// of its own (each workgroup then reads fewer token rows, and the weights are read once per block, the
// second time from the L2).  Cost of a workgroup in clock cycles: what its compute unit loads at 64 bytes
// per cycle against what its matrix cores multiply (a 16 x 16 x 64 product takes 16 cycles on one of four SIMDs).
// Only plans in which a workgroup's channel groups fit ONE tile are taken: a second tile reads the token
// rows again and pays the start-up of the load pipeline again, and measured slower than the tile kernels
// that split K between workgroups (N = 22016 at M = 148: 28.6 against 28.3 us; N = 32000: 42 against 30 us),
// while single-tile shapes measured 25-45 % faster (N = 4096: 9.1 against 15.0 us, N = 12288: 15.7 against
// 20.8 us, K = 11008: 15.2 against 22.1 us, all at M = 148).
static bool rows_plan(int M, int N, int K, int cus, RowsParams *p)
{
    if (M <= kSkinnyMaxM || K % kRowsStepCodes != 0 || K / kRowsStepCodes < 4 || N < 16) return false;
    const int c16 = (N + 15) / 16;
    double best = 0.0;
    for (int tb = 1; tb <= 4; tb *= 2) {
        const int rows = ((M + tb - 1) / tb + 15) / 16 * 16;
        if (rows > 16 * kRowsMaxA) continue;
        const int a = (rows / 16 + 1) & ~1;                     // two wavefront halves of equal size
        int per_xcd = (cus / 8) / tb;
        if (per_xcd < 1) per_xcd = 1;
        const int W = 8 * per_xcd;
        const int n = (c16 + W - 1) / W;
        if (n > kRowsMaxB) continue;                            // more than one tile per workgroup
        const double bytes = (a * 16.0 + 2 * 16.0 * n) * (K / 2);
        const double mfma = (double)a * n * (K / 128) * 2 * 16 / 4;
        const double cost = std::max(bytes / 64.0, mfma / 0.7);
        if (best == 0.0 || cost < best) {
            best = cost;
            p->tblocks = tb;
            p->rows_per_block = rows;
            p->per_xcd = per_xcd;
        }
    }
    p->c16 = c16;
    return best > 0.0;
}

static int rows_cus()
{
    int cus = device_cu_count();
    return cus > 256 ? 256 : cus < 8 ? 8 : cus;
}

// Shapes this kernel takes: K a multiple of 256 with at least one step per wavefront, up to four blocks of 160
// token rows, and few enough channels that every workgroup has a single tile.
bool rows_kernel_applies(int M, int N, int K)
{
    RowsParams p = {};
    return rows_plan(M, N, K, rows_cus(), &p);
}

template <int AH>
static sqap_status launch_rows_a(const RowsParams &p, int blocks, hipStream_t st)
{
    static std::atomic<bool> configured[kMaxDeviceSlots];
    const int dslot = device_slot();
    if (!configured[dslot].load(std::memory_order_acquire)) {
        SQAP_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_rows_kernel<AH>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kRowsLdsBytes));
        configured[dslot].store(true, std::memory_order_release);
    }
    hipLaunchKernelGGL((gemm_rows_kernel<AH>), dim3(blocks), dim3(64 * kRowsWaves), kRowsLdsBytes, st, p);
    SQAP_HIP_CHECK(hipGetLastError());
    return SQAP_OK;
}

sqap_status launch_rows_linear(const uint8_t *Xq, const __half *sx, int M, const Weight &w, __half *Y, int64_t ldy,
                               int32_t *acc_out, hipStream_t st)
{
    RowsParams p = {};
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
    p.chunks = w.chunks;
    if (!rows_plan(M, w.N, w.K, rows_cus(), &p))
        return fail(SQAP_EUNSUPPORTED, "sqap_w4a4_linear: M = %d, N = %d, K = %d outside the row kernel's range", M, w.N, w.K);
    const int blocks = 8 * p.per_xcd * p.tblocks;
    const int ah = (p.rows_per_block / 16 + 1) / 2;             // token groups per wavefront
    switch (ah) {
    case 1: return launch_rows_a<1>(p, blocks, st);
    case 2: return launch_rows_a<2>(p, blocks, st);
    case 3: return launch_rows_a<3>(p, blocks, st);
    case 4: return launch_rows_a<4>(p, blocks, st);
    default: return launch_rows_a<5>(p, blocks, st);
    }
}

}  // namespace sqap
