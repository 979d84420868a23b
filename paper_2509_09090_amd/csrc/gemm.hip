// W4A4 linear: acc = Xq * Wq^T exactly in int32 on the int8 MFMA units, with
// the per-token x per-channel dequantisation fused into the epilogue.
//
// CDNA4 has no int4 MFMA, so both operands are widened on the fly.  A 16-byte
// piece of a packed row holds 32 codes; `(x << 4) & 0xF0F0F0F0` turns the 16
// low nibbles into 16 int8 values equal to 16 * code (the nibble's sign bit
// lands on the byte's sign bit) and `x & 0xF0F0F0F0` does the same for the high
// nibbles.  The low-nibble bytes feed one 32x32x32 MFMA and the high-nibble
// bytes a second one; the activation rows are split the same way, so every
// product pairs codes of the same k.  The accumulator is then 256 * sum(x*w),
// |.| <= 256 * 64 * K < 2^31 for K <= 131071, and the epilogue shifts it back:
// the integer result is exact.
#include <atomic>
#include <cstdlib>
#include <algorithm>
#include <map>
#include <mutex>
#include <random>
#include <tuple>
#include <type_traits>
#include <vector>

#include "common.h"

namespace sqap {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kBK = 128;            // codes of the reduction axis per main-loop step
constexpr int kChunksPerStep = 4;   // = kBK / 32, 16-byte packed pieces per row per step
constexpr int kMaxK = 131040;       // keeps 256 * 64 * K below 2^31

// Persistent (stream-K) launch: at most this many workgroups, 8 XCDs.
constexpr int kMaxPersistentBlocks = 256;
constexpr int kXcds = 8;
// Workspace header, in 64-bit words: [0, 256) one flag per workgroup (256 x 256 tiles), 500 the
// error word, [512, 1024) arrival and [1024, 1536) departure flags of the narrow-tile kernel
// (one per partial slot: 2 x 256).
constexpr size_t kFlagBytes = 16384;
constexpr int kErrWord = 500;
constexpr int kArriveWord = 512;
constexpr int kDepartWord = 1024;
constexpr int kStreamKMinM = 512;           // from this M on the persistent kernel is used
constexpr long long kSpinLimit = 2000000;   // bounded wait: a poll is a short sleep plus one L2 round trip, about 2 us, so a few seconds

// Shares of the stream-K kernel: workgroup j of XCD x runs main-loop steps [bounds[x][j], bounds[x][j + 1]) of
// that XCD's tiles (numbered tile after tile).  Passed by value as a kernel argument.
struct StreamKShares {
    uint32_t bounds[kXcds][kMaxPersistentBlocks / kXcds + 1];
};

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
    bool y_vec_ok;         // Y and its pitch are 16-byte aligned
    // persistent kernel only
    unsigned long long *flags;   // workspace header: one 64-bit flag per workgroup
    unsigned long long epoch;    // value that marks a flag as set by THIS launch
    uint8_t *partials;     // one BM x BN int32 slot per workgroup
    int blocks_per_xcd;
};

// Error word of the workspace header.  The first workgroup of a persistent launch clears it when it starts and a
// wait that gives up writes the launch's (nonzero) epoch, both as agent-scope stores (written through to
// memory, so the later store is the one that stays whichever XCD issued it): after a launch the word is
// zero, or that launch gave up a wait and its output is wrong, whatever the workspace held before.
__device__ __forceinline__ void clear_error_word(const GemmParams &p)
{
    if (blockIdx.x == 0 && threadIdx.x == 0)
        __hip_atomic_store(&p.flags[kErrWord], 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void raise_error_word(const GemmParams &p)
{
    __hip_atomic_store(&p.flags[kErrWord], p.epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ void widen(const v4i p, v4i &lo, v4i &hi)
{
    const v4i mask = {(int)0xF0F0F0F0, (int)0xF0F0F0F0, (int)0xF0F0F0F0, (int)0xF0F0F0F0};
    lo = (p << 4) & mask;
    hi = p & mask;
}

// Y = half((float(acc >> 8) * sx) * sw): two binary32 products, then one rounding to
// half.  The accumulator is 256 * v with |v| < 2^23, so float(acc) = 256 * float(v)
// exactly, and with the token scale pre-multiplied by 2^-8 (exact: it is at least 2^-24)
// the first product is the same real number, hence the same float, without the shift.
// The empty asm keeps the compiler from folding the second product and the conversion
// into v_fma_mixlo_f16, which rounds the exact product once and so differs from the
// two-step definition in about one result in 2^13.  Two results are converted at a time
// (v_cvt_pk_f16_f32, round to nearest even).
typedef float v2f __attribute__((ext_vector_type(2)));
typedef _Float16 v2h __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t dequant2(int acc0, int acc1, float sx_over_256, float sw0, float sw1)
{
    float y0 = ((float)acc0 * sx_over_256) * sw0;
    float y1 = ((float)acc1 * sx_over_256) * sw1;
    asm volatile("" : "+v"(y0), "+v"(y1));
    const v2f y = {y0, y1};
    union { v2h h; uint32_t u; } r;
    r.h = __builtin_convertvector(y, v2h);
    return r.u;
}

// Static shape of one tile configuration: block tile BM x BN, WAVES_M x WAVES_N
// wavefronts, each owning (BM/WAVES_M) x (BN/WAVES_N) as 32x32 MFMA tiles.
template <int BM_, int BN_, int WAVES_M_, int WAVES_N_>
struct Cfg {
    static constexpr int BM = BM_, BN = BN_, WAVES_M = WAVES_M_, WAVES_N = WAVES_N_;
    static constexpr int NW = WAVES_M * WAVES_N, THREADS = NW * 64;
    static constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    static constexpr int TM = WM / 32, TN = WN / 32;
    static constexpr int CP = kChunksPerStep / 2;                 // chunk pairs per step
    static constexpr int A_FRAGS = (BM / 32) * CP, B_FRAGS = (BN / 32) * CP;
    static constexpr int A_BYTES = A_FRAGS * 1024, B_BYTES = B_FRAGS * 1024;
    static constexpr int STAGE = A_BYTES + B_BYTES;
    static constexpr int A_LOADS = (A_FRAGS + NW - 1) / NW, B_LOADS = (B_FRAGS + NW - 1) / NW;
    static_assert(B_FRAGS % NW == 0, "weight fragments divide over the wavefronts");
    static constexpr bool A_EVEN = A_FRAGS % NW == 0;           // else the last slots of some wavefronts are idle
    // epilogue staging: 32 rows of each wavefront's tile in halves (+16 bytes of
    // padding per row) followed by BM token scales and BN channel scales as floats
    static constexpr int EP_PITCH = WN * 2 + 16;
    static constexpr int EP_BYTES = NW * 32 * EP_PITCH + (BM + BN) * 4;
    static constexpr int PIPE_BYTES = 2 * STAGE;                  // two stages
    static constexpr int LDS_BYTES = PIPE_BYTES > EP_BYTES ? PIPE_BYTES : EP_BYTES;
};

// Main loop over steps [step_begin, step_end) of one tile (one step = 128
// codes of K), accumulating into acc.
//
// Operands stay PACKED in LDS (half the LDS traffic of int8) and are widened
// in registers right before the MFMAs.  LDS holds two stages in "fragment
// order": for row group rg (32 rows) and chunk pair cp (2 x 32 codes) the 1 KiB
// at ((rg * 2 + cp) * 1024) is what one ds_read_b128 of a wavefront fetches
// (lane l at l * 16): lanes 0-31 hold rows 0-31 of chunk 2cp, lanes 32-63 the
// same rows of chunk 2cp+1.  Widening a lane's 16 bytes gives its operand for
// two MFMAs: the even codes (both chunks, across the two lane halves) and the
// odd codes.  The weight layout in global memory is already in this order, so
// its path global -> register -> LDS is a straight 1 KiB copy per wavefront.
//
// The MFMAs take the WEIGHT fragment first, so an accumulator tile is the
// transpose of the output tile (see the epilogue).
//
// Rows: the wavefront in row wm of the wavefront grid owns row groups wm, wm + WAVES_M, wm + 2 WAVES_M,
// ... of the tile (accumulator i = row group i * WAVES_M + wm), so the few valid row groups of a ragged
// last tile are spread over all wavefronts (see mainloop_ragged).
//
// Loads are unguarded in M and N: rows past M re-read row M-1 and row groups
// past the end exist as zero padding in the weight layout; what they produce
// lands in accumulators that are never stored.  RAGGED_K = true guards the
// reduction axis (K not a multiple of 128) and is the slow, general variant.
//
// Pipeline: while stage `cur` feeds the MFMAs, the registers loaded one step
// ago are copied into the other stage and the loads for two steps ahead are
// issued.  One barrier per step; a trailing barrier leaves LDS free.
template <class C>
struct OperandMover {
    // Wavefront w moves fragments w*LOADS .. w*LOADS+LOADS-1 of each operand (when the
    // A fragments do not divide evenly, slots past the last fragment load it again and
    // are not stored).
    const v4i *a_src[C::A_LOADS];
    int a_dst[C::A_LOADS], a_chunk[C::A_LOADS];
    bool a_live[C::A_LOADS];
    const v4i *b_src[C::B_LOADS];
    int b_dst[C::B_LOADS], b_chunk[C::B_LOADS];

    // groups: row groups of the tile that hold tokens (fragments of the others are not moved)
    __device__ __forceinline__ OperandMover(const GemmParams &p, int m0, int ng0, int groups)
    {
        constexpr int CP = C::CP;
        const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
        const int Kh = p.K >> 1;
#pragma unroll
        for (int i = 0; i < C::A_LOADS; ++i) {
            const int f = min(wave * C::A_LOADS + i, C::A_FRAGS - 1), rg = f / CP, cp = f % CP;
            a_live[i] = wave * C::A_LOADS + i < C::A_FRAGS && rg < groups;
            const int grow = min(m0 + rg * 32 + (lane & 31), p.M - 1);
            a_chunk[i] = 2 * cp + (lane >> 5);
            a_src[i] = reinterpret_cast<const v4i *>(p.Xq + (size_t)grow * Kh) + a_chunk[i];
            a_dst[i] = (f << 10) + (lane << 4);
        }
#pragma unroll
        for (int i = 0; i < C::B_LOADS; ++i) {
            const int f = wave * C::B_LOADS + i, rg = f / CP, cp = f % CP;
            b_chunk[i] = 2 * cp + (lane >> 5);
            b_src[i] = reinterpret_cast<const v4i *>(p.Wd + ((size_t)(ng0 + rg) * p.chunks + 2 * cp) * 512) + lane;
            b_dst[i] = C::A_BYTES + (f << 10) + (lane << 4);
        }
    }
};

template <class C, bool RAGGED_K>
__device__ __forceinline__ void mainloop(const GemmParams &p, uint8_t *smem, int m0, int ng0, int step_begin,
                                         int step_end, v16i (&acc)[C::TM][C::TN])
{
    constexpr int TM = C::TM, TN = C::TN, CP = C::CP;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave / C::WAVES_N, wn = wave % C::WAVES_N;
    const OperandMover<C> mv(p, m0, ng0, C::BM / 32);

    // Register sets for operands in flight.  The narrow tiles (one row of wavefronts; a few hundred token
    // rows) have short steps and use two sets, so that a load has two steps to arrive (3-6 % faster at
    // M = 84 and 276); the 256 x 256 tiles use one (two measured 2.5 % slower there).
    constexpr int SETS = C::WAVES_M == 1 ? 2 : 1;
    v4i ga[SETS][C::A_LOADS], gb[SETS][C::B_LOADS];

    auto load_global = [&](int step, auto set_c) {
        constexpr int set = decltype(set_c)::value;
        const v4i zero4 = {0, 0, 0, 0};
#pragma unroll
        for (int i = 0; i < C::A_LOADS; ++i) {
            if (!RAGGED_K || step * kChunksPerStep + mv.a_chunk[i] < p.chunks)
                ga[set][i] = mv.a_src[i][step * kChunksPerStep];
            else
                ga[set][i] = zero4;
        }
#pragma unroll
        for (int i = 0; i < C::B_LOADS; ++i) {
            if (!RAGGED_K || step * kChunksPerStep + mv.b_chunk[i] < p.chunks)
                gb[set][i] = mv.b_src[i][step * kChunksPerStep * 32];
            else
                gb[set][i] = zero4;
        }
    };
    auto store_lds = [&](int stage, auto set_c) {
        constexpr int set = decltype(set_c)::value;
        uint8_t *base = smem + stage * C::STAGE;
#pragma unroll
        for (int i = 0; i < C::A_LOADS; ++i)
            if (C::A_EVEN || mv.a_live[i]) *reinterpret_cast<v4i *>(base + mv.a_dst[i]) = ga[set][i];
#pragma unroll
        for (int i = 0; i < C::B_LOADS; ++i) *reinterpret_cast<v4i *>(base + mv.b_dst[i]) = gb[set][i];
    };
    auto compute = [&](int stage) {
        const uint8_t *sa = smem + stage * C::STAGE + ((wm * CP) << 10) + (lane << 4);
        const uint8_t *sb = smem + stage * C::STAGE + C::A_BYTES + ((wn * TN * CP) << 10) + (lane << 4);
#pragma unroll
        for (int cp = 0; cp < CP; ++cp) {
            v4i alo[TM], ahi[TM], blo[TN], bhi[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i)
                widen(*reinterpret_cast<const v4i *>(sa + ((i * C::WAVES_M * CP + cp) << 10)), alo[i], ahi[i]);
#pragma unroll
            for (int jn = 0; jn < TN; ++jn)
                widen(*reinterpret_cast<const v4i *>(sb + ((jn * CP + cp) << 10)), blo[jn], bhi[jn]);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int jn = 0; jn < TN; ++jn)
                    acc[i][jn] = __builtin_amdgcn_mfma_i32_32x32x32_i8(blo[jn], alo[i], acc[i][jn], 0, 0, 0);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int jn = 0; jn < TN; ++jn)
                    acc[i][jn] = __builtin_amdgcn_mfma_i32_32x32x32_i8(bhi[jn], ahi[i], acc[i][jn], 0, 0, 0);
        }
    };

    constexpr std::integral_constant<int, 0> set0{};
    int it = step_begin, stage = 0;
    if constexpr (SETS == 2) {
        // Step s of the segment travels in set (s - step_begin) & 1.  Loads past the end of the segment
        // re-read its last step (and are dropped): every iteration issues the same loads, so the wait
        // before a copy to LDS lets exactly the one younger step stay in flight.  (Two steps per trip and
        // a single loop exit: with an exit between the halves the accumulators get copied.)
        constexpr std::integral_constant<int, 1> set1{};
        const int last = step_end - 1;
        load_global(step_begin, set0);
        store_lds(0, set0);
        load_global(min(step_begin + 1, last), set1);
        load_global(min(step_begin + 2, last), set0);
        __syncthreads();
        auto body = [&](auto set) {
            store_lds(stage ^ 1, set);
            __builtin_amdgcn_sched_barrier(0);
            load_global(min(it + 3, last), set);
            __builtin_amdgcn_sched_barrier(0);
            compute(stage);
            __syncthreads();
            stage ^= 1;
            ++it;
        };
        while (it + 2 < step_end) {
            body(set1);
            body(set0);
        }
        if (it + 1 < step_end) body(set1);
    } else {
        load_global(step_begin, set0);
        store_lds(0, set0);
        if (step_begin + 1 < step_end) load_global(step_begin + 1, set0);
        __syncthreads();
        for (; it + 2 < step_end; ++it) {
            store_lds(stage ^ 1, set0);
            __builtin_amdgcn_sched_barrier(0);
            load_global(it + 2, set0);
            __builtin_amdgcn_sched_barrier(0);
            compute(stage);
            __syncthreads();
            stage ^= 1;
        }
        if (it + 1 < step_end) {
            store_lds(stage ^ 1, set0);
            compute(stage);
            __syncthreads();
            stage ^= 1;
        }
    }
    compute(stage);
    __syncthreads();
}

// The same loop for a tile of the last tile row when only `groups` < BM / 32 of its row groups hold
// tokens: every wavefront runs NI = ceil(groups / WAVES_M) of its TM accumulator rows (a wavefront
// whose last one lies past `groups` multiplies stale LDS contents into an accumulator that is never
// stored).  Such a step has a quarter to three quarters of the MFMAs of a full one and is shorter
// than the round trip of a global load, so the operands travel in a ring of kRing register sets
// (the unused accumulator rows leave room for them): a load has kRing steps to arrive before it is
// copied to LDS.  Step s of the segment uses set (s - step_begin) % kRing; loads past the end of the
// segment re-read its last step and are dropped, so every iteration issues the same loads and the
// wait before a copy lets exactly the younger kRing - 1 steps stay in flight.
constexpr int kRing = 4;

template <class C, int NI>
__device__ __forceinline__ void mainloop_ragged(const GemmParams &p, uint8_t *smem, int m0, int ng0, int step_begin,
                                                int step_end, v16i (&acc)[C::TM][C::TN], int groups)
{
    constexpr int TN = C::TN, CP = C::CP;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave / C::WAVES_N, wn = wave % C::WAVES_N;
    const OperandMover<C> mv(p, m0, ng0, groups);

    v4i ga[kRing][C::A_LOADS], gb[kRing][C::B_LOADS];

    auto load_global = [&](int step, auto set_c) {
        constexpr int set = decltype(set_c)::value;
#pragma unroll
        for (int i = 0; i < C::A_LOADS; ++i) ga[set][i] = mv.a_src[i][step * kChunksPerStep];
#pragma unroll
        for (int i = 0; i < C::B_LOADS; ++i) gb[set][i] = mv.b_src[i][step * kChunksPerStep * 32];
    };
    auto store_lds = [&](int stage, auto set_c) {
        constexpr int set = decltype(set_c)::value;
        uint8_t *base = smem + stage * C::STAGE;
#pragma unroll
        for (int i = 0; i < C::A_LOADS; ++i)
            if (mv.a_live[i]) *reinterpret_cast<v4i *>(base + mv.a_dst[i]) = ga[set][i];
#pragma unroll
        for (int i = 0; i < C::B_LOADS; ++i) *reinterpret_cast<v4i *>(base + mv.b_dst[i]) = gb[set][i];
    };
    auto compute = [&](int stage) {
        const uint8_t *sa = smem + stage * C::STAGE + ((wm * CP) << 10) + (lane << 4);
        const uint8_t *sb = smem + stage * C::STAGE + C::A_BYTES + ((wn * TN * CP) << 10) + (lane << 4);
#pragma unroll
        for (int cp = 0; cp < CP; ++cp) {
            v4i alo[NI], ahi[NI], blo[TN], bhi[TN];
#pragma unroll
            for (int i = 0; i < NI; ++i)
                widen(*reinterpret_cast<const v4i *>(sa + ((i * C::WAVES_M * CP + cp) << 10)), alo[i], ahi[i]);
#pragma unroll
            for (int jn = 0; jn < TN; ++jn)
                widen(*reinterpret_cast<const v4i *>(sb + ((jn * CP + cp) << 10)), blo[jn], bhi[jn]);
#pragma unroll
            for (int i = 0; i < NI; ++i)
#pragma unroll
                for (int jn = 0; jn < TN; ++jn) {
                    acc[i][jn] = __builtin_amdgcn_mfma_i32_32x32x32_i8(blo[jn], alo[i], acc[i][jn], 0, 0, 0);
                    acc[i][jn] = __builtin_amdgcn_mfma_i32_32x32x32_i8(bhi[jn], ahi[i], acc[i][jn], 0, 0, 0);
                }
        }
    };

    constexpr std::integral_constant<int, 0> set0{};
    constexpr std::integral_constant<int, 1> set1{};
    constexpr std::integral_constant<int, 2> set2{};
    constexpr std::integral_constant<int, 3> set3{};
    static_assert(kRing == 4, "the loop below is unrolled for four register sets");
    const int last = step_end - 1;
    load_global(step_begin, set0);
    store_lds(0, set0);
    load_global(min(step_begin + 1, last), set1);
    load_global(min(step_begin + 2, last), set2);
    load_global(min(step_begin + 3, last), set3);
    load_global(min(step_begin + 4, last), set0);
    __syncthreads();
    int it = step_begin, stage = 0;
    auto body = [&](auto set) {               // the set holds step it + 1
        store_lds(stage ^ 1, set);
        __builtin_amdgcn_sched_barrier(0);
        load_global(min(it + 1 + kRing, last), set);
        __builtin_amdgcn_sched_barrier(0);
        compute(stage);
        __syncthreads();
        stage ^= 1;
        ++it;
    };
    while (it + kRing < step_end) {
        body(set1);
        body(set2);
        body(set3);
        body(set0);
    }
    const int rest = last - it;               // 0 .. kRing - 1 steps still to be staged
    if (rest >= 1) body(set1);
    if (rest >= 2) body(set2);
    if (rest >= 3) body(set3);
    compute(stage);
    __syncthreads();
}

// Picks the loop for a tile with `groups` valid row groups.
template <class C>
__device__ __forceinline__ void mainloop_rows(const GemmParams &p, uint8_t *smem, int m0, int ng0, int step_begin,
                                              int step_end, v16i (&acc)[C::TM][C::TN], int groups)
{
    if constexpr (C::WAVES_M > 1 && C::TM == 4) {
        const int ni = (groups + C::WAVES_M - 1) / C::WAVES_M;
        if (ni == 1) return mainloop_ragged<C, 1>(p, smem, m0, ng0, step_begin, step_end, acc, groups);
        if (ni == 2) return mainloop_ragged<C, 2>(p, smem, m0, ng0, step_begin, step_end, acc, groups);
        if (ni == 3) return mainloop_ragged<C, 3>(p, smem, m0, ng0, step_begin, step_end, acc, groups);
    }
    mainloop<C, false>(p, smem, m0, ng0, step_begin, step_end, acc);
}

// Epilogue: dequantise and store one wavefront's accumulators.  Called by every
// wavefront of the block (it contains barriers); LDS must be free on entry and
// is free again on return.
//
// Accumulator i of the wavefront in grid row wm is row group i * WAVES_M + wm of the block tile.
// An accumulator tile is the transpose of the output tile: lane l holds token
// row l%32 and, in register e, channel 8*(e/4) + 4*(l/32) + (e%4).  Four
// consecutive registers are four consecutive channels of one token: 8 bytes of
// halves, written to LDS in one piece and read back 16 bytes per lane so that
// a wavefront's global store covers whole rows of its tile.
template <class C>
__device__ __forceinline__ void epilogue(const GemmParams &p, v16i (&acc)[C::TM][C::TN], uint8_t *smem, int m0,
                                         int ng0)
{
    constexpr int TM = C::TM, TN = C::TN, WN = C::WN, PITCH = C::EP_PITCH;
    constexpr int LANES_PER_ROW = WN * 2 / 16;
    constexpr int ROWS_PER_PASS = 64 / LANES_PER_ROW;
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wm = wave / C::WAVES_N, wn = wave % C::WAVES_N;
    const int tok = lane & 31, ch4 = (lane >> 5) * 4;
    const int wave_col0 = (ng0 << 5) + wn * WN;

    if (p.acc_out) {
        const bool vec = (p.N & 3) == 0 && (reinterpret_cast<uintptr_t>(p.acc_out) & 15u) == 0;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int row = m0 + (i * C::WAVES_M + wm) * 32 + tok;
#pragma unroll
            for (int jn = 0; jn < TN; ++jn)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int col = wave_col0 + jn * 32 + q * 8 + ch4;
                    if (row < p.M && col < p.N) {
                        int32_t *dst = p.acc_out + (size_t)row * p.N + col;
                        v4i v = {acc[i][jn][4 * q] >> 8, acc[i][jn][4 * q + 1] >> 8, acc[i][jn][4 * q + 2] >> 8,
                                 acc[i][jn][4 * q + 3] >> 8};
                        if (vec) {
                            *reinterpret_cast<v4i *>(dst) = v;
                        } else {
#pragma unroll
                            for (int x = 0; x < 4; ++x)
                                if (col + x < p.N) dst[x] = v[x];
                        }
                    }
                }
        }
    }

    float *sxs = reinterpret_cast<float *>(smem + C::NW * 32 * PITCH);   // BM token scales, times 2^-8
    float *sws = sxs + C::BM;                                            // BN channel scales
    for (int r = t; r < C::BM; r += C::THREADS) sxs[r] = __half2float(p.sx[min(m0 + r, p.M - 1)]) * 0.00390625f;
    for (int c = t; c < C::BN; c += C::THREADS) sws[c] = __half2float(p.sw[(ng0 << 5) + c]);   // zero padded past N
    __syncthreads();
    uint8_t *ep = smem + wave * (32 * PITCH);
    const bool vec_ok = p.y_vec_ok;
    // This lane's channel scales are the same for every accumulator row: read once (the compiler cannot
    // move these reads above the staging writes itself, and a read in the loop costs an LDS round trip
    // per four channels).
    float4 sw4[TN * 4];
#pragma unroll
    for (int jn = 0; jn < TN; ++jn)
#pragma unroll
        for (int q = 0; q < 4; ++q)
            sw4[jn * 4 + q] = *reinterpret_cast<const float4 *>(&sws[wn * WN + jn * 32 + q * 8 + ch4]);
    // Whole tile inside the matrix and 16-byte stores possible (wave-uniform): no checks per store, and the
    // four row passes of an accumulator row are read together before they are stored.
    const bool inside = vec_ok && m0 + C::BM <= p.M && (ng0 << 5) + C::BN <= p.N;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int row0 = m0 + (i * C::WAVES_M + wm) * 32;
        if (row0 >= p.M) continue;                     // a row group without tokens (wave-uniform)
        const float sxf = sxs[(i * C::WAVES_M + wm) * 32 + tok];
#pragma unroll
        for (int jn = 0; jn < TN; ++jn)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int cin = jn * 32 + q * 8 + ch4;
                const float4 s4 = sw4[jn * 4 + q];
                uint2 pk;
                pk.x = dequant2(acc[i][jn][4 * q + 0], acc[i][jn][4 * q + 1], sxf, s4.x, s4.y);
                pk.y = dequant2(acc[i][jn][4 * q + 2], acc[i][jn][4 * q + 3], sxf, s4.z, s4.w);
                *reinterpret_cast<uint2 *>(ep + tok * PITCH + cin * 2) = pk;
            }
        // The staging area is private to the wavefront and LDS operations of one
        // wavefront complete in order, so no block barrier is needed around it.
        __builtin_amdgcn_wave_barrier();
        if (inside) {
            constexpr int PASSES = 32 / ROWS_PER_PASS;
            const int rin0 = lane / LANES_PER_ROW, cb = (lane % LANES_PER_ROW) * 16;
            __half *dst = p.Y + (size_t)(row0 + rin0) * p.ldy + wave_col0 + (cb >> 1);
            v4i v[PASSES];
#pragma unroll
            for (int ps = 0; ps < PASSES; ++ps)
                v[ps] = *reinterpret_cast<const v4i *>(ep + (ps * ROWS_PER_PASS + rin0) * PITCH + cb);
#pragma unroll
            for (int ps = 0; ps < PASSES; ++ps)
                __builtin_nontemporal_store(v[ps], reinterpret_cast<v4i *>(dst + (size_t)ps * ROWS_PER_PASS * p.ldy));
        } else {
#pragma unroll
            for (int ps = 0; ps < 32 / ROWS_PER_PASS; ++ps) {
                const int rin = ps * ROWS_PER_PASS + lane / LANES_PER_ROW;
                const int cb = (lane % LANES_PER_ROW) * 16;
                const int row = row0 + rin, col = wave_col0 + (cb >> 1);
                if (row < p.M && col < p.N) {
                    const v4i v = *reinterpret_cast<const v4i *>(ep + rin * PITCH + cb);
                    __half *dst = p.Y + (size_t)row * p.ldy + col;
                    if (vec_ok && col + 8 <= p.N) {
                        __builtin_nontemporal_store(v, reinterpret_cast<v4i *>(dst));
                    } else {
                        const __half *h = reinterpret_cast<const __half *>(&v);
#pragma unroll
                        for (int x = 0; x < 8; ++x)
                            if (col + x < p.N) dst[x] = h[x];
                    }
                }
            }
        }
        __builtin_amdgcn_wave_barrier();
    }
    __syncthreads();                                   // LDS is free again
}

template <class C>
__device__ __forceinline__ void zero_acc(v16i (&acc)[C::TM][C::TN])
{
#pragma unroll
    for (int i = 0; i < C::TM; ++i)
#pragma unroll
        for (int jn = 0; jn < C::TN; ++jn)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][jn][e] = 0;
}

// One tile per workgroup.  Tile order: the hardware deals consecutive
// workgroups to the 8 XCDs in turn; each XCD gets a contiguous run of tiles
// (n-tile major, m-tile minor) so that the tiles sharing a weight panel sit
// behind one L2.
template <class C, bool RAGGED_K>
__global__ __launch_bounds__(C::THREADS, 1) void gemm_tiled_kernel(const GemmParams p)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    const int tiles = p.m_tiles * p.n_tiles;
    const int bid = blockIdx.x;
    const int xcd = bid & 7, j = bid >> 3;
    const int q = tiles >> 3, r = tiles & 7;
    const int tile = xcd * q + (xcd < r ? xcd : r) + j;
    const int nt = tile / p.m_tiles, mt = tile - nt * p.m_tiles;
    const int m0 = mt * C::BM, ng0 = nt * (C::BN / 32);
    v16i acc[C::TM][C::TN];
    zero_acc<C>(acc);
    const int steps = (p.chunks + kChunksPerStep - 1) / kChunksPerStep;
    mainloop<C, RAGGED_K>(p, smem, m0, ng0, 0, steps, acc);
    epilogue<C>(p, acc, smem, m0, ng0);
}

// Persistent stream-K kernel.  The tiles are dealt to the 8 XCDs in whole
// tiles (contiguous runs, as above); inside an XCD the run's main-loop steps
// are split over that XCD's workgroups in consecutive shares (planned on the
// host and passed as a kernel argument, see plan_shares), so a tile may be shared
// by several workgroups.  The workgroup holding the LAST steps of a tile finishes
// it: it adds the partial accumulators the others left in the workspace (exact:
// integer sums commute) and runs the epilogue.  A workgroup computes a
// segment it does not finish FIRST and publishes it at once; the segment it
// finishes comes LAST.  A finisher therefore only ever waits for workgroups of
// its own XCD with a lower index, which were dispatched before it and publish
// before doing anything else, so the wait cannot deadlock; it is bounded all
// the same, and a timeout raises the error word in the workspace header.
template <class C>
__global__ __launch_bounds__(C::THREADS, 1) void gemm_streamk_kernel(const GemmParams p, const StreamKShares sched)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    const int t = threadIdx.x;
    const int tiles = p.m_tiles * p.n_tiles;
    const int steps = p.chunks / kChunksPerStep;
    const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
    // whole tiles of this XCD
    const int q = tiles >> 3, r = tiles & 7;
    const int tile0 = xcd * q + (xcd < r ? xcd : r);
    // This workgroup's share [begin, end) of the XCD's main-loop steps (tile after tile, `steps` each):
    // the host planned it (see plan_shares).
    const int begin = (int)sched.bounds[xcd][j], end = (int)sched.bounds[xcd][j + 1];
    clear_error_word(p);
    if (begin >= end) return;
    const int mtl = p.m_tiles;
    const int t_first = begin / steps, t_last = (end - 1) / steps;
    // steps [s0, s1) of XCD-local tile tl that fall to the share [b, e); tb = the tile's first step
    auto segment = [&](int b, int e, int tl, int &tb, int &s0, int &s1) {
        tb = tl * steps;
        s0 = min(max(b - tb, 0), steps);
        s1 = min(max(e - tb, 0), steps);
    };
    // valid row groups of a tile: all of them except in a ragged last tile row
    const int last_groups = (p.M - (mtl - 1) * C::BM + 31) >> 5;
    const int slot = blockIdx.x;

    // Visit order: downwards from t_last.  Only t_last can be left unfinished by
    // this workgroup (its steps end before the tile does), and only t_first can
    // need partial sums from others, so "publish first, finish last" holds.
    // The two cases are separate code regions (each with its own copy of the main
    // loop) because one region serving both needs more registers than there are.
    //
    // Slot layout: wavefront w, accumulator tile a, quarter q, lane l at
    // ((w * TM*TN + a) * 4 + q) * 1024 + l * 16 bytes: every store and load of a
    // wavefront is 1 KiB contiguous, and a tile's four pieces share one base.
    constexpr int SLOT_BYTES = C::BM * C::BN * 4;
    const int lane = t & 63, wave = t >> 6;
    const int my_off = wave * (C::TM * C::TN * 4096) + lane * 16;
    int tl = t_last;
    int tb, s0, s1;
    segment(begin, end, tl, tb, s0, s1);
    if (s1 < steps) {
        // not the finisher of t_last: compute the head segment and publish it
        const int tile = tile0 + tl;
        const int nt = tile / mtl, mt = tile - nt * mtl;
        --tl;
        if (s0 < s1) {
        v16i acc[C::TM][C::TN];
        zero_acc<C>(acc);
        mainloop_rows<C>(p, smem, mt * C::BM, nt * (C::BN / 32), s0, s1, acc, mt == mtl - 1 ? last_groups : C::BM / 32);
        uint8_t *dst = p.partials + (size_t)slot * SLOT_BYTES + my_off;
#pragma unroll
        for (int i = 0; i < C::TM; ++i)
#pragma unroll
            for (int jn = 0; jn < C::TN; ++jn) {
#pragma unroll
                for (int qd = 0; qd < 4; ++qd) {
                    v4i v = {acc[i][jn][4 * qd], acc[i][jn][4 * qd + 1], acc[i][jn][4 * qd + 2],
                             acc[i][jn][4 * qd + 3]};
                    *reinterpret_cast<v4i *>(dst + qd * 1024) = v;
                }
                dst += 4096;
            }
        // The consumers sit behind the same L2 (same XCD); the stores are complete
        // there once the vector-memory counter drains, and the flag goes out after that.
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (t == 0) __hip_atomic_store(&p.flags[slot], p.epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    for (; tl >= t_first; --tl) {
        segment(begin, end, tl, tb, s0, s1);           // s1 == steps: the share reaches past this tile
        if (s0 >= s1) continue;                        // no step of this tile starts inside the share
        const int tile = tile0 + tl;
        const int nt = tile / mtl, mt = tile - nt * mtl;
        const int m0 = mt * C::BM, ng0 = nt * (C::BN / 32);
        v16i acc[C::TM][C::TN];
        zero_acc<C>(acc);
        mainloop_rows<C>(p, smem, m0, ng0, s0, steps, acc, mt == mtl - 1 ? last_groups : C::BM / 32);
        if (s0 > 0) {
            // finisher of a shared tile: steps [0, s0) were done by lower workgroups of this XCD.
            // One lane per workgroup of the XCD (at most 32) looks up whether that workgroup holds
            // steps of this tile and waits for its flag: the waits overlap instead of costing one
            // memory round trip each.
            unsigned *share = reinterpret_cast<unsigned *>(smem);       // LDS is free between main loop and epilogue
            if (t < 64) {
                bool live = false;
                if (t < j) {
                    const int jb = (int)sched.bounds[xcd][t], je = (int)sched.bounds[xcd][t + 1];
                    live = jb < je && je > tb && jb < tb + s0;
                }
                if (live) {
                    unsigned long long *f = &p.flags[t * 8 + xcd];
                    long long spins = 0;
                    while (__hip_atomic_load(f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != p.epoch) {
                        __builtin_amdgcn_s_sleep(8);
                        if (++spins > kSpinLimit) {
                            raise_error_word(p);      // give up: the result of this tile is wrong
                            break;
                        }
                    }
                    // A flag has exactly one consumer.  Taking it down again makes a replay of
                    // a captured launch (same epoch argument) start from clear flags.
                    __hip_atomic_store(f, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
                const unsigned long long mk = __ballot(live);
                if (t == 0) *share = (unsigned)mk;
            }
            __syncthreads();
            const unsigned live_mask = *share;                // bit u: workgroup u of this XCD left a partial
            __syncthreads();
            // Partials are read with agent-scope loads (sc1): they bypass this CU's L1 and
            // are served by the L2 the producer wrote through.
            constexpr int TILES = C::TM * C::TN;
            {
                for (int jj = 0; jj < j; ++jj) {
                    if (!((live_mask >> jj) & 1u)) continue;
                    __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
                        p.partials + (size_t)(jj * 8 + xcd) * SLOT_BYTES, 0, SLOT_BYTES, 0x00020000);
                    // half of the accumulator at a time: up to 16 loads in flight per thread
                    constexpr int HALF = (TILES + 1) / 2;
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        v4i tmp[HALF * 4];
#pragma unroll
                        for (int a = 0; a < HALF; ++a)
#pragma unroll
                            for (int qd = 0; qd < 4; ++qd) {
                                if (h * HALF + a >= TILES) continue;
                                const auto v = __builtin_amdgcn_raw_buffer_load_b128(
                                    rsrc, my_off + (h * HALF + a) * 4096 + qd * 1024, 0, 16);
                                tmp[a * 4 + qd] = v4i{(int)v[0], (int)v[1], (int)v[2], (int)v[3]};
                            }
#pragma unroll
                        for (int a = 0; a < HALF; ++a) {
                            if (h * HALF + a >= TILES) continue;
                            const int ta = h * HALF + a, i = ta / C::TN, jn = ta % C::TN;
#pragma unroll
                            for (int qd = 0; qd < 4; ++qd) {
                                acc[i][jn][4 * qd] += tmp[a * 4 + qd].x;
                                acc[i][jn][4 * qd + 1] += tmp[a * 4 + qd].y;
                                acc[i][jn][4 * qd + 2] += tmp[a * 4 + qd].z;
                                acc[i][jn][4 * qd + 3] += tmp[a * 4 + qd].w;
                            }
                        }
                    }
                }
            }
        }
        epilogue<C>(p, acc, smem, m0, ng0);
    }
}

// Split-K kernel for the narrow tile shapes (a few hundred token rows).  Same persistent
// launch and the same division of every XCD's main-loop steps as above, but a tile is then
// shared by many workgroups (eight at M = 148, N = K = 4096), and one finisher pulling every
// partial through its own CU is bound by that CU's load path (560 KB: 9 us measured).  Here
// the contributors of a tile finish it together:
//   every contributor stores its accumulators and raises its arrival flag as soon as its
//   steps of the tile are done, and goes on with its other main-loop work;
//   at the end, once all flags of the tile are up, contributor number r adds the r-th slice
//   of ALL the partials (its own included), dequantises that slice and stores it;
//   it then raises its departure flag; contributor 0 waits for all departures and takes every
//   flag of the tile down again, so that a replay of a captured launch, which carries the
//   same epoch, starts clean.  Every flag has one writer: no read-modify-write atomics (a
//   contended compare-and-swap costs about 1.7 us here).
// A workgroup waits for workgroups with higher numbers too.  That cannot deadlock because
// the launch has at most one workgroup per compute unit and each fits one, so all of them
// are resident at the same time; the wait is bounded all the same (error word).
// A workgroup can be part of two shared tiles (where its share ends: slot 0, and where it
// begins: slot 1).
template <class C>
__global__ __launch_bounds__(C::THREADS, 1) void gemm_splitk_kernel(const GemmParams p)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    constexpr int TILES = C::TM * C::TN;
    constexpr int SLOT_BYTES = C::BM * C::BN * 4, UNITS = SLOT_BYTES / 16;
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int tiles = p.m_tiles * p.n_tiles;
    const int steps = p.chunks / kChunksPerStep;
    const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3, nb = p.blocks_per_xcd;
    const int q = tiles >> 3, r = tiles & 7;
    const int tile0 = xcd * q + (xcd < r ? xcd : r);
    const int ntile = q + (xcd < r ? 1 : 0);
    // (32-bit arithmetic: this kernel runs with at most 64 tiles, so ntile * steps * nb stays far below 2^31;
    // 64-bit divisions cost about a microsecond at the start of a launch that takes fifteen)
    const int total = ntile * steps;
    const int begin = total * j / nb, end = total * (j + 1) / nb;
    clear_error_word(p);
    if (begin >= end) return;
    const int t_first = begin / steps, t_last = (end - 1) / steps;
    const int my_off = wave * (TILES * 4096) + lane * 16;
    int *cslot = reinterpret_cast<int *>(smem);            // [0, 32): slot numbers of the tile's contributors
    int *cinfo = cslot + 32;                               // [0]: how many, [1]: this workgroup's number among them
    int *ckeep = cslot + 64;                               // [0, 64): slots whose flags this workgroup takes down at the end

    // Phase 1: all the main-loop work.  A shared tile's partial sums are stored and this
    // workgroup is counted in, without waiting for anybody: a workgroup that waited here would
    // make its neighbour wait for everything the workgroup still has to do.
    for (int tl = t_last; tl >= t_first; --tl) {
        const int tb = tl * steps;
        const int s0 = (begin > tb ? begin : tb) - tb;
        const int s1 = (end < tb + steps ? end : tb + steps) - tb;
        const int tile = tile0 + tl;
        const int nt = tile / p.m_tiles, mt = tile - nt * p.m_tiles;
        const int m0 = mt * C::BM, ng0 = nt * (C::BN / 32);
        v16i acc[C::TM][C::TN];
        zero_acc<C>(acc);
        mainloop<C, false>(p, smem, m0, ng0, s0, s1, acc);
        if (s0 == 0 && s1 == steps) {
            epilogue<C>(p, acc, smem, m0, ng0);            // the whole tile is this workgroup's
            continue;
        }
        const int which = tl == t_last ? 0 : 1;
        uint8_t *dst = p.partials + ((size_t)which * kMaxPersistentBlocks + blockIdx.x) * SLOT_BYTES + my_off;
#pragma unroll
        for (int i = 0; i < C::TM; ++i)
#pragma unroll
            for (int jn = 0; jn < C::TN; ++jn) {
#pragma unroll
                for (int qd = 0; qd < 4; ++qd) {
                    v4i v = {acc[i][jn][4 * qd], acc[i][jn][4 * qd + 1], acc[i][jn][4 * qd + 2],
                             acc[i][jn][4 * qd + 3]};
                    *reinterpret_cast<v4i *>(dst + qd * 1024) = v;
                }
                dst += 4096;
            }
        // The others sit behind the same L2 (same XCD); the stores are complete there once the
        // vector-memory counter drains, and only then is this workgroup counted in.
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (t == 0)
            __hip_atomic_store(&p.flags[kArriveWord + which * kMaxPersistentBlocks + blockIdx.x], p.epoch,
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }

    // Phase 2: finish the shared tiles (at most two: where the share ends and where it begins).
    if (t < 64) ckeep[t] = -1;                             // (LDS is free: the last main loop ended with a barrier)
    for (int pass = 0; pass < 2; ++pass) {
        const int tl = pass == 0 ? t_last : t_first;
        if (pass == 1 && t_first == t_last) break;
        const int tb = tl * steps;
        const int s0 = (begin > tb ? begin : tb) - tb;
        const int s1 = (end < tb + steps ? end : tb + steps) - tb;
        if (s0 == 0 && s1 == steps) continue;              // was a whole tile
        const int tile = tile0 + tl;
        const int nt = tile / p.m_tiles, mt = tile - nt * p.m_tiles;
        const int m0 = mt * C::BM, ng0 = nt * (C::BN / 32);
        // who shares this tile: the workgroups of this XCD from the holder of its first step to
        // the holder of its last step (those with an empty share excepted)
        int first = (tb * nb) / total;
        while (total * (first + 1) / nb <= tb) ++first;
        while (total * first / nb > tb) --first;
        __syncthreads();                                   // cslot / cinfo of the previous pass are no longer read
        if (t < 64) {
            const int jj = first + t;
            const int jb = jj < nb ? total * jj / nb : 0, je = jj < nb ? total * (jj + 1) / nb : 0;
            const bool live = jj < nb && jb < je && jb < tb + steps;          // has steps, and they start inside the tile
            const unsigned long long mk = __ballot(live);
            if (live) {
                const int rank = __popcll(mk & ((1ull << t) - 1ull));
                const int w2 = tl == (je - 1) / steps ? 0 : 1;          // the slot that workgroup used for this tile
                cslot[rank] = w2 * kMaxPersistentBlocks + jj * 8 + xcd;
                if (jj == j) cinfo[1] = rank;
            }
            if (t == 0) cinfo[0] = __popcll(mk);
        }
        __syncthreads();
        const int nc = cinfo[0], rank = cinfo[1];
        // one lane per contributor waits for that contributor's arrival
        if (t < nc) {
            const unsigned long long *f = &p.flags[kArriveWord + cslot[t]];
            long long spins = 0;
            while (__hip_atomic_load(f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != p.epoch) {
                __builtin_amdgcn_s_sleep(8);
                if (++spins > kSpinLimit) {
                    raise_error_word(p);          // give up: the result of this tile is wrong
                    break;
                }
            }
        }
        __syncthreads();

        // this workgroup's slice of the tile, 16 bytes (4 channels of one token) per thread at a time;
        // partials are read with agent-scope loads (sc1): they bypass this CU's L1
        const int ub = UNITS * rank / nc, ue = UNITS * (rank + 1) / nc;
        const bool y_vec = (p.ldy & 3) == 0 && (reinterpret_cast<uintptr_t>(p.Y) & 7u) == 0;
        constexpr int UPT = 4;                             // units per thread per trip
        for (int u0 = ub + t; u0 < ue; u0 += UPT * C::THREADS) {
            // where each unit goes, and its scales: issued before the partial sums so that the
            // two kinds of load overlap.  unit u = ((w * TILES + a) * 4 + qd) * 64 + l
            int row[UPT], col[UPT];
            bool live[UPT];
            float sxf[UPT];
            uint2 swr[UPT];
#pragma unroll
            for (int x = 0; x < UPT; ++x) {
                const int u = u0 + x * C::THREADS;
                const int l = u & 63, qd = (u >> 6) & 3, a = (u >> 8) % TILES, w = (u >> 8) / TILES;
                row[x] = m0 + ((a / C::TN) * C::WAVES_M + w / C::WAVES_N) * 32 + (l & 31);
                col[x] = (ng0 << 5) + (w % C::WAVES_N) * C::WN + (a % C::TN) * 32 + qd * 8 + (l >> 5) * 4;
                live[x] = u < ue && row[x] < p.M && col[x] < p.N;
                sxf[x] = 0.f;
                swr[x] = uint2{0u, 0u};
                if (live[x]) {
                    sxf[x] = __half2float(p.sx[row[x]]) * 0.00390625f;
                    swr[x] = *reinterpret_cast<const uint2 *>(p.sw + col[x]);        // zero padded past N
                }
            }
            // four contributors at a time: up to 16 loads in flight
            v4i sums[UPT];
#pragma unroll
            for (int x = 0; x < UPT; ++x) sums[x] = v4i{0, 0, 0, 0};
            for (int c0 = 0; c0 < nc; c0 += 4) {
                v4i tmp[4][UPT];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    if (c0 + k < nc) {
                        __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
                            p.partials + (size_t)__builtin_amdgcn_readfirstlane(cslot[c0 + k]) * SLOT_BYTES, 0,
                            SLOT_BYTES, 0x00020000);
#pragma unroll
                        for (int x = 0; x < UPT; ++x) {
                            if (live[x]) {
                                const auto v = __builtin_amdgcn_raw_buffer_load_b128(
                                    rsrc, (u0 + x * C::THREADS) * 16, 0, 16);
                                tmp[k][x] = v4i{(int)v[0], (int)v[1], (int)v[2], (int)v[3]};
                            }
                        }
                    }
                }
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    if (c0 + k < nc) {
#pragma unroll
                        for (int x = 0; x < UPT; ++x)
                            if (live[x]) sums[x] += tmp[k][x];
                    }
            }
#pragma unroll
            for (int x = 0; x < UPT; ++x) {
                if (!live[x]) continue;
                const v4i sum = sums[x];
                const __half2 *sw2 = reinterpret_cast<const __half2 *>(&swr[x]);
                const float2 s01 = __half22float2(sw2[0]), s23 = __half22float2(sw2[1]);
                uint2 pk;
                pk.x = dequant2(sum.x, sum.y, sxf[x], s01.x, s01.y);
                pk.y = dequant2(sum.z, sum.w, sxf[x], s23.x, s23.y);
                __half *dst = p.Y + (size_t)row[x] * p.ldy + col[x];
                if (y_vec && col[x] + 4 <= p.N) {
                    *reinterpret_cast<uint2 *>(dst) = pk;
                } else {
                    const __half *h = reinterpret_cast<const __half *>(&pk);
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (col[x] + e < p.N) dst[e] = h[e];
                }
                if (p.acc_out) {
                    int32_t *ad = p.acc_out + (size_t)row[x] * p.N + col[x];
                    const int v4[4] = {sum.x >> 8, sum.y >> 8, sum.z >> 8, sum.w >> 8};
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (col[x] + e < p.N) ad[e] = v4[e];
                }
            }
        }
        // every load of the others' partials has been consumed above: count out
        __syncthreads();
        if (t == 0)
            __hip_atomic_store(&p.flags[kDepartWord + cslot[rank]], p.epoch, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
        // contributor 0 takes the tile's flags down once everybody is out: phase 3
        if (rank == 0 && t < nc) ckeep[pass * 32 + t] = cslot[t];
    }

    // Phase 3: flags of the tiles this workgroup is contributor 0 of.  Waiting for the others'
    // departures here, after this workgroup's own, keeps the waits from forming a chain.
    __syncthreads();
    if (t < 64) {
        const int slot = ckeep[t];
        if (slot >= 0) {
            unsigned long long *d = &p.flags[kDepartWord + slot];
            long long spins = 0;
            while (__hip_atomic_load(d, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != p.epoch) {
                __builtin_amdgcn_s_sleep(8);
                if (++spins > kSpinLimit) {
                    raise_error_word(p);
                    break;
                }
            }
            __hip_atomic_store(d, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(&p.flags[kArriveWord + slot], 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

// Flags need no clearing between launches: a flag counts as set only when it
// holds the launch's own epoch, a 64-bit value never used before in this
// process (a per-process random upper half and a counter).  Whatever an earlier
// launch or another owner of the memory left there differs from it.  A launch
// replayed from a captured graph carries the epoch it was captured with; that
// is safe because every flag a launch raises is taken down by its one consumer
// before the launch ends.
static unsigned long long next_epoch()
{
    static std::atomic<unsigned long long> counter{0};
    static const unsigned long long salt = [] {
        std::random_device rd;
        unsigned long long s = ((unsigned long long)rd() << 32) ^ (unsigned long long)rd();
        return (s | 1ull) << 32;
    }();
    return salt + (++counter);
}

// The persistent kernels hand partial sums from workgroup b to a workgroup b' with b' % 8 == b % 8
// through ordinary stores, which is valid only when the two sit behind one L2: the dispatcher has to
// deal workgroup b of a launch to XCD b % 8 (or the device has a single L2).  The probe reads the
// XCC_ID register in every workgroup of a launch shaped like the persistent ones; a device where the
// rule does not hold gets the one-tile-per-workgroup kernels, which share nothing.
__device__ unsigned int g_xcc_of_block[kMaxPersistentBlocks];

__global__ __launch_bounds__(512) void xcc_probe_kernel()
{
    unsigned int x;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(x));
    if (threadIdx.x == 0) g_xcc_of_block[blockIdx.x] = x & 15u;
}

constexpr int kMaxDevices = kMaxDeviceSlots;
static std::atomic<int> g_dealing[kMaxDevices];      // 0 not probed, 1 the rule holds, 2 it does not

sqap_status probe_dispatch(int device, hipStream_t st, uint32_t *table_out)
{
    if (device < 0 || device >= kMaxDevices) return fail(SQAP_EUNSUPPORTED, "device ordinal %d above %d", device, kMaxDevices - 1);
    if (g_dealing[device].load() != 0 && !table_out) return SQAP_OK;
    // The probe synchronises the stream, which a capturing stream does not allow: leave the device unprobed
    // (the one-tile-per-workgroup kernels are used until a later call probes it).
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(st, &cap) == hipSuccess && cap != hipStreamCaptureStatusNone) {
        if (table_out) return fail(SQAP_EUNSUPPORTED, "dispatch probe: the stream is capturing");
        return SQAP_OK;
    }
    unsigned int host[kMaxPersistentBlocks];
    hipLaunchKernelGGL(xcc_probe_kernel, dim3(kMaxPersistentBlocks), dim3(512), 0, st);
    SQAP_HIP_CHECK(hipGetLastError());
    SQAP_HIP_CHECK(hipStreamSynchronize(st));
    SQAP_HIP_CHECK(hipMemcpyFromSymbol(host, HIP_SYMBOL(g_xcc_of_block), sizeof(host), 0, hipMemcpyDeviceToHost));
    bool ok = true;
    for (int b = 0; b < kMaxPersistentBlocks; ++b) ok = ok && host[b] == host[b % kXcds];
    g_dealing[device].store(ok ? 1 : 2);
    if (table_out)
        for (int b = 0; b < kMaxPersistentBlocks; ++b) table_out[b] = host[b];
    return SQAP_OK;
}

static std::atomic<int> g_mid_m_kernel{1};            // 1: gemm_rows_kernel where it applies, 0: the split-K tile kernels

void set_mid_m_kernel(int which) { g_mid_m_kernel.store(which ? 1 : 0); }

static std::atomic<int> g_persistent_switch{-1};      // -1: follow the environment, 0: off, 1: on

void set_persistent_kernels(int enabled) { g_persistent_switch.store(enabled ? 1 : 0); }

static bool persistent_allowed()
{
    // SQAP_DISABLE_PERSISTENT=1 in the environment selects the fallback kernels; read once per process
    static const bool disabled = [] {
        const char *off = getenv("SQAP_DISABLE_PERSISTENT");
        return off && off[0] == '1';
    }();
    const int sw = g_persistent_switch.load(std::memory_order_relaxed);
    if (sw == 0 || (sw < 0 && disabled)) return false;
    int dev = 0;
    return hipGetDevice(&dev) == hipSuccess && dev >= 0 && dev < kMaxDevices && g_dealing[dev].load() == 1;
}

static int persistent_blocks()
{
    int cus = device_cu_count();
    if (cus < kXcds) cus = kMaxPersistentBlocks;
    if (cus > kMaxPersistentBlocks) cus = kMaxPersistentBlocks;
    return (cus / kXcds) * kXcds;
}

// Tile shapes.  Large M: 256 x 256, eight wavefronts.  Below that the output is too
// small to fill the machine with whole tiles (M = 148, N = 4096 is 19 x 128 MFMA tiles
// for 1024 SIMDs), so narrow 128-column tiles of 96 or 160 rows are split along K by the
// same stream-K kernel.
using CfgBig = Cfg<256, 256, 2, 4>;
using CfgMid = Cfg<160, 128, 1, 4>;
using CfgLow = Cfg<96, 128, 1, 4>;

// Below kStreamKMinM rows: 160- or 96-row tiles, whichever pads M less (148 -> one tile of 160;
// 84 -> one of 96; 174, 199 or 276 -> two or three of 96 rather than two of 160).
static bool narrow_tile_is_mid(int M)
{
    const int pad_mid = (M + CfgMid::BM - 1) / CfgMid::BM * CfgMid::BM;
    const int pad_low = (M + CfgLow::BM - 1) / CfgLow::BM * CfgLow::BM;
    return pad_mid <= pad_low;
}

size_t linear_workspace_bytes(int M, int, int K)
{
    if (K % kBK != 0 || M <= kSkinnyMaxM) return 0;
    // one tile-sized int32 slot per workgroup; the narrow shapes need two (see gemm_splitk_kernel)
    if (M >= kStreamKMinM) return kFlagBytes + (size_t)kMaxPersistentBlocks * CfgBig::BM * CfgBig::BN * sizeof(int32_t);
    const size_t slot = narrow_tile_is_mid(M) ? (size_t)CfgMid::BM * CfgMid::BN : (size_t)CfgLow::BM * CfgLow::BN;
    return kFlagBytes + 2 * (size_t)kMaxPersistentBlocks * slot * sizeof(int32_t);
}

template <class C, class K>
static sqap_status set_lds(K kernel)
{
    SQAP_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES));
    return SQAP_OK;
}

template <class C, bool RAGGED_K>
static sqap_status launch_tiled_k(GemmParams &p, hipStream_t st)
{
    p.m_tiles = (p.M + C::BM - 1) / C::BM;
    p.n_tiles = (p.N + C::BN - 1) / C::BN;
    static std::atomic<bool> configured[kMaxDeviceSlots];
    const int dslot = device_slot();
    if (!configured[dslot].load(std::memory_order_acquire)) {
        sqap_status s = set_lds<C>(&gemm_tiled_kernel<C, RAGGED_K>);
        if (s != SQAP_OK) return s;
        configured[dslot].store(true, std::memory_order_release);
    }
    const int64_t blocks = (int64_t)p.m_tiles * p.n_tiles;
    if (blocks > 0x7fffffff) return fail(SQAP_EUNSUPPORTED, "sqap_w4a4_linear: too many tiles");
    hipLaunchKernelGGL((gemm_tiled_kernel<C, RAGGED_K>), dim3((unsigned)blocks), dim3(C::THREADS), C::LDS_BYTES, st,
                       p);
    SQAP_HIP_CHECK(hipGetLastError());
    return SQAP_OK;
}

template <class C>
static sqap_status launch_tiled(GemmParams &p, hipStream_t st)
{
    if (p.chunks % kChunksPerStep) return launch_tiled_k<C, true>(p, st);
    return launch_tiled_k<C, false>(p, st);
}

// ---------------------------------------------------------------------------------------------
// Shares of the stream-K launch.  Equal step counts do not give equal finishing times: a workgroup
// that finishes two tiles runs two epilogues, a tile of a ragged last tile row has short steps, and a
// finisher cannot start its reduction before the last contributor has published (a workgroup whose
// whole share is one published segment publishes at the very end of its work).  The host therefore
// plays the launch through with measured costs and looks for the smallest finishing time T for which
// a sweep over the workgroups of an XCD, each taking the largest share it completes by T, uses up all
// the steps.  A finisher only depends on lower-numbered workgroups, so one pass in index order knows
// every publishing time it needs.  Costs are in units of one full main-loop step.
struct SplitModel {
    double step_last;      // a step of a tile of the last tile row (1 when that row is full)
    double epi, epi_last;  // epilogue of a full tile / of a last-row tile
    double ramp;           // entering a main loop: first loads, pipeline fill, bookkeeping around it
    double publish;        // storing a partial and raising the flag
    double reduce_fixed, reduce_each;   // flag look-up; reading and adding one contributor's partial
};

// Measured on MI355X with time stamps inside the kernel (256 x 256 tiles; one full step is about 1.4 us):
// main-loop entry 1.5-1.7 us, partial store and flag 2.6-2.9 us, flag look-up 1.3 us, one partial read and
// added 2.5-3.9 us, epilogue 4.1-5.0 us; a last-row tile that uses 1, 2 or 3 of the 4 accumulator rows
// runs a step in 0.41 / 0.60 / 0.83 of a full one.
constexpr SplitModel kBigTileModel = {1.0, 2.9, 2.9, 1.1, 1.8, 0.9, 2.3};
// The narrow tiles (96 or 160 rows x 128 columns; a step is about 0.35 us): costs set by trial, 1-3 % faster than equal
// step counts at M = 84 and 148, no different at M = 276 (twice these values gain more at M = 148 and lose at M = 276).
constexpr SplitModel kNarrowTileModel = {1.0, 3.0, 3.0, 4.0, 2.0, 2.0, 2.3};
constexpr double kRaggedStep[4] = {0.41, 0.60, 0.83, 1.0};
constexpr double kRaggedEpilogue[4] = {1.1, 1.8, 2.4, 2.9};

// Finishing time of a workgroup with share [b, e) of an XCD whose tiles start at global tile number tile0;
// pub[jj] = publishing time of workgroup jj (lower numbers only are read); *my_pub receives this one's.
static double play_share(int b, int e, int steps, int tile0, int mtl, const SplitModel &m, const uint32_t *bounds,
                         const double *pub, int j, double *my_pub)
{
    *my_pub = 0.0;
    if (b >= e) return 0.0;
    double t = 0.0, chain = 0.0;
    const int t_first = b / steps, t_last = (e - 1) / steps;
    int tl = t_last;
    auto is_last_row = [&](int tl_) { return (tile0 + tl_) % mtl == mtl - 1; };
    {
        const int tb = tl * steps, s0 = std::max(b - tb, 0), s1 = std::min(e - tb, steps);
        if (s1 < steps) {
            const bool lr = is_last_row(tl);
            t += m.ramp + (s1 - s0) * (lr ? m.step_last : 1.0) + m.publish;
            *my_pub = t;
            // What this partial holds up: the tile's finisher still has to add the partials (this one,
            // those of the lower workgroups in the tile, and one more if what is left of the tile is
            // more than a share of average size) and to run the epilogue after it.
            int n = 1;
            for (int jj = 0; jj < j; ++jj)
                if (bounds[jj] < bounds[jj + 1] && (int)bounds[jj + 1] > tb) ++n;
            if (steps - s1 > (int)(bounds[j] / (j > 0 ? j : 1)) && j > 0) ++n;
            chain = t + m.reduce_fixed + n * m.reduce_each + (lr ? m.epi_last : m.epi);
            --tl;
        }
    }
    for (; tl >= t_first; --tl) {
        const int tb = tl * steps, s0 = std::max(b - tb, 0);
        const bool lr = is_last_row(tl);
        t += m.ramp + (steps - s0) * (lr ? m.step_last : 1.0);
        if (s0 > 0) {
            int n = 0;
            for (int jj = 0; jj < j; ++jj) {
                const int jb = (int)bounds[jj], je = (int)bounds[jj + 1];
                if (jb < je && je > tb && jb < tb + s0) {
                    t = std::max(t, pub[jj]);
                    ++n;
                }
            }
            t += m.reduce_fixed + n * m.reduce_each;
        }
        t += lr ? m.epi_last : m.epi;
    }
    return std::max(t, chain);
}

// Fills bounds[0 .. nb] for one XCD; returns false when no plan was found (the caller then splits evenly).
static bool plan_xcd(int tile0, int ntile, int steps, int mtl, int nb, const SplitModel &m, uint32_t *bounds,
                     double *t_out)
{
    const int total = ntile * steps;
    double work = 0.0;
    for (int tl = 0; tl < ntile; ++tl)
        work += ((tile0 + tl) % mtl == mtl - 1) ? steps * m.step_last + m.epi_last : steps + m.epi;
    double lo = work / nb, hi = 2.0 * work / nb + 4.0 * (m.epi + m.publish + m.reduce_fixed + m.reduce_each + m.ramp) + steps;
    std::vector<uint32_t> trial(nb + 1), best;
    std::vector<double> pub(nb);
    double best_t = 0.0;
    auto sweep = [&](double T) -> bool {
        trial[0] = 0;
        double worst = 0.0;
        for (int j = 0; j < nb; ++j) {
            const int b = (int)trial[j];
            int pick = -1;
            double pick_t = 0.0, pick_pub = 0.0;
            if (j == nb - 1) {
                trial[j + 1] = (uint32_t)total;
                double pj;
                const double t = play_share(b, total, steps, tile0, mtl, m, trial.data(), pub.data(), j, &pj);
                if (t > T) return false;
                worst = std::max(worst, t);
                pub[j] = pj;
                break;
            }
            // The largest share that is done by T.  The finishing time grows with the share except
            // where the share crosses into another tile, so: bisect, then look one tile further.
            auto fits = [&](int e, double *t, double *pj) {
                trial[j + 1] = (uint32_t)e;
                *t = play_share(b, e, steps, tile0, mtl, m, trial.data(), pub.data(), j, pj);
                return *t <= T;
            };
            const int e_max = std::min((long long)total, (long long)b + (long long)(T / std::min(1.0, m.step_last)) + 1);
            int good = b, bad = e_max + 1;                     // an empty share always fits
            double t, pj;
            while (bad - good > 1) {
                const int mid = good + (bad - good) / 2;
                if (fits(mid, &t, &pj)) good = mid;
                else bad = mid;
            }
            for (int e = std::min(e_max, good + steps + 1); e >= good; --e)
                if (fits(e, &t, &pj)) {
                    pick = e;
                    pick_t = t;
                    pick_pub = pj;
                    break;
                }
            if (pick < 0) return false;
            trial[j + 1] = (uint32_t)pick;
            pub[j] = pick_pub;
            worst = std::max(worst, pick_t);
        }
        best = trial;
        best_t = worst;
        return true;
    };
    if (!sweep(hi)) return false;
    for (int it = 0; it < 24 && hi - lo > 0.05; ++it) {
        const double mid = 0.5 * (lo + hi);
        if (sweep(mid)) hi = mid;
        else lo = mid;
    }
    for (int j = 0; j <= nb; ++j) bounds[j] = best[j];
    *t_out = best_t;
    return true;
}

static void even_shares(int ntile, int steps, int nb, uint32_t *bounds)
{
    const long long total = (long long)ntile * steps;
    for (int j = 0; j <= nb; ++j) bounds[j] = (uint32_t)(total * j / nb);
}

// Finishing time the model gives the slowest workgroup of an XCD under the shares `bounds`.
static double predict_xcd(const uint32_t *bounds, int nb, int steps, int tile0, int mtl, const SplitModel &m)
{
    double pub[kMaxPersistentBlocks / kXcds], worst = 0.0;
    for (int j = 0; j < nb; ++j)
        worst = std::max(worst, play_share((int)bounds[j], (int)bounds[j + 1], steps, tile0, mtl, m, bounds, pub, j, &pub[j]));
    return worst;
}

// Plans the shares of one launch (cached per shape: a plan takes a few milliseconds of host time).
// model == nullptr: equal step counts.
static void plan_shares(int tiles, int steps, int mtl, int nb, const SplitModel *model, StreamKShares *out)
{
    const int q = tiles / kXcds, r = tiles % kXcds;
    for (int x = 0; x < kXcds; ++x) {
        const int tile0 = x * q + std::min(x, r), ntile = q + (x < r ? 1 : 0);
        double t;
        for (int j = 0; j <= kMaxPersistentBlocks / kXcds; ++j) out->bounds[x][j] = (uint32_t)((long long)ntile * steps);
        // XCDs whose runs of tiles look alike (same length, same place in the tile column) share a plan
        int twin = -1;
        for (int y = 0; y < x && twin < 0; ++y) {
            const int tile0y = y * q + std::min(y, r), ntiley = q + (y < r ? 1 : 0);
            if (ntiley == ntile && tile0y % mtl == tile0 % mtl) twin = y;
        }
        if (twin >= 0) {
            for (int j = 0; j <= nb; ++j) out->bounds[x][j] = out->bounds[twin][j];
            continue;
        }
        uint32_t even[kMaxPersistentBlocks / kXcds + 1];
        even_shares(ntile, steps, nb, even);
        // equal step counts when there is no model, no plan, or a plan the model itself rates no better
        // (with sixteen or more tiles per workgroup the differences are below two percent: not worth a plan)
        if (!model || ntile >= 16 * nb || !plan_xcd(tile0, ntile, steps, mtl, nb, *model, out->bounds[x], &t) ||
            t >= predict_xcd(even, nb, steps, tile0, mtl, *model))
            for (int j = 0; j <= nb; ++j) out->bounds[x][j] = even[j];
    }
}

struct PlanKey {
    int tiles, steps, mtl, nb, groups, kind;
    bool operator<(const PlanKey &o) const
    {
        return std::tie(tiles, steps, mtl, nb, groups, kind) < std::tie(o.tiles, o.steps, o.mtl, o.nb, o.groups, o.kind);
    }
};

template <class C, bool SPLITK>
static sqap_status launch_streamk(GemmParams &p, void *workspace, hipStream_t st)
{
    p.m_tiles = (p.M + C::BM - 1) / C::BM;
    p.n_tiles = (p.N + C::BN - 1) / C::BN;
    const int blocks = persistent_blocks();
    p.blocks_per_xcd = blocks / kXcds;
    p.flags = reinterpret_cast<unsigned long long *>(workspace);
    p.epoch = next_epoch();
    p.partials = reinterpret_cast<uint8_t *>(workspace) + kFlagBytes;
    static std::atomic<bool> configured[kMaxDeviceSlots];
    const int dslot = device_slot();
    if (!configured[dslot].load(std::memory_order_acquire)) {
        sqap_status s;
        if constexpr (SPLITK) s = set_lds<C>(&gemm_splitk_kernel<C>);
        else s = set_lds<C>(&gemm_streamk_kernel<C>);
        if (s != SQAP_OK) return s;
        configured[dslot].store(true, std::memory_order_release);
    }
    if constexpr (SPLITK) {
        hipLaunchKernelGGL((gemm_splitk_kernel<C>), dim3(blocks), dim3(C::THREADS), C::LDS_BYTES, st, p);
    } else {
        const int steps = p.chunks / kChunksPerStep;
        const int64_t tiles = (int64_t)p.m_tiles * p.n_tiles;
        if ((tiles / kXcds + 1) * steps > 0x7fffffff) return launch_tiled<C>(p, st);    // shares are 32-bit step counts
        const int groups = (p.M - (p.m_tiles - 1) * C::BM + 31) / 32;
        const PlanKey key = {(int)tiles, steps, p.m_tiles, p.blocks_per_xcd, groups, C::BM * 1024 + C::BN};
        static std::mutex mu;
        static std::map<PlanKey, StreamKShares> plans;
        StreamKShares shares;
        {
            std::lock_guard<std::mutex> lock(mu);
            auto it = plans.find(key);
            if (it == plans.end()) {
                StreamKShares fresh;
                if constexpr (C::WAVES_M > 1) {
                    const int rows_used = (groups + C::WAVES_M - 1) / C::WAVES_M;     // accumulator rows of a last-row tile
                    SplitModel m = kBigTileModel;
                    m.step_last = kRaggedStep[rows_used - 1];
                    m.epi_last = kRaggedEpilogue[rows_used - 1];
                    plan_shares((int)tiles, steps, p.m_tiles, p.blocks_per_xcd, &m, &fresh);
                } else {
                    plan_shares((int)tiles, steps, p.m_tiles, p.blocks_per_xcd, &kNarrowTileModel, &fresh);
                }
                if (plans.size() > 4096) plans.clear();
                it = plans.emplace(key, fresh).first;
            }
            shares = it->second;
        }
        hipLaunchKernelGGL((gemm_streamk_kernel<C>), dim3(blocks), dim3(C::THREADS), C::LDS_BYTES, st, p, shares);
    }
    SQAP_HIP_CHECK(hipGetLastError());
    return SQAP_OK;
}

// Host-only view of the planner (tests and diagnostics): the shares a stream-K launch of
// shape (M, N, K) on blocks_per_xcd workgroups per XCD would get, and per XCD the finishing time the
// model predicts for them and for equal step counts, in main-loop steps.
sqap_status plan_linear_shares(int M, int N, int K, int blocks_per_xcd, uint32_t *bounds_out, double *planned_out,
                               double *even_out, int *tile_rows_out, int *tile_cols_out)
{
    if (M <= kSkinnyMaxM || K % kBK != 0 || K > kMaxK)
        return fail(SQAP_EUNSUPPORTED, "sqap_plan_linear_shares: M > %d and K a multiple of %d only", kSkinnyMaxM, kBK);
    if (blocks_per_xcd < 1 || blocks_per_xcd > kMaxPersistentBlocks / kXcds)
        return fail(SQAP_EINVAL, "sqap_plan_linear_shares: 1 to %d workgroups per XCD", kMaxPersistentBlocks / kXcds);
    // tile shape and cost model as launch_w4a4_linear / launch_streamk choose them
    const bool big = M >= kStreamKMinM;
    const int BM = big ? CfgBig::BM : narrow_tile_is_mid(M) ? CfgMid::BM : CfgLow::BM;
    const int BN = big ? CfgBig::BN : CfgMid::BN;
    const int m_tiles = (M + BM - 1) / BM, n_tiles = (N + BN - 1) / BN, steps = K / kBK;
    const int64_t tiles = (int64_t)m_tiles * n_tiles;
    if ((tiles / kXcds + 1) * steps > 0x7fffffff) return fail(SQAP_EUNSUPPORTED, "sqap_plan_linear_shares: too many steps");
    SplitModel m = kNarrowTileModel;
    if (big) {
        const int groups = (M - (m_tiles - 1) * BM + 31) / 32;
        const int rows_used = (groups + CfgBig::WAVES_M - 1) / CfgBig::WAVES_M;
        m = kBigTileModel;
        m.step_last = kRaggedStep[rows_used - 1];
        m.epi_last = kRaggedEpilogue[rows_used - 1];
    }
    StreamKShares planned, even;
    plan_shares((int)tiles, steps, m_tiles, blocks_per_xcd, &m, &planned);
    plan_shares((int)tiles, steps, m_tiles, blocks_per_xcd, nullptr, &even);
    const int q = (int)(tiles / kXcds), r = (int)(tiles % kXcds), per = kMaxPersistentBlocks / kXcds + 1;
    for (int x = 0; x < kXcds; ++x) {
        const int tile0 = x * q + std::min(x, r);
        planned_out[x] = predict_xcd(planned.bounds[x], blocks_per_xcd, steps, tile0, m_tiles, m);
        even_out[x] = predict_xcd(even.bounds[x], blocks_per_xcd, steps, tile0, m_tiles, m);
        for (int j = 0; j < per; ++j) bounds_out[x * per + j] = planned.bounds[x][j];
    }
    *tile_rows_out = BM;
    *tile_cols_out = BN;
    return SQAP_OK;
}

sqap_status launch_w4a4_linear(const uint8_t *Xq, const __half *sx, int M, const Weight &w,
                               __half *Y, int64_t ldy, int32_t *acc_out, void *workspace, hipStream_t st)
{
    if (w.K > kMaxK) return fail(SQAP_EUNSUPPORTED, "sqap_w4a4_linear: K = %d above %d", w.K, kMaxK);
    GemmParams p = {};
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
    p.y_vec_ok = (reinterpret_cast<uintptr_t>(Y) & 15u) == 0 && (ldy & 7) == 0;
    // A few hundred token rows: whole outputs per workgroup, nothing exchanged between workgroups
    if (M < kStreamKMinM && g_mid_m_kernel.load(std::memory_order_relaxed) == 1 && rows_kernel_applies(M, w.N, w.K))
        return launch_rows_linear(Xq, sx, M, w, Y, ldy, acc_out, st);
    if (w.K % kBK == 0 && persistent_allowed()) {
        if (M >= kStreamKMinM) return launch_streamk<CfgBig, false>(p, workspace, st);
        // Narrow tiles.  With few tiles, each is shared by many workgroups (256 / tiles of them) and
        // the contributors finish it together; with many tiles a single finisher has only two or
        // three partials to add, which measured faster than the joint finish (23.6 vs 28.6 us at
        // M = 148, N = 11008, K = 4096; the other way round, 21.6 vs 15.2 us, at N = 4096).
        const bool mid = narrow_tile_is_mid(M);
        const int64_t tiles = (int64_t)((M + (mid ? CfgMid::BM : CfgLow::BM) - 1) / (mid ? CfgMid::BM : CfgLow::BM)) *
                              ((w.N + CfgMid::BN - 1) / CfgMid::BN);
        const bool joint = tiles * 4 <= kMaxPersistentBlocks;
        if (mid) return joint ? launch_streamk<CfgMid, true>(p, workspace, st) : launch_streamk<CfgMid, false>(p, workspace, st);
        return joint ? launch_streamk<CfgLow, true>(p, workspace, st) : launch_streamk<CfgLow, false>(p, workspace, st);
    }
    // K not a multiple of 128 (or a device whose dispatch order the persistent kernels cannot rely on):
    // one tile per workgroup, reduction axis guarded
    if (M <= CfgLow::BM) return launch_tiled<CfgLow>(p, st);
    if (M <= CfgMid::BM) return launch_tiled<CfgMid>(p, st);
    return launch_tiled<CfgBig>(p, st);
}

}  // namespace sqap
