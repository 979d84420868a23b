// Small-M (decode) W4A4 linear: M <= 8 token rows against a weight matrix that
// is streamed from HBM exactly once.  The work is memory bound, so the kernel
// is organised around keeping many 1 KiB weight loads in flight per wavefront;
// the arithmetic (same int8 MFMA and dequantisation as the prefill GEMM) rides
// along.
//
// One launch serves a whole table of independent problems (a "group"): q/k/v
// of a layer, gate/up, or every linear of a benchmark step.  A work item is one
// row group (32 output channels) of one problem and belongs to ONE wavefront,
// which walks the item's whole reduction axis with a ring of loads in flight:
// no cross-wavefront reduction, no barrier per item.  Each block owns a
// contiguous run of items holding an equal share of the launch's weight bytes,
// so it keeps streaming across problem boundaries instead of paying a launch
// per linear; the block re-stages the (tiny) activations in LDS only when its
// run enters another problem.
#include "common.h"

namespace sqap {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kSkinnyWaves = 8;         // wavefronts per workgroup, two workgroups per CU ...
constexpr int kSkinnyWavesBig = 16;     // ... or one workgroup of 16 for the launches that stream for long (see launch_skinny)
constexpr int kSkinnyDepth = 8;          // 1 KiB weight loads in flight per wavefront
constexpr int kSkinnyZeroBytes = 16;

__device__ __forceinline__ void widen4(const v4i p, v4i &lo, v4i &hi)
{
    const v4i mask = {(int)0xF0F0F0F0, (int)0xF0F0F0F0, (int)0xF0F0F0F0, (int)0xF0F0F0F0};
    lo = (p << 4) & mask;
    hi = p & mask;
}

// same two-step rounding as the prefill epilogue (see gemm.hip)
__device__ __forceinline__ __half dequant2(int acc, float sx, float sw)
{
    float y = ((float)acc * sx) * sw;
    asm volatile("" : "+v"(y));
    return __float2half_rn(y);
}

// The problem table is read with vector loads, so the compiler treats what it
// reads as per-lane values.  Everything below IS wavefront-uniform; saying so
// keeps the bookkeeping in scalar registers and the hot loop free of lane masks.
__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ long long uni(long long v)
{
    const unsigned lo = __builtin_amdgcn_readfirstlane((int)(v & 0xffffffffll));
    const unsigned hi = __builtin_amdgcn_readfirstlane((int)(v >> 32));
    return (long long)(((unsigned long long)hi << 32) | lo);
}
template <class T>
__device__ __forceinline__ T *uni(T *p)
{
    return reinterpret_cast<T *>(uni((long long)reinterpret_cast<uintptr_t>(p)));
}

// A block's run of items: the first item whose cumulative cost (in 16-byte weight pieces per
// row) reaches the block's share boundary, for both of its boundaries at once.  The problem
// holding a boundary is found by counting, across the lanes, the problems that start at or
// before it (cost_begin is nondecreasing): one round of loads for both boundaries instead of
// a scan with one dependent load per problem, which used to cost the last blocks of a 225-problem
// launch tens of microseconds before their first weight load.
__device__ __forceinline__ void block_run(const SkinnyEntry *table, int count, int total_items, long long lo,
                                          long long hi, bool to_the_end, int lane, int *beg, int *end, int *problem)
{
    int n_lo = 0, n_hi = 0;
    for (int base = 0; base < count; base += 64) {
        const int e = base + lane;
        const long long c = e < count ? table[e].cost_begin : 0x7fffffffffffffffll;
        n_lo += __popcll(__ballot(c <= lo));
        n_hi += __popcll(__ballot(c <= hi));
    }
    auto item_of = [&](int p, long long target) {
        const long long into = target - uni(table[p].cost_begin);
        const int ch = uni(table[p].chunks);
        const long long it = uni(table[p].rg_begin) + (into + ch - 1) / ch;
        return it < total_items ? (int)it : total_items;
    };
    *problem = n_lo - 1;                          // cost_begin of problem 0 is 0: at least one counted
    *beg = item_of(n_lo - 1, lo);
    *end = to_the_end ? total_items : item_of(n_hi - 1, hi);
}

// A launch with at most kSkinnyInline problems carries them in the kernel arguments.  They are read
// with constant indices only: taking the address of a kernel argument would make the compiler copy the
// whole argument block (368 bytes) into every lane's scratch memory at kernel start.
#define SQAP_INLINE_FIELD(a, p, field) \
    ((p) == 0 ? (a).inline_entries[0].field : (p) == 1 ? (a).inline_entries[1].field : \
     (p) == 2 ? (a).inline_entries[2].field : (a).inline_entries[3].field)

// block_run for inline problems (count <= 4): the same boundaries, from scalar arithmetic.
__device__ __forceinline__ void inline_run(const SkinnyArgs &a, long long lo, long long hi, bool to_the_end, int *beg,
                                           int *end, int *problem)
{
    int n_lo = 0, n_hi = 0;
#pragma unroll
    for (int p = 0; p < kSkinnyInline; ++p) {
        if (p < a.count) {
            const long long c = SQAP_INLINE_FIELD(a, p, cost_begin);
            n_lo += c <= lo ? 1 : 0;
            n_hi += c <= hi ? 1 : 0;
        }
    }
    auto item_of = [&](int p, long long target) {
        const long long into = target - SQAP_INLINE_FIELD(a, p, cost_begin);
        const int ch = SQAP_INLINE_FIELD(a, p, chunks);
        const long long it = SQAP_INLINE_FIELD(a, p, rg_begin) + (into + ch - 1) / ch;
        return it < a.total_items ? (int)it : a.total_items;
    };
    *problem = n_lo - 1;
    *beg = item_of(n_lo - 1, lo);
    *end = to_the_end ? a.total_items : item_of(n_hi - 1, hi);
}

// LDS: [0, 16): zeros; then the packed activations of the current problem,
// 256 bytes per chunk pair cp: [k-half h][row r < 8][16 bytes]; then (S > 1)
// 1 KiB per wavefront for the partial sums.
//
// S = number of wavefronts that share one item, each taking a slice of the
// reduction axis.  S = 1 is the streaming configuration for large groups.  A
// launch with few items (one linear, one layer) would otherwise run on a few
// hundred wavefronts, each latency bound on its own ring; S > 1 spreads the same
// bytes over up to 8 times as many wavefronts and adds their partial
// accumulators through LDS.

// Every weight byte is read once: a nontemporal load keeps the stream from displacing the rest of
// the caches' contents (a plain streaming read measures 6.1 TB/s on this part, a nontemporal one 6.8).
__device__ __forceinline__ v4i stream_load(const v4i *p) { return __builtin_nontemporal_load(p); }

template <int S, int W>
__global__ __launch_bounds__(W * 64, 4) void skinny_kernel(const SkinnyArgs a)
{
    constexpr bool LATE = W == kSkinnyWavesBig;  // outputs wait in LDS (the 16-wavefront form)
    // The 16-wavefront form also hands out a segment's items on demand.  With a fixed stride a block's run
    // of about 170 items leaves some wavefronts one item more than others (a twelfth of their work), and a
    // wavefront that gets less of the memory system than its neighbours cannot pass work on: the
    // wavefronts of a block ended up to 60 us apart at 450 us.  The first W items of a segment are dealt
    // by wavefront index; after that a wavefront takes the next one from a counter in LDS, one item ahead
    // of its need so that the load ring runs on across the item boundary as before.
    constexpr bool DYN = LATE && S == 1;
    __shared__ int seg_next;
    constexpr int R = W / S;                     // items a block works on at a time
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);     // uniform: keeps item bookkeeping scalar
    uint8_t *xs = smem + kSkinnyZeroBytes;
    if (t < 4) reinterpret_cast<int *>(smem)[t] = 0;

    // Outputs wait in LDS until the wavefront has no weights left to stream.  Vector-memory operations of
    // a wavefront retire in order, so a ring slot loaded after an output store cannot be consumed before the
    // store is acknowledged, and under this load that takes as long as the ring is deep; with 8 token rows
    // (8 lines far apart per store) the stream stood still for about 8 % of the time.  Slot k of this
    // wavefront: 8 rows x 64 bytes of halves at out_data + k * 512, its destination in out_meta[k].
    struct OutMeta {
        __half *Y;
        long long ldy;
        int M, N, rg, pad;
    };
    uint8_t *out_data = smem + (LATE ? a.out_off + (size_t)wave * a.out_cap * 512 : 0);
    OutMeta *out_meta = reinterpret_cast<OutMeta *>(smem + (LATE ? a.out_off + (size_t)W * a.out_cap * 512 : 0)) + (LATE ? wave * a.out_cap : 0);
    int out_n = 0;
    auto flush_outputs = [&]() {
        for (int k = 0; k < out_n; ++k) {
            const OutMeta m = out_meta[k];
            __half *Y = uni(m.Y);
            const long long ldy = uni(m.ldy);
            const int Mk = uni(m.M), Nk = uni(m.N), rgk = uni(m.rg);
            const int row = lane >> 2, col = rgk * 32 + (lane & 3) * 8;
            if (lane < 32 && row < Mk && col < Nk)
                *reinterpret_cast<v4i *>(Y + (size_t)row * ldy + col) =
                    *reinterpret_cast<const v4i *>(out_data + k * 512 + row * 64 + (lane & 3) * 16);
        }
        __builtin_amdgcn_wave_barrier();
        out_n = 0;
    };

    const SkinnyEntry *table = a.table;
    const bool inl = table == nullptr;             // the problems are in the kernel arguments
    int prob, beg, end;                            // prob: the problem the first item belongs to (or the one before it)
    if (inl)
        inline_run(a, a.total_cost * blockIdx.x / gridDim.x, a.total_cost * (blockIdx.x + 1) / gridDim.x,
                   blockIdx.x + 1 == gridDim.x, &beg, &end, &prob);
    else
        block_run(table, a.count, a.total_items, a.total_cost * blockIdx.x / gridDim.x,
                  a.total_cost * (blockIdx.x + 1) / gridDim.x, blockIdx.x + 1 == gridDim.x, lane, &beg, &end, &prob);
    auto rg_begin_of = [&](int p) { return inl ? SQAP_INLINE_FIELD(a, p, rg_begin) : uni(table[p].rg_begin); };
    const int r = lane & 31, h = lane >> 5;
    for (int cur = beg; cur < end;) {
        while (prob + 1 < a.count && cur >= rg_begin_of(prob + 1)) ++prob;
        SkinnyEntry e;
        if (inl) {
            e.Xq = SQAP_INLINE_FIELD(a, prob, Xq);
            e.sx = SQAP_INLINE_FIELD(a, prob, sx);
            e.Wd = SQAP_INLINE_FIELD(a, prob, Wd);
            e.sw = SQAP_INLINE_FIELD(a, prob, sw);
            e.Y = SQAP_INLINE_FIELD(a, prob, Y);
            e.acc_out = SQAP_INLINE_FIELD(a, prob, acc_out);
            e.ldy = SQAP_INLINE_FIELD(a, prob, ldy);
            e.M = SQAP_INLINE_FIELD(a, prob, M);
            e.N = SQAP_INLINE_FIELD(a, prob, N);
            e.chunks = SQAP_INLINE_FIELD(a, prob, chunks);
            e.rg_begin = SQAP_INLINE_FIELD(a, prob, rg_begin);
        } else {
            e = table[prob];
            e.Xq = uni(e.Xq);
            e.sx = uni(e.sx);
            e.Wd = uni(e.Wd);
            e.sw = uni(e.sw);
            e.Y = uni(e.Y);
            e.acc_out = uni(e.acc_out);
            e.ldy = uni((long long)e.ldy);
            e.M = uni(e.M);
            e.N = uni(e.N);
            e.chunks = uni(e.chunks);
            e.rg_begin = uni(e.rg_begin);
        }
        const int next_begin = prob + 1 < a.count ? rg_begin_of(prob + 1) : end;
        const int seg_end = next_begin < end ? next_begin : end;
        const int cps = e.chunks >> 1;

        // this wavefront's first item and slice [c0, c0 + cn) of its chunk pairs: start the
        // weight stream before staging the activations
        const int sub = wave / S, ks = wave % S;
        int item = cur + sub;
        const int c0 = (int)((long long)cps * ks / S);
        const int cn = (int)((long long)cps * (ks + 1) / S) - c0;
        const int rounds = (cn + kSkinnyDepth - 1) / kSkinnyDepth;
        const size_t item_stride = (size_t)R * e.chunks * 32;     // in v4i: R row groups on
        auto item_weights = [&](int it) {
            return reinterpret_cast<const v4i *>(e.Wd + ((size_t)(it - e.rg_begin) * e.chunks + 2 * c0) * 512) + lane;
        };
        const v4i *wsrc = item_weights(item);
        v4i wbuf[kSkinnyDepth];
        if (item < seg_end) {
#pragma unroll
            for (int d = 0; d < kSkinnyDepth; ++d) wbuf[d] = stream_load(wsrc + (size_t)(d < cn ? d : 0) * 64);
        }

        __syncthreads();                           // every wavefront is done with the previous problem's xs
        const int Kh = e.chunks * 16;
        for (int u = t; u < cps * 16; u += W * 64) {
            const int cp = u >> 4, hh = (u >> 3) & 1, rr = u & 7;
            v4i v = {0, 0, 0, 0};
            if (rr < e.M) v = reinterpret_cast<const v4i *>(e.Xq + (size_t)rr * Kh)[2 * cp + hh];
            *reinterpret_cast<v4i *>(xs + cp * 256 + hh * 128 + rr * 16) = v;
        }
        if (DYN && t == 0) seg_next = cur + R;     // everybody has left the previous segment's loop (barrier above)
        __syncthreads();
        // lanes whose token row does not exist read the zero block, with stride 0
        const bool has_row = r < e.M;
        const int xoff = has_row ? (kSkinnyZeroBytes + c0 * 256 + h * 128 + r * 16) : 0;
        const int xstride = has_row ? 256 : 0;
        const float sxf = has_row ? __half2float(e.sx[r]) : 0.f;
        const bool y_vec = (e.N & 3) == 0 && (e.ldy & 3) == 0 && (reinterpret_cast<uintptr_t>(e.Y) & 7u) == 0;
        // 16-byte stores possible: the output goes through the LDS slots (when the launch has any)
        const bool y_late = LATE && a.out_cap > 0 && (e.N & 7) == 0 && (e.ldy & 7) == 0 &&
                            (reinterpret_cast<uintptr_t>(e.Y) & 15u) == 0;

        for (int base = cur; DYN ? item < seg_end : base < seg_end; base += R) {
            const int rg = item - e.rg_begin;
            const bool active = item < seg_end;
            int next_item = item + R;
            if (DYN) {
                int taken = 0;
                if (lane == 0) taken = atomicAdd(&seg_next, 1);
                next_item = __builtin_amdgcn_readfirstlane(taken);
            }
            const bool has_next = next_item < seg_end;
            const v4i *wnext = has_next ? (DYN ? item_weights(next_item) : wsrc + item_stride) : wsrc;
            v16i acc;
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[i] = 0;
            // this lane's 16 channel scales (4 runs of 4 halves), asked for before the weights are
            // walked so that the epilogue does not wait for them; the scale array is padded to whole
            // row groups and 8-byte aligned
            uint2 swraw[4] = {};
            if (active && ks == 0) {
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    swraw[q] = *reinterpret_cast<const uint2 *>(e.sw + rg * 32 + q * 8 + h * 4);
            }
            if (active) {
            // The loop body is branch free: every step consumes ring slot d and refills it
            // with exactly one load.  The reduction axis is padded to whole rounds; a
            // padding step multiplies by the zero block and its refill re-reads piece 0.
            for (int rd = 0; rd < rounds; ++rd) {
#pragma unroll
                for (int d = 0; d < kSkinnyDepth; ++d) {
                    const int cp = rd * kSkinnyDepth + d;
                    const bool valid = cp < cn;
                    v4i wlo, whi, xlo, xhi;
                    widen4(wbuf[d], wlo, whi);
                    const int p2 = cp + kSkinnyDepth;
                    const v4i *src = p2 < cn ? wsrc + (size_t)p2 * 64
                                             : (rd + 1 == rounds ? wnext + (size_t)(d < cn ? d : 0) * 64 : wsrc);
                    wbuf[d] = stream_load(src);
                    widen4(*reinterpret_cast<const v4i *>(smem + (valid ? xoff + cp * xstride : 0)), xlo, xhi);
                    acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(wlo, xlo, acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(whi, xhi, acc, 0, 0, 0);
                    // keep the steps apart: otherwise the compiler gathers all eight slots at
                    // the top of a round and drains the ring before refilling it
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            }
            wsrc = wnext;
            item = next_item;
            // Accumulator layout: lane l holds token l%32 and, in register i, channel
            // 8*(i/4) + 4*(l/32) + (i%4) of the row group: four consecutive channels per quad.
            if (S > 1) {
                // add the S slices: token lanes park their 16 registers in LDS (64 bytes per
                // lane slot r + 8h), the slice-0 wavefront of each item collects them
                int *red = reinterpret_cast<int *>(smem + kSkinnyZeroBytes + a.xs_bytes);
                if (has_row && ks != 0) {
                    int *dst = red + wave * 256 + (r + 8 * h) * 16;
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        *reinterpret_cast<v4i *>(dst + 4 * q) =
                            v4i{acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]};
                }
                __syncthreads();
                if (has_row && ks == 0) {
#pragma unroll
                    for (int o = 1; o < S; ++o) {
                        const int *src = red + (wave + o) * 256 + (r + 8 * h) * 16;
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const v4i v = *reinterpret_cast<const v4i *>(src + 4 * q);
                            acc[4 * q] += v.x;
                            acc[4 * q + 1] += v.y;
                            acc[4 * q + 2] += v.z;
                            acc[4 * q + 3] += v.w;
                        }
                    }
                }
                __syncthreads();
            }
            if (y_late && active && ks == 0) {
                if (out_n == a.out_cap) flush_outputs();
                if (has_row) {
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        union { __half hv[4]; uint2 u; } pk, swq;
                        swq.u = swraw[q];
#pragma unroll
                        for (int x = 0; x < 4; ++x)
                            pk.hv[x] = dequant2(acc[4 * q + x] >> 8, sxf, __half2float(swq.hv[x]));
                        *reinterpret_cast<uint2 *>(out_data + out_n * 512 + r * 64 + (q * 8 + h * 4) * 2) = pk.u;
                    }
                }
                if (lane == 0) out_meta[out_n] = OutMeta{e.Y, e.ldy, e.M, e.N, rg, 0};
                __builtin_amdgcn_wave_barrier();
                ++out_n;
            }
            if (has_row && active && ks == 0 && (!y_late || e.acc_out)) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int n = rg * 32 + q * 8 + h * 4;
                    if (n < e.N) {
                        union { __half hv[4]; uint2 u; } pk, swq;
                        swq.u = swraw[q];
                        int v[4];
#pragma unroll
                        for (int x = 0; x < 4; ++x) {
                            v[x] = acc[4 * q + x] >> 8;
                            pk.hv[x] = dequant2(v[x], sxf, __half2float(swq.hv[x]));
                        }
                        __half *dst = e.Y + (size_t)r * e.ldy + n;
                        if (y_late) {
                            // the halves are in the LDS slot; only the integer accumulators are stored here
                        } else if (y_vec) {
                            *reinterpret_cast<uint2 *>(dst) = pk.u;
                        } else {
#pragma unroll
                            for (int x = 0; x < 4; ++x)
                                if (n + x < e.N) dst[x] = pk.hv[x];
                        }
                        if (e.acc_out) {
#pragma unroll
                            for (int x = 0; x < 4; ++x)
                                if (n + x < e.N) e.acc_out[(size_t)r * e.N + n + x] = v[x];
                        }
                    }
                }
            }
        }
        cur = seg_end;
    }
    if (LATE) flush_outputs();
}

// LDS of a launch: zero block, activations of one problem, 1 KiB per wavefront for the sliced reduction,
// then (16-wavefront form only) the output slots, 512 + 32 bytes each, out_cap per wavefront, in what is
// left of the CU's 160 KiB.
constexpr int kSkinnyOutSlot = 512 + 32;
constexpr int kSkinnyOutCapMax = 16;
static size_t skinny_base_lds_bytes(int max_chunks, int waves)
{
    return (kSkinnyZeroBytes + (size_t)(max_chunks / 2) * 256 + (size_t)waves * 1024 + 15) & ~(size_t)15;
}
static int skinny_out_cap(size_t base)
{
    const size_t limit = 160 * 1024 - 64;       // the kernel's few statically allocated bytes come on top
    const size_t room = base < limit ? limit - base : 0;
    const int cap = (int)(room / ((size_t)kSkinnyWavesBig * kSkinnyOutSlot));
    return cap > kSkinnyOutCapMax ? kSkinnyOutCapMax : cap;
}
size_t skinny_lds_bytes(int max_chunks) { return skinny_base_lds_bytes(max_chunks, kSkinnyWaves); }

template <int S, int W>
static sqap_status launch_skinny_s(SkinnyArgs &a, size_t lds, int grid_cap, hipStream_t st)
{
    static std::atomic<size_t> configured[kMaxDeviceSlots];
    const int dslot = device_slot();
    if (lds > configured[dslot].load(std::memory_order_acquire)) {
        SQAP_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void *>(&skinny_kernel<S, W>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        configured[dslot].store(lds, std::memory_order_release);
    }
    constexpr int R = W / S;
    const int want = (a.total_items + R - 1) / R;
    const int grid = want < grid_cap ? want : grid_cap;
    hipLaunchKernelGGL((skinny_kernel<S, W>), dim3(grid), dim3(W * 64), lds, st, a);
    SQAP_HIP_CHECK(hipGetLastError());
    return SQAP_OK;
}

// Which form of the kernel a launch of total_items row groups (longest row: max_chunks pieces) takes on a
// device with `cus` compute units: S wavefronts per row group, W wavefronts per workgroup, out_cap LDS
// output slots per wavefront (0: outputs are stored at once).  Host arithmetic only.
void skinny_plan(int total_items, int max_chunks, int cus, int *S, int *W, int *out_cap)
{
    // Launches in which every wavefront streams several items (a whole model's linears in one group): one
    // workgroup of 16 wavefronts per CU, whose outputs wait in LDS until the wavefront has streamed its
    // last weight (see the kernel).  532 -> 527 us at M = 1 and 577 -> 541 us at M = 8 for the 225 linears of
    // the 7B shape.  Shorter launches are bound by start-up and by how many CUs pull weights, not by the
    // stores, and ran 15-30 % slower in this form: they keep two workgroups of 8 per CU and store at once.
    const int cap = skinny_out_cap(skinny_base_lds_bytes(max_chunks, kSkinnyWavesBig));
    if ((long long)total_items >= 4ll * cus * kSkinnyWavesBig && cap >= 4) {
        *S = 1;
        *W = kSkinnyWavesBig;
        *out_cap = cap;
        return;
    }
    // aim at about 4096 wavefronts: share an item between S of them when items are few
    const long long waves = 2ll * cus * kSkinnyWaves;
    *W = kSkinnyWaves;
    *out_cap = 0;
    *S = total_items * 8ll <= waves ? 8 : total_items * 4ll <= waves ? 4 : total_items * 2ll <= waves ? 2 : 1;
}

sqap_status launch_skinny(const SkinnyArgs &args, int max_chunks, hipStream_t st)
{
    const size_t lds = skinny_lds_bytes(max_chunks);
    if (lds > 160 * 1024) return fail(SQAP_EUNSUPPORTED, "small-M linear: K too large for the LDS staging");
    const int cus = device_cu_count();
    SkinnyArgs a = args;
    a.xs_bytes = (max_chunks / 2) * 256;
    a.out_off = 0;
    a.out_cap = 0;
    int S, W, cap;
    skinny_plan(a.total_items, max_chunks, cus, &S, &W, &cap);
    if (W == kSkinnyWavesBig) {
        const size_t big_base = skinny_base_lds_bytes(max_chunks, kSkinnyWavesBig);
        a.out_off = (int)big_base;
        a.out_cap = cap;
        return launch_skinny_s<1, kSkinnyWavesBig>(a, big_base + (size_t)cap * kSkinnyWavesBig * kSkinnyOutSlot, cus, st);
    }
    const int grid_cap = 2 * cus;
    if (S == 8) return launch_skinny_s<8, kSkinnyWaves>(a, lds, grid_cap, st);
    if (S == 4) return launch_skinny_s<4, kSkinnyWaves>(a, lds, grid_cap, st);
    if (S == 2) return launch_skinny_s<2, kSkinnyWaves>(a, lds, grid_cap, st);
    return launch_skinny_s<1, kSkinnyWaves>(a, lds, grid_cap, st);
}

}  // namespace sqap
