// One decode step (one new token of one sequence through every layer and the vocabulary head) as ONE
// persistent launch.
//
// A decode step streams every weight once and each linear depends on the one before it.  As a chain of
// launches (nine per layer) a step costs the sum of their start-up and drain times: 2.6 ms per token for the
// 7B shape against 0.52 ms for the weights alone.  Here one workgroup per compute unit stays resident for
// the whole step and walks the linears in order:
//
//   phase  = [glue in front of the linear, redone by every workgroup] -> [its share of the linear] -> barrier
//   layer  = norm -> q|k|v | attention | quantize -> o | add, norm -> gate|up (+ SwiGLU) | quantize -> down
//
//   * The input of a linear is one row of at most 11008 values: every workgroup rebuilds it for itself (residual
//     add, RMSNorm with the exact sum of squares, int4 quantization: the arithmetic of the fused quantizer
//     kernels, statement by statement) and keeps the codes in LDS.  Nothing but the small rows between the
//     linears crosses workgroups, through agent-scope stores and loads.
//   * A linear's output channels are dealt to the workgroups in runs of 16-channel groups; inside a
//     workgroup the eight wavefronts split the run's reduction axis evenly and add through LDS.  With one
//     token there is nothing for a matrix core to reuse: each lane multiplies 32 weight codes of its
//     channel with the 32 activation codes by four v_dot8_i32_i4 (signed int4 x int4 -> int32, exact, no
//     widening).  A 1 KiB wavefront load is 16 channels x 4 pieces in the packed weight layout.
//   * Weights do not depend on activations, so the weight stream never waits for them: every wavefront
//     walks ITS pieces of all the linears of the step as one sequence, fifteen 1 KiB loads ahead of what
//     it multiplies, whatever phase those pieces belong to.  The loads land in a ring in LDS
//     (global_load_lds_dwordx4: no registers held, slots addressed at run time), 120 KiB per compute unit:
//     while the workgroup waits at a barrier or rebuilds an input row, the next linear's weights, and
//     often those of the one after, are arriving.  A full ring would stop the stream for the rest of the
//     wait (slots only free up when their pieces are multiplied), so on arriving at a barrier a wavefront
//     moves the eight oldest landed pieces into registers and asks for eight more.
//   * gate and up channels are dealt in pairs, so the workgroup that owns a pair applies SwiGLU to it and only
//     h = silu(g) * u crosses to the down projection.
//   * The barrier: every workgroup owns one 64-bit flag; arriving is a store of the launch's generation plus
//     the barrier's number, waiting is 256 lanes polling the 256 flags.  No read-modify-write atomics.  The
//     generation lives in device memory and moves on with every launch, so a launch captured in a graph can
//     be replayed.  All 256 workgroups must be resident at once: one per compute unit, checked at creation.
#include <new>
#include <vector>

#include "common.h"
#include "decode_attn.h"
#include "quant_math.h"

namespace sqap {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int kStepThreads = 512, kStepWaves = 8;
constexpr int kStepRing = 15;              // 1 KiB weight loads in flight (or landed, not yet used) per wavefront
constexpr int kStepPark = 8;               // landed pieces a wavefront moves from the ring into registers at a barrier
constexpr int kStepMaxGroups = 16;         // 16-channel groups a workgroup owns in one phase
constexpr int kStepGpt = 3;                // groups of 8 row elements per thread: K <= 12288
constexpr int kStepMaxK = kStepThreads * 8 * kStepGpt;
constexpr long long kStepSpinLimit = 400000;      // polls of a flag before a wait gives up (about a second)

enum StepKind { kStepQkv = 0, kStepO = 1, kStepGateUp = 2, kStepDown = 3, kStepHead = 4 };

struct StepPhase {
    int kind;
    int N, K, chunks;       // of the packed weight
    int units;              // work units: 16-channel groups; for gate|up: pairs of a gate and an up group
    int layer;
    const uint8_t *Wd;
    const __half *sw;
    const __half *gamma;    // norm gain (kinds q|k|v, gate|up, head)
    __half *kv;             // q|k|v: the layer's key/value cache
    long long ldkv;
};

struct StepArgs {
    const StepPhase *phases;
    int n_phases, blocks;
    int hidden, ffn, H, d;
    float eps;
    double base;
    const __half *x_in;     // [hidden] the token's embedding
    const int32_t *pos;     // [1]
    int past;
    __half *r1, *r2;        // residual stream after the attention block / after the feed-forward of the layer before
    __half *qkv, *attn, *o, *h, *dn;
    __half *logits;
    __half *attn_trace;     // nullable: [layers, hidden]
    unsigned long long *flags, *gen, *err;
    RopeFreq freq;
};

struct StepLds {
    __attribute__((aligned(16))) uint8_t xs[kStepMaxK / 2];                       // the linear's input row as int4 codes
    __attribute__((aligned(16))) int partial[kStepMaxGroups][kStepWaves][16];      // per wavefront sums of a group's 16 channels
    unsigned long long wsum[2 * kStepWaves];
    float wmax[kStepWaves];
    float sx;
    int dead;               // a wait gave up: later waits return at once (the step's result is wrong and says so)
    double2 sincos_tab[kDecMaxD / 2];      // sine, cosine of the token's rotation angles (the same for every layer)
    DecodeAttnLds attn;
    __attribute__((aligned(16))) uint8_t ring[kStepWaves][kStepRing][1024];         // weights asked for, per wavefront
};
static_assert(sizeof(StepLds) <= 160 * 1024, "one workgroup per compute unit: all of its LDS");

// ---- small rows that cross workgroups: agent-scope accesses, 8 elements (two 64-bit words) at a time ----
__device__ __forceinline__ void load8(const __half *p, int g, float (&f)[8])
{
    const unsigned long long *w = reinterpret_cast<const unsigned long long *>(p) + 2 * (size_t)g;
    const unsigned long long a = __hip_atomic_load(w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const unsigned long long b = __hip_atomic_load(w + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    uint4 raw = make_uint4((unsigned)a, (unsigned)(a >> 32), (unsigned)b, (unsigned)(b >> 32));
    unpack_halves(raw, f);
}

__device__ __forceinline__ void store8(__half *p, int g, const float (&f)[8])
{
    uint4 raw;
    __half2 *h2 = reinterpret_cast<__half2 *>(&raw);
#pragma unroll
    for (int q = 0; q < 4; ++q) h2[q] = __floats2half2_rn(f[2 * q], f[2 * q + 1]);
    unsigned long long *w = reinterpret_cast<unsigned long long *>(p) + 2 * (size_t)g;
    __hip_atomic_store(w, (unsigned long long)raw.x | ((unsigned long long)raw.y << 32), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(w + 1, (unsigned long long)raw.z | ((unsigned long long)raw.w << 32), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}

// The empty asm makes x exist as a binary32 value: otherwise the compiler folds the operation that produced it
// and the conversion into one mixed-precision instruction that rounds only once.
__device__ __forceinline__ float to_half_value(float x)
{
    asm volatile("" : "+v"(x));
    return __half2float(__float2half_rn(x));
}

// Residual update and RMSNorm of the row in v (thread t owns groups t, t + 512, ... of 8 elements), exactly as
// the fused quantizer kernel does it:  x' = half(x + delta);  S = sum x'^2 as a 128-bit integer (a half is an
// integer below 2^11 times 2^e, e >= -24, so x^2 * 2^48 is an integer: the sum does not depend on the order);
// r = (float)(1 / sqrt(S / K + eps)) in binary64;  v = half((x' * r) * gamma).  Contains a barrier.
__device__ __forceinline__ void step_norm(float (&v)[kStepGpt][8], int K, const __half *delta, __half *xsum_out,
                                          const __half *gamma, float eps, StepLds &lds)
{
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6, groups = K >> 3;
    unsigned long long hi = 0, lo = 0;
#pragma unroll
    for (int gi = 0; gi < kStepGpt; ++gi) {
        const int g = t + gi * kStepThreads;
        if (g < groups) {
            if (delta) {
                float dl[8];
                load8(delta, g, dl);
#pragma unroll
                for (int e = 0; e < 8; ++e) v[gi][e] = to_half_value(v[gi][e] + dl[e]);
            }
            if (xsum_out) store8(xsum_out, g, v[gi]);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const unsigned bits = __half_as_ushort(__float2half_rn(v[gi][e]));      // exact: v is a half value
                const unsigned ex = (bits >> 10) & 31u, man = bits & 1023u;
                const unsigned long long m = ex ? man + 1024u : man;
                const int sh = ex ? 2 * (int)ex - 2 : 0;                                // 2e + 48, at most 58
                const unsigned long long m2 = m * m;                                    // below 2^22
                const unsigned long long add_lo = m2 << sh;
                const unsigned long long add_hi = sh > 42 ? m2 >> (64 - sh) : 0ull;
                lo += add_lo;
                hi += add_hi + (lo < add_lo ? 1ull : 0ull);
            }
        }
    }
    for (int o = 32; o > 0; o >>= 1) {
        const unsigned long long ohi = __shfl_xor(hi, o), olo = __shfl_xor(lo, o);
        lo += olo;
        hi += ohi + (lo < olo ? 1ull : 0ull);
    }
    if (lane == 0) {
        lds.wsum[2 * wave] = hi;
        lds.wsum[2 * wave + 1] = lo;
    }
    __syncthreads();
    hi = lds.wsum[0];
    lo = lds.wsum[1];
#pragma unroll
    for (int w = 1; w < kStepWaves; ++w) {
        const unsigned long long olo = lds.wsum[2 * w + 1];
        lo += olo;
        hi += lds.wsum[2 * w] + (lo < olo ? 1ull : 0ull);
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
    const float r = (float)(1.0 / sqrt(Sd / (double)K + (double)eps));
#pragma unroll
    for (int gi = 0; gi < kStepGpt; ++gi) {
        const int g = t + gi * kStepThreads;
        if (g < groups) {
            float gm[8];
            unpack_halves(global_load16(reinterpret_cast<const uint4 *>(gamma) + g), gm);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float xr = v[gi][e] * r;
                v[gi][e] = to_half_value(xr * gm[e]);
            }
        }
    }
}

// Per-token int4 quantization of the row in v into lds.xs (canonical packing) and lds.sx, as the quantizer
// kernel does it: scale = half(max|v| / 7) (2^-24 when that is zero), code = clamp(rint(v / scale), -8, 7).
// Contains barriers; on return every thread may read the codes.
__device__ __forceinline__ void step_quantize(const float (&v)[kStepGpt][8], int K, StepLds &lds)
{
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6, groups = K >> 3;
    float amax = 0.f;
#pragma unroll
    for (int gi = 0; gi < kStepGpt; ++gi)
        if (t + gi * kStepThreads < groups) {
#pragma unroll
            for (int e = 0; e < 8; ++e) amax = fmaxf(amax, fabsf(v[gi][e]));
        }
    for (int o = 32; o > 0; o >>= 1) amax = fmaxf(amax, __shfl_xor(amax, o));
    __syncthreads();                                   // earlier readers of wmax and xs are done
    if (lane == 0) lds.wmax[wave] = amax;
    __syncthreads();
    amax = lds.wmax[0];
#pragma unroll
    for (int w = 1; w < kStepWaves; ++w) amax = fmaxf(amax, lds.wmax[w]);
    const __half sh = row_scale(amax);
    const float sf = __half2float(sh);
    const float rcp = 1.0f / sf;
    if (t == 0) lds.sx = sf;
#pragma unroll
    for (int gi = 0; gi < kStepGpt; ++gi) {
        const int g = t + gi * kStepThreads;
        if (g < groups) {
            uint32_t packed = 0;
#pragma unroll
            for (int e = 0; e < 8; ++e) packed |= code4(quotient(v[gi][e], sf, rcp)) << (4 * e);
            reinterpret_cast<uint32_t *>(lds.xs)[g] = packed;
        }
    }
    __syncthreads();
}

// ---- a workgroup's share of a linear ----
struct StepShare {
    int u0, n_groups;       // first unit, 16-channel groups owned (units x 1, or x 2 for gate|up)
    int i0, i1;             // this wavefront's items: (group, piece-of-four-chunks) pairs numbered group-major
    int Q;                  // items per group = chunks / 4
};

__device__ __forceinline__ StepShare step_share(const StepPhase &P, int block, int blocks, int wave)
{
    StepShare s;
    s.u0 = (int)((long long)P.units * block / blocks);
    const int u1 = (int)((long long)P.units * (block + 1) / blocks);
    s.n_groups = (u1 - s.u0) * (P.kind == kStepGateUp ? 2 : 1);
    s.Q = P.chunks >> 2;
    const int total = s.n_groups * s.Q;
    s.i0 = total * wave / kStepWaves;
    s.i1 = total * (wave + 1) / kStepWaves;
    return s;
}

// global 16-channel group of the share's local group j (gate|up: local 2p is the gate group of pair u0 + p,
// local 2p + 1 the up group, which sits F / 16 groups further on)
__device__ __forceinline__ int step_group(const StepPhase &P, const StepShare &s, int j)
{
    if (P.kind != kStepGateUp) return s.u0 + j;
    return s.u0 + (j >> 1) + (j & 1) * P.units;
}

// this lane's 16 bytes of item i: channel lane % 16 of the group, chunk 4 q + lane / 16
__device__ __forceinline__ const v4i *step_item(const StepPhase &P, const StepShare &s, int i, int lane)
{
    const int j = i / s.Q, q = i - j * s.Q;
    const int g = step_group(P, s, j);
    return reinterpret_cast<const v4i *>(P.Wd + ((size_t)(g >> 1) * P.chunks + 4 * q + (lane >> 4)) * 512 +
                                         ((g & 1) * 16 + (lane & 15)) * 16);
}

// Where a wavefront is in the sequence of weight pieces it asks for: the pieces of its share of phase 0, then
// of phase 1, ... (a phase in which it has none is skipped).  Everything but lane_ptr is wavefront-uniform.
struct StepStream {
    int ph;                    // phase of the next piece (n_phases: the sequence has ended)
    int i, i1;                 // the piece's number within the wavefront's share of that phase; the share's end
    int q, Q;                  // piece within its 16-channel group; pieces per group
    int issued;                // pieces asked for so far
    int slot;                  // ring slot of the next piece = issued % kStepRing
    const uint8_t *lane_ptr;   // this lane's 16 bytes of the next piece
};

__device__ __forceinline__ void stream_enter(StepStream &c, const StepArgs &a, int block, int wave, int lane)
{
    while (c.ph < a.n_phases) {
        const StepPhase &P = a.phases[c.ph];
        const StepShare sh = step_share(P, block, a.blocks, wave);
        if (sh.i0 < sh.i1) {
            c.i = sh.i0;
            c.i1 = sh.i1;
            c.Q = sh.Q;
            c.q = sh.i0 % sh.Q;
            c.lane_ptr = reinterpret_cast<const uint8_t *>(step_item(P, sh, sh.i0, lane));
            return;
        }
        ++c.ph;
    }
}

// Asks for the next piece of the sequence (into the ring slot that the piece kStepRing before it has left).
__device__ __forceinline__ void stream_issue(StepStream &c, const StepArgs &a, StepLds &lds, int block, int wave, int lane)
{
    if (c.ph >= a.n_phases) return;
    __builtin_amdgcn_global_load_lds(reinterpret_cast<const v4i *>(c.lane_ptr),
                                     (__attribute__((address_space(3))) void *)(&lds.ring[wave][c.slot][0]), 16, 0, 0);
    ++c.issued;
    c.slot = c.slot + 1 == kStepRing ? 0 : c.slot + 1;
    ++c.i;
    ++c.q;
    c.lane_ptr += 4 * 512;                             // the next four chunks of the same 16 channels
    if (c.i == c.i1) {
        ++c.ph;
        stream_enter(c, a, block, wave, lane);
    } else if (c.q == c.Q) {                           // the next group of the share
        c.q = 0;
        const StepPhase &P = a.phases[c.ph];
        const StepShare sh = step_share(P, block, a.blocks, wave);
        c.lane_ptr = reinterpret_cast<const uint8_t *>(step_item(P, sh, c.i, lane));
    }
}

__device__ __forceinline__ void step_arrive(const StepArgs &a, unsigned long long value)
{
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this thread's stores of the phase are complete
    __syncthreads();
    if (threadIdx.x == 0) __hip_atomic_store(&a.flags[blockIdx.x], value, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ void step_wait(const StepArgs &a, unsigned long long value, StepLds &lds)
{
    const int t = threadIdx.x;
    if (t < a.blocks && lds.dead == 0) {
        long long spins = 0;
        while (__hip_atomic_load(&a.flags[t], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < value) {
            __builtin_amdgcn_s_sleep(2);
            if (++spins > kStepSpinLimit) {            // give up: the step's result is wrong, and says so
                __hip_atomic_store(a.err, value, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                lds.dead = 1;
                break;
            }
        }
    }
    __syncthreads();
}

// Diagnostic builds (-DSQAP_STEP_STAMPS) record the 100 MHz wall clock of four workgroups at eight points of every
// phase into the attention trace buffer; product builds compile the macro away.
#ifdef SQAP_STEP_STAMPS
#define STEP_STAMP(k)                                                                                       \
    do {                                                                                                    \
        if (t == 0 && (block & 63) == 0 && a.attn_trace)                                                    \
            reinterpret_cast<unsigned long long *>(a.attn_trace + 262144)[((block >> 6) * 400 + ph) * 8 + (k)] = wall_clock64(); \
    } while (0)
#else
#define STEP_STAMP(k) do { } while (0)
#endif

__global__ __launch_bounds__(kStepThreads, 1) void decoder_step_kernel(const StepArgs a)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    StepLds &lds = *reinterpret_cast<StepLds *>(smem);
    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int block = blockIdx.x;
    const unsigned long long gen0 = *a.gen;            // left by the launch before this one
    unsigned long long bar = 0;
    const int pos0 = a.pos[0];
    if (block == 0 && t == 0) __hip_atomic_store(a.err, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (t == 0) lds.dead = 0;
    if (block < a.H && t < (a.d >> 1)) {               // the rotation's sines and cosines: once per step instead of per layer
        double sn, cs;
        sincos(rope_angle(a.freq, pos0, t, a.d, a.base), &sn, &cs);
        lds.sincos_tab[t] = double2{sn, cs};
    }
    __syncthreads();

    StepStream stream = {};
    stream_enter(stream, a, block, wave, lane);
    for (int k = 0; k < kStepRing; ++k) stream_issue(stream, a, lds, block, wave, lane);
    int consumed = 0, cslot = 0;                       // pieces that have left the ring so far; ring slot of the oldest one in it
    v4i park[kStepPark];                               // the oldest pieces not yet multiplied, moved out of the ring
    int park_c = 0, park_n = 0;                        // park[park_c .. park_n) are waiting
    // moves landed pieces from the ring into the park registers (when those are empty) and asks for as many new ones
    auto park_pieces = [&]() {
        if (park_c != park_n) return;
        const int avail = stream.issued - consumed;
        const int n = avail < kStepPark ? avail : kStepPark;
        park_c = 0;
        park_n = n;
#pragma unroll
        for (int dd = 0; dd < kStepPark; ++dd)
            if (dd < n) {
                int sl = cslot + dd;
                if (sl >= kStepRing) sl -= kStepRing;
                park[dd] = *reinterpret_cast<const v4i *>(&lds.ring[wave][sl][lane * 16]);
            }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");      // the slots are read before new pieces may land in them
        consumed += n;
        cslot += n;
        if (cslot >= kStepRing) cslot -= kStepRing;
        for (int k = 0; k < n; ++k) stream_issue(stream, a, lds, block, wave, lane);
    };

    for (int ph = 0; ph < a.n_phases; ++ph) {
        const StepPhase P = a.phases[ph];
        const StepShare share = step_share(P, block, a.blocks, wave);
        STEP_STAMP(0);
        // ---- the linear's input row: built by every workgroup for itself ----
        {
            float v[kStepGpt][8];
            const int K = P.K, groups = K >> 3;
            const __half *src = nullptr, *delta = nullptr;
            __half *xsum = nullptr;
            if (P.kind == kStepQkv) {
                src = P.layer == 0 ? a.x_in : a.r2;
                delta = P.layer == 0 ? nullptr : a.dn;
                xsum = a.r1;
            } else if (P.kind == kStepGateUp) {
                src = a.r1;
                delta = a.o;
                xsum = a.r2;
            } else if (P.kind == kStepHead) {
                src = a.r2;
                delta = a.dn;
            } else if (P.kind == kStepO) {
                src = a.attn;
            } else {
                src = a.h;
            }
#pragma unroll
            for (int gi = 0; gi < kStepGpt; ++gi) {
                const int g = t + gi * kStepThreads;
                if (g < groups) {
                    load8(src, g, v[gi]);
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e) v[gi][e] = 0.f;
                }
            }
            if (P.gamma) step_norm(v, K, delta, block == 0 ? xsum : nullptr, P.gamma, a.eps, lds);
            step_quantize(v, K, lds);
        }
        STEP_STAMP(1);
        // ---- this workgroup's channels: the wavefronts split the reduction axis ----
        for (int i = t; i < kStepMaxGroups * kStepWaves * 16; i += kStepThreads) (&lds.partial[0][0][0])[i] = 0;
        __syncthreads();
        {
            int acc = 0;
            int j = share.i0 < share.i1 ? share.i0 / share.Q : 0, q = share.i0 < share.i1 ? share.i0 - j * share.Q : 0;
            auto flush = [&]() {
                int sum = acc;
                sum += __shfl_xor(sum, 16);
                sum += __shfl_xor(sum, 32);
                if (lane < 16) lds.partial[j][wave][lane] = sum;
                acc = 0;
            };
            auto multiply = [&](const v4i w) {
                const v4i x = *reinterpret_cast<const v4i *>(lds.xs + (4 * q + (lane >> 4)) * 16);
                acc = __builtin_amdgcn_sdot8(w.x, x.x, acc, false);
                acc = __builtin_amdgcn_sdot8(w.y, x.y, acc, false);
                acc = __builtin_amdgcn_sdot8(w.z, x.z, acc, false);
                acc = __builtin_amdgcn_sdot8(w.w, x.w, acc, false);
                if (++q == share.Q) {
                    flush();
                    q = 0;
                    ++j;
                }
            };
            int i = share.i0;
            // first the pieces parked in registers (they are the oldest), then the ring
#pragma unroll
            for (int dd = 0; dd < kStepPark; ++dd)
                if (dd >= park_c && dd < park_n && i < share.i1) {
                    multiply(park[dd]);
                    ++park_c;
                    ++i;
                }
            for (; i < share.i1; ++i) {
                // The piece to multiply was asked for kStepRing pieces ago (fewer at the very end of the step): it
                // has landed once at most the younger pieces are still on their way (loads return in order).
                if (stream.issued - consumed == kStepRing) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kStepRing - 1) : "memory");
                else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                const v4i w = *reinterpret_cast<const v4i *>(&lds.ring[wave][cslot][lane * 16]);
                multiply(w);
                // the slot is free (its contents are in registers: the products above needed them)
                stream_issue(stream, a, lds, block, wave, lane);
                ++consumed;
                cslot = cslot + 1 == kStepRing ? 0 : cslot + 1;
            }
            if (share.i0 < share.i1 && q != 0) flush();
        }
        __syncthreads();
        STEP_STAMP(2);
        // ---- outputs: two adjacent channels per thread (one 32-bit agent-scope store) ----
        {
            const float sxf = lds.sx;
            const bool gate_up = P.kind == kStepGateUp;
            const int n_out = gate_up ? share.n_groups >> 1 : share.n_groups;        // groups of 16 outputs
            if (t < n_out * 8) {
                const int jo = t >> 3, row = (t & 7) * 2;
                auto channel_pair = [&](int j, float (&y)[2]) {       // dequantised outputs of local group j, rows row, row + 1
                    int s0 = 0, s1 = 0;
#pragma unroll
                    for (int w = 0; w < kStepWaves; ++w) {
                        s0 += lds.partial[j][w][row];
                        s1 += lds.partial[j][w][row + 1];
                    }
                    const int n = step_group(P, share, j) * 16 + row;
                    const unsigned swb = *(const SQAP_GLOBAL unsigned *)(P.sw + n);       // two scales; padded to whole row groups
                    const __half2 sw2 = *reinterpret_cast<const __half2 *>(&swb);
                    float y0 = ((float)s0 * sxf) * __low2float(sw2), y1 = ((float)s1 * sxf) * __high2float(sw2);
                    asm volatile("" : "+v"(y0), "+v"(y1));            // two binary32 products, then one rounding to half
                    y[0] = __half2float(__float2half_rn(y0));
                    y[1] = __half2float(__float2half_rn(y1));
                };
                float y[2];
                int n;
                __half *out;
                if (!gate_up) {
                    channel_pair(jo, y);
                    n = (share.u0 + jo) * 16 + row;
                    out = P.kind == kStepQkv ? a.qkv : P.kind == kStepO ? a.o : P.kind == kStepDown ? a.dn : a.logits;
                } else {
                    // h = half(silu(g) * u), silu(g) = (float)(g / (1 + exp(-g))) in binary64
                    float g2[2], u2[2];
                    channel_pair(2 * jo, g2);
                    channel_pair(2 * jo + 1, u2);
#pragma unroll
                    for (int e = 0; e < 2; ++e) {
                        const double gd = (double)g2[e];
                        const float sl = (float)(gd / (1.0 + exp(-gd)));
                        y[e] = to_half_value(sl * u2[e]);
                    }
                    n = (share.u0 + jo) * 16 + row;
                    out = a.h;
                }
                const int n_limit = gate_up ? P.N >> 1 : P.N;
                if (n < n_limit) {
                    const __half2 pk = __floats2half2_rn(y[0], y[1]);
                    __hip_atomic_store(reinterpret_cast<unsigned *>(out + n), *reinterpret_cast<const unsigned *>(&pk),
                                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
        }
        // ---- barrier, with the next linear's first weights asked for before the wait ----
        STEP_STAMP(3);
        ++bar;
        step_arrive(a, gen0 + bar);
        park_pieces();                                 // (everything in the ring has landed: the arrival waited for it)
        STEP_STAMP(4);
        if (P.kind == kStepQkv) {
            // attention of the new token over the layer's cache: one workgroup per head
            step_wait(a, gen0 + bar, lds);
            STEP_STAMP(5);
            if (block < a.H)
                decode_attention_head<true>(lds.attn, block, a.qkv, pos0, a.H, a.d, a.base, P.kv, P.ldkv, a.past, a.attn,
                                            a.attn_trace ? a.attn_trace + (size_t)P.layer * a.hidden : nullptr, a.freq, lds.sincos_tab);
            STEP_STAMP(6);
            ++bar;
            step_arrive(a, gen0 + bar);
        }
        step_wait(a, gen0 + bar, lds);
        STEP_STAMP(7);
    }
    // every workgroup has read the generation (it took part in a barrier since): move it on for the next launch
    if (block == 0 && t == 0) *a.gen = gen0 + bar;
}

// ---------------------------------------------------------------------------------------------
struct Decoder {
    uint32_t magic;
    int device, n_layers, hidden, ffn, H, d, vocab, n_phases, blocks;
    float eps;
    double base;
    StepPhase *phases;          // device
    __half *rows;               // device: r1, r2, qkv, attn, o, h, dn
    unsigned long long *sync;   // device: flags[256], generation, error word
    size_t off_r2, off_qkv, off_attn, off_o, off_h, off_dn;
};
constexpr uint32_t kDecoderMagic = 0x53514443u;  // "SQDC"
constexpr int kStepBlocks = 256;

static const Weight *as_weight(const sqap_weight *w)
{
    const Weight *ww = reinterpret_cast<const Weight *>(w);
    return ww && ww->magic == kWeightMagic ? ww : nullptr;
}

sqap_status decoder_create(const sqap_decoder_layer *layers, int n_layers, int n_heads, int head_dim,
                           const sqap_f16 *gamma_final, const sqap_weight *head, float eps, double rope_base,
                           Decoder **out)
{
    const Weight *hw = as_weight(head);
    if (!hw) return fail(SQAP_EINVAL, "sqap_decoder_create: head is not a weight handle");
    if (n_layers < 1 || n_heads < 1 || head_dim < 1)
        return fail(SQAP_EINVAL, "sqap_decoder_create: %d layers, %d heads of %d", n_layers, n_heads, head_dim);
    const int hidden = n_heads * head_dim;
    if (hw->K != hidden) return fail(SQAP_EINVAL, "sqap_decoder_create: head K = %d, hidden = %d", hw->K, hidden);
    if ((head_dim & 7) || head_dim > kDecMaxD) return fail(SQAP_EUNSUPPORTED, "sqap_decoder_create: head size %d (multiple of 8, <= %d)", head_dim, kDecMaxD);
    if (n_heads > kStepBlocks) return fail(SQAP_EUNSUPPORTED, "sqap_decoder_create: %d heads (at most %d)", n_heads, kStepBlocks);
    int ffn = 0;
    std::vector<StepPhase> ph;
    auto add = [&](int kind, int layer, const Weight *w, const sqap_f16 *gamma, sqap_f16 *kv, long long ldkv) {
        StepPhase p = {};
        p.kind = kind;
        p.layer = layer;
        p.N = w->N;
        p.K = w->K;
        p.chunks = w->chunks;
        p.units = kind == kStepGateUp ? w->N / 32 : (w->N + 15) / 16;
        p.Wd = w->data;
        p.sw = w->scales;
        p.gamma = reinterpret_cast<const __half *>(gamma);
        p.kv = reinterpret_cast<__half *>(kv);
        p.ldkv = ldkv;
        ph.push_back(p);
    };
    auto shape_ok = [&](const Weight *w, int N, int K, const char *what, int layer) -> sqap_status {
        if (!w) return fail(SQAP_EINVAL, "sqap_decoder_create: layer %d: %s is not a weight handle", layer, what);
        if (w->N != N || w->K != K)
            return fail(SQAP_EINVAL, "sqap_decoder_create: layer %d: %s is %d x %d, expected %d x %d", layer, what, w->N,
                        w->K, N, K);
        return SQAP_OK;
    };
    for (int l = 0; l < n_layers; ++l) {
        const sqap_decoder_layer &L = layers[l];
        const Weight *gu = as_weight(L.gate_up);
        if (!gu) return fail(SQAP_EINVAL, "sqap_decoder_create: layer %d: gate_up is not a weight handle", l);
        if (l == 0) ffn = gu->N / 2;
        sqap_status s;
        if ((s = shape_ok(as_weight(L.qkv), 3 * hidden, hidden, "qkv", l)) != SQAP_OK) return s;
        if ((s = shape_ok(as_weight(L.o), hidden, hidden, "o", l)) != SQAP_OK) return s;
        if ((s = shape_ok(gu, 2 * ffn, hidden, "gate_up", l)) != SQAP_OK) return s;
        if ((s = shape_ok(as_weight(L.down), hidden, ffn, "down", l)) != SQAP_OK) return s;
        if (!L.gamma_attn || !L.gamma_mlp || !L.kv) return fail(SQAP_EINVAL, "sqap_decoder_create: layer %d: null pointer", l);
        if (L.ldkv < 2 * hidden || (L.ldkv & 7) || (reinterpret_cast<uintptr_t>(L.kv) & 15u))
            return fail(SQAP_EINVAL, "sqap_decoder_create: layer %d: cache pitch below 2 * hidden or cache not 16-byte aligned", l);
        if ((reinterpret_cast<uintptr_t>(L.gamma_attn) | reinterpret_cast<uintptr_t>(L.gamma_mlp)) & 15u)
            return fail(SQAP_EUNSUPPORTED, "sqap_decoder_create: layer %d: norm gains must be 16-byte aligned", l);
        add(kStepQkv, l, as_weight(L.qkv), L.gamma_attn, L.kv, L.ldkv);
        add(kStepO, l, as_weight(L.o), nullptr, nullptr, 0);
        add(kStepGateUp, l, gu, L.gamma_mlp, nullptr, 0);
        add(kStepDown, l, as_weight(L.down), nullptr, nullptr, 0);
    }
    if (n_layers > 0 && ((ffn & 15) || ffn <= 0)) return fail(SQAP_EUNSUPPORTED, "sqap_decoder_create: ffn = %d (multiple of 16)", ffn);
    if (!gamma_final || (reinterpret_cast<uintptr_t>(gamma_final) & 15u))
        return fail(SQAP_EINVAL, "sqap_decoder_create: final norm gain null or not 16-byte aligned");
    add(kStepHead, n_layers, hw, gamma_final, nullptr, 0);
    // what the kernel's fixed-size pieces hold
    for (const StepPhase &p : ph) {
        if (p.K > kStepMaxK || (p.K & 127)) return fail(SQAP_EUNSUPPORTED, "sqap_decoder_create: K = %d (multiple of 128, <= %d)", p.K, kStepMaxK);
        if (p.N & 1) return fail(SQAP_EUNSUPPORTED, "sqap_decoder_create: N = %d is odd", p.N);
        const int per = (p.units + kStepBlocks - 1) / kStepBlocks * (p.kind == kStepGateUp ? 2 : 1);
        if (per > kStepMaxGroups)
            return fail(SQAP_EUNSUPPORTED, "sqap_decoder_create: a %d x %d linear is too large for one launch (%d channel groups "
                        "per compute unit)", p.N, p.K, per);
    }
    Decoder *d = new (std::nothrow) Decoder();
    if (!d) return fail(SQAP_ENOMEM, "sqap_decoder_create: host allocation failed");
    d->magic = kDecoderMagic;
    d->n_layers = n_layers;
    d->hidden = hidden;
    d->ffn = ffn > 0 ? ffn : hidden;
    d->H = n_heads;
    d->d = head_dim;
    d->vocab = hw->N;
    d->eps = eps;
    d->base = rope_base;
    d->n_phases = (int)ph.size();
    d->blocks = kStepBlocks;
    d->phases = nullptr;
    d->rows = nullptr;
    d->sync = nullptr;
    auto round8 = [](size_t n) { return (n + 63) & ~(size_t)63; };
    size_t off = round8(hidden);
    d->off_r2 = off; off += round8(hidden);
    d->off_qkv = off; off += round8(3 * (size_t)hidden);
    d->off_attn = off; off += round8(hidden);
    d->off_o = off; off += round8(hidden);
    d->off_h = off; off += round8(d->ffn);
    d->off_dn = off; off += round8(hidden);
    hipError_t e = hipGetDevice(&d->device);
    int cus = 0;
    if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, d->device);
    if (e == hipSuccess && cus < kStepBlocks) {
        delete d;
        return fail(SQAP_EUNSUPPORTED, "sqap_decoder_create: the step kernel needs %d compute units, the device has %d",
                    kStepBlocks, cus);
    }
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&d->phases), sizeof(StepPhase) * ph.size());
    if (e == hipSuccess) e = hipMemcpy(d->phases, ph.data(), sizeof(StepPhase) * ph.size(), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&d->rows), off * sizeof(__half));
    if (e == hipSuccess) e = hipMemset(d->rows, 0, off * sizeof(__half));
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&d->sync), (kStepBlocks + 2) * sizeof(unsigned long long));
    if (e == hipSuccess) e = hipMemset(d->sync, 0, (kStepBlocks + 2) * sizeof(unsigned long long));
    if (e == hipSuccess)
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(&decoder_step_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)sizeof(StepLds));
    if (e != hipSuccess) {
        if (d->phases) (void)hipFree(d->phases);
        if (d->rows) (void)hipFree(d->rows);
        if (d->sync) (void)hipFree(d->sync);
        delete d;
        return fail(e == hipErrorOutOfMemory ? SQAP_ENOMEM : SQAP_EDEVICE, "sqap_decoder_create: %s", hipGetErrorString(e));
    }
    *out = d;
    return SQAP_OK;
}

sqap_status decoder_step(Decoder *d, const sqap_f16 *x, const int32_t *pos, int past, sqap_f16 *logits,
                         sqap_f16 *attn_trace, hipStream_t st)
{
    StepArgs a = {};
    a.phases = d->phases;
    a.n_phases = d->n_phases;
    a.blocks = d->blocks;
    a.hidden = d->hidden;
    a.ffn = d->ffn;
    a.H = d->H;
    a.d = d->d;
    a.eps = d->eps;
    a.base = d->base;
    a.x_in = reinterpret_cast<const __half *>(x);
    a.pos = pos;
    a.past = past;
    a.r1 = d->rows;
    a.r2 = d->rows + d->off_r2;
    a.qkv = d->rows + d->off_qkv;
    a.attn = d->rows + d->off_attn;
    a.o = d->rows + d->off_o;
    a.h = d->rows + d->off_h;
    a.dn = d->rows + d->off_dn;
    a.logits = reinterpret_cast<__half *>(logits);
    a.attn_trace = reinterpret_cast<__half *>(attn_trace);
    a.flags = d->sync;
    a.gen = d->sync + kStepBlocks;
    a.err = d->sync + kStepBlocks + 1;
    a.freq = rope_frequencies(d->d, d->base);
    hipLaunchKernelGGL(decoder_step_kernel, dim3(d->blocks), dim3(kStepThreads), sizeof(StepLds), st, a);
    SQAP_HIP_CHECK(hipGetLastError());
    return SQAP_OK;
}

sqap_status decoder_error(const Decoder *d, unsigned long long *word_out, hipStream_t st)
{
    SQAP_HIP_CHECK(hipMemcpyAsync(word_out, d->sync + kStepBlocks + 1, sizeof(unsigned long long), hipMemcpyDeviceToHost, st));
    SQAP_HIP_CHECK(hipStreamSynchronize(st));
    return SQAP_OK;
}

sqap_status decoder_free(Decoder *d)
{
    d->magic = 0;
    hipError_t e1 = hipFree(d->phases), e2 = hipFree(d->rows), e3 = hipFree(d->sync);
    delete d;
    const hipError_t e = e1 != hipSuccess ? e1 : e2 != hipSuccess ? e2 : e3;
    if (e != hipSuccess) return fail(SQAP_EDEVICE, "sqap_decoder_free: %s", hipGetErrorString(e));
    return SQAP_OK;
}

bool decoder_valid(const Decoder *d) { return d && d->magic == kDecoderMagic; }
int decoder_hidden(const Decoder *d) { return d->hidden; }

}  // namespace sqap
