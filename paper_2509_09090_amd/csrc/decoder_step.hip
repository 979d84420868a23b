// One decode step (one new token of one sequence through every layer and the vocabulary head) as ONE
// persistent launch.
//
// A decode step streams every weight once and each linear depends on the one before it.  As a chain of
// launches (nine per layer) a step costs the sum of their start-up and drain times: 2.6 ms per token for the
// 7B shape against 0.52 ms for the weights alone.  Here one workgroup per compute unit stays resident for
// the whole step and walks the linears in order:
//
//   phase  = [wait for the row the linear needs] -> [glue in front of the linear, redone by every workgroup]
//            -> [its share of the linear] -> [its outputs, tagged]
//   layer  = norm -> q|k|v | attention | quantize -> o | add, norm -> gate|up (+ SwiGLU) | quantize -> down
//
//   * The input of a linear is one row of at most 12288 values: every workgroup rebuilds it for itself (residual
//     add, RMSNorm with the exact sum of squares, int4 quantization: the arithmetic of the fused quantizer
//     kernels, statement by statement) and keeps the codes in LDS.  The residual stream never leaves the
//     workgroups: each keeps its own copy of the row in LDS and adds every update to it.
//   * A linear's output channels are dealt to the workgroups in runs of 16-channel groups; inside a
//     workgroup the seven streaming wavefronts split the run's reduction axis evenly and add through LDS.  With one
//     token there is nothing for a matrix core to reuse: each lane multiplies 32 weight codes of its
//     channel with the 32 activation codes by four v_dot8_i32_i4 (signed int4 x int4 -> int32, exact, no
//     widening).  A 1 KiB wavefront load is 16 channels x 4 pieces in the packed weight layout.
//   * Weights do not depend on activations, so the weight stream never waits for them: every streaming wavefront
//     walks ITS pieces of all the linears of the step as one sequence, twelve 1 KiB loads ahead of what
//     it multiplies, whatever phase those pieces belong to.  The loads land in a ring in LDS
//     (global_load_lds_dwordx4: no registers held, slots addressed at run time), 84 KiB per compute unit:
//     while the workgroup waits for a row or rebuilds it, the next linear's weights, and often those of the one
//     after, are arriving.  A full ring would stop the stream for the rest of the wait (slots only free up
//     when their pieces are multiplied), so before it waits a wavefront moves the eight oldest landed pieces
//     into registers and asks for eight more.
//   * gate and up channels are dealt in pairs, so the workgroup that owns a pair applies SwiGLU to it and only
//     h = silu(g) * u crosses to the down projection.
//   * What crosses workgroups (q|k|v, the attention output, o, h, the down projection's output) travels as
//     32-bit words: the half in the low 16 bits, a TAG in the high 16 bits that names the step and the place in
//     it (generation + 5 * layer + 1 .. 5) where the row is produced.  A producer stores its words, then its
//     progress flag, and goes on: nothing waits for a store.  A consumer polls the 256 flags (2 KiB, cheap) until
//     all producers have got that far, reads the row once, straight into LDS, and every thread checks the tags of
//     the words it uses; the flags say "stored", not "arrived", so a word can be late: then the row is read
//     again.  The tags decide, the flags only say when reading is worth while.  Against a barrier (data
//     complete, flag up, flag seen, data fetched) this saves the producer's wait for its stores; a word is
//     written by one 64-bit store of two tagged words, so it is never half old.  There is no barrier between
//     workgroups: a workgroup only ever waits for the rows it needs (the attention for its head's q, k, v: it
//     polls those three pieces directly).
//   * Every layer has row buffers of its own, so no address is written twice within a launch (caches are
//     invalidated between launches).  The first read of a row therefore goes through the caches: one workgroup
//     per chiplet pulls a line into the chiplet's L2, the other 31 hit there, instead of 256 reads past the
//     caches.  A line read too early all the same would stay stale in the caches; the tags show it and the
//     repeat reads past them (agent scope).  A workgroup that fell behind finds nothing newer than it waits for.
//   * Loads of a wavefront return in order, and a store counts as a load: a wavefront with weight loads in
//     flight would see the rows it polls only after all those loads have landed.  So the eighth wavefront
//     of the workgroup streams no weights: it polls the flags and reads the rows, the norm gains and the weight
//     scales into LDS, where all eight work on them (and, in a workgroup with a head, pulls the head's cached
//     keys and values into L2 ahead of the attention).  The weight stream is read with nontemporal loads, so
//     that it does not push those lines, the rows and the flags out of the L2 again.
//   * Barriers inside the workgroup wait for the wavefront's LDS operations only (lds_barrier): __syncthreads()
//     would also wait for every weight load in flight, several times per phase.  For the same reason LDS is
//     read and written as plain vectors (lds_load16) and every load in a path of the fetching wavefront is
//     waited for where the compiler can see it.
//   * The generation lives in device memory and moves on with every launch (the last workgroup to finish
//     writes it), so a launch captured in a graph can be replayed.  All 256 workgroups must be resident at
//     once: one per compute unit, checked at creation.  Every wait is bounded: a wait that gives up raises the
//     error word, and the step's result is then wrong and says so.
#include <new>
#include <vector>

#include "common.h"
#include "decode_attn.h"
#include "quant_math.h"

namespace sqap {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int kStepBlocks = 256;           // workgroups: one per compute unit, all resident at once
constexpr int kStepThreads = 512, kStepWaves = 8;
constexpr int kStepStreamWaves = 7;        // wavefronts 0 .. 6 stream weights; wavefront 7 reads the rows
constexpr int kStepGlueWave = 7;
constexpr int kStepRing = 12;              // 1 KiB weight loads in flight (or landed, not yet used) per streaming wavefront
constexpr int kStepPark = 8;               // landed pieces a wavefront moves from the ring into registers before it waits
constexpr int kStepMaxGroups = 16;         // 16-channel groups a workgroup owns in one phase
constexpr int kStepGpt = 3;                // groups of 8 row elements per thread: K <= 12288
constexpr int kStepMaxK = kStepThreads * 8 * kStepGpt;
constexpr int kStepMaxHidden = 4096;       // the residual row in LDS; a tagged row and the gains side by side
constexpr int kStepTagsPerLayer = 5;       // q|k|v, attention, o, h, down
constexpr int kStepWarmKeys = 2048;         // cached keys whose rows a workgroup warms the L2 cache with before its attention
constexpr long long kStepPollLimit = 200000;      // polls, or repeated reads of a row, before a wait gives up (a few tenths of a second)

enum StepKind { kStepQkv = 0, kStepO = 1, kStepGateUp = 2, kStepDown = 3, kStepHead = 4 };
enum StepTag { kTagQkv = 1, kTagAttn = 2, kTagO = 3, kTagH = 4, kTagDown = 5 };

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
    int n_phases, blocks, n_layers;
    int hidden, ffn, H, d;
    float eps;
    double base;
    const __half *x_in;     // [hidden] the token's embedding
    const int32_t *pos;     // [1]
    int past;
    unsigned *qkv, *attn, *o, *h, *dn;     // tagged rows of layer 0; layer l's are l * row_stride words further on
    size_t row_stride;
    __half *logits;
    __half *attn_trace;     // nullable: [layers, hidden]
    unsigned long long *flags, *gen, *err, *done;   // flags: one per workgroup
    long long poll_limit;   // polls (and repeated reads of a row) before a wait gives up
    RopeFreq freq;
};

constexpr int kStepStageWords = kStepMaxK;             // a tagged row of the longest kind
constexpr int kStepStageWarm = 10240 + 3 * 256;       // word offset of 1 KiB that only receives the cache-warming loads
constexpr int kStepStageNew = 10240;                   // word offset of the staged q, k, v of the new token (3 x 256 words)
struct StepLds {
    __attribute__((aligned(16))) uint8_t xs[kStepMaxK / 2];                       // the linear's input row as int4 codes
    __attribute__((aligned(16))) int partial[kStepMaxGroups][kStepWaves][16];      // per wavefront sums of a group's 16 channels
    __attribute__((aligned(16))) unsigned swl[2][kStepMaxGroups * 8];              // weight scales of the workgroup's channels (pairs), by phase parity
    unsigned long long wsum[2 * kStepWaves];
    float wmax[kStepWaves];
    float sx;
    int stale[2];           // some word of the row just read does not carry its tag yet (by attempt parity)
    int dead;               // a wait gave up: later waits read once and return (the step's result is wrong and says so)
    double2 sincos_tab[kDecMaxD / 2];      // sine, cosine of the token's rotation angles (the same for every layer)
    __attribute__((aligned(16))) __half resid[kStepMaxHidden];                    // the residual stream (this workgroup's copy)
    union {                                // the attention runs between two fetches
        __attribute__((aligned(16))) unsigned stage[kStepStageWords];             // rows as fetched: tagged words; the gains behind them
        DecodeAttnLds attn;
    };
    __attribute__((aligned(16))) uint8_t ring[kStepStreamWaves][kStepRing][1024];   // weights asked for, per streaming wavefront
};
static_assert(sizeof(StepLds) <= 160 * 1024, "one workgroup per compute unit: all of its LDS");
static_assert(sizeof(DecodeAttnLds) <= kStepStageNew * 4 && (kStepStageWarm + 256) <= kStepStageWords,
              "the new token's staged q, k, v sit behind the attention's own LDS");
static_assert(kStepMaxHidden * 4 + kStepMaxHidden * 2 <= kStepStageWords * 4, "a tagged row and the gains");

// An entry of the phase table, read through the constant address space: the table is never written while the
// kernel runs and the index is wavefront-uniform, so these become scalar loads, which do not queue behind the
// weight loads in flight (a vector load would: the first use of its result waits for every older load).
__device__ __forceinline__ StepPhase load_phase(const StepPhase *table, int ph)
{
    typedef const __attribute__((address_space(4))) unsigned long long *Words;
    static_assert(sizeof(StepPhase) == 64, "eight 64-bit words");
    const Words w = (Words)(unsigned long long)(table + __builtin_amdgcn_readfirstlane(ph));
    unsigned long long v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = w[i];
    StepPhase P;
    __builtin_memcpy(&P, v, sizeof(P));
    return P;
}

// 64 lanes x 16 bytes from global memory into 1 KiB of LDS at `to` (wavefront-uniform), no registers in between.
// AGENT: the load is coherent at agent scope (sc1).  Completion: vmcnt.
template <bool AGENT>
__device__ __forceinline__ void fetch_piece(const void *lane_from, void *to)
{
    __builtin_amdgcn_global_load_lds(reinterpret_cast<const SQAP_GLOBAL v4i *>((unsigned long long)lane_from),
                                     (__attribute__((address_space(3))) void *)to, 16, 0, AGENT ? 16 : 0);
}

// The empty asm makes x exist as a binary32 value: otherwise the compiler folds the operation that produced it
// and the conversion into one mixed-precision instruction that rounds only once.
__device__ __forceinline__ float to_half_value(float x)
{
    asm volatile("" : "+v"(x));
    return __half2float(__float2half_rn(x));
}

// two adjacent outputs as tagged words, one 64-bit store (agent scope: written through to where every
// workgroup reads)
__device__ __forceinline__ void store_tagged_pair(unsigned *row, int n, float y0, float y1, unsigned tag)
{
    const unsigned long long lo = (tag << 16) | __half_as_ushort(__float2half_rn(y0));
    const unsigned long long hi = (tag << 16) | __half_as_ushort(__float2half_rn(y1));
    __hip_atomic_store(reinterpret_cast<unsigned long long *>(row + n), lo | (hi << 32), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}

// ---- the pieces of the fused quantizer kernels' arithmetic, statement by statement ----
// RMSNorm:  x' = half(x + delta);  S = sum x'^2 as a 128-bit integer (add_squares8: the sum does not depend on
// the order);  r = (float)(1 / sqrt(S / K + eps))
// in binary64;  y = half((x' * r) * gamma).
// Quantizer:  scale = half(max|y| / 7) (2^-24 when that is zero), code = clamp(rint(y / scale), -8, 7).

// r from the eight wavefronts' sums (hi, lo pairs)
__device__ __forceinline__ float norm_factor(const unsigned long long *wsum, int K, float eps)
{
    unsigned long long hi = wsum[0], lo = wsum[1];
#pragma unroll
    for (int w = 1; w < kStepWaves; ++w) {
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
    // (eps widened here: hoisted out of the loop over the phases the double would sit in registers, in practice in
    // scratch memory, for the whole step)
    float e = eps;
    asm volatile("" : "+v"(e));
    return (float)(1.0 / sqrt(mean_of(Sd, K) + (double)e));
}

// ---- a workgroup's share of a linear ----
struct StepShare {
    int u0, n_groups;       // first unit, 16-channel groups owned (units x 1, or x 2 for gate|up)
    int i0, i1;             // this wavefront's items: (group, piece-of-four-chunks) pairs numbered group-major
    int Q;                  // items per group = chunks / 4
};

__device__ __forceinline__ StepShare step_share(const StepPhase &P, int block, int wave)
{
    StepShare s;
    // (the number of workgroups is a constant power of two: a shift, where a division by a launch argument would
    // be some hundred scalar instructions every time a wavefront's stream of pieces changes group)
    static_assert((kStepBlocks & (kStepBlocks - 1)) == 0, "power of two");
    s.u0 = (int)(((long long)P.units * block) / kStepBlocks);
    const int u1 = (int)(((long long)P.units * (block + 1)) / kStepBlocks);
    s.n_groups = (u1 - s.u0) * (P.kind == kStepGateUp ? 2 : 1);
    s.Q = P.chunks >> 2;
    const int total = s.n_groups * s.Q;
    if (wave < kStepStreamWaves) {
        s.i0 = total * wave / kStepStreamWaves;
        s.i1 = total * (wave + 1) / kStepStreamWaves;
    } else {
        s.i0 = s.i1 = 0;                               // the glue wavefront streams nothing
    }
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
        const StepPhase P = load_phase(a.phases, c.ph);
        const StepShare sh = step_share(P, block, wave);
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
    // (nontemporal: every weight byte is used once, and the stream should not push the rows, the flags and the
    // cached keys and values out of the L2)
    __builtin_amdgcn_global_load_lds(reinterpret_cast<const v4i *>(c.lane_ptr),
                                     (__attribute__((address_space(3))) void *)(&lds.ring[wave][c.slot][0]), 16, 0, 2);
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
        const StepPhase P = load_phase(a.phases, c.ph);
        const StepShare sh = step_share(P, block, wave);
        c.lane_ptr = reinterpret_cast<const uint8_t *>(step_item(P, sh, c.i, lane));
    }
}

// Every workgroup says how far it has got (generation + 5 * layer + 1 .. 5: everything it produces up to
// that point has been STORED, not necessarily arrived) in a flag of its own.  The glue wavefront reads the 256
// flags, four per lane, until all have reached `value`: a cheap hint that the row is worth reading.  The tags
// in the row decide.  False when it gave up.
__device__ __forceinline__ bool poll_flags(const unsigned long long *flags, int blocks, unsigned long long value, int lane,
                                           bool dead, long long poll_limit)
{
    if (dead) return false;
    for (long long round = 0;; ++round) {
        unsigned long long seen[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int f = lane + 64 * k;
            seen[k] = __hip_atomic_load(&flags[f < blocks ? f : blocks - 1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        const int here = (int)(seen[0] >= value) & (int)(seen[1] >= value) & (int)(seen[2] >= value) & (int)(seen[3] >= value);
        if (__all(here)) return true;
        if (round >= poll_limit) return false;
    }
}

// The glue wavefront waits for rows: `n` pieces of up to 1 KiB (piece(p, from, to, lanes): this lane's 16 bytes
// in global memory, the piece's place in LDS, the lanes that take part) are read into LDS until every word of
// every piece carries `tag` in its high half; pieces that do are not read again.  False when it gave up (or
// gave up before: then one read, so that LDS holds something to go on with).
template <class Piece>
__device__ __forceinline__ bool poll_pieces(int n, Piece piece, unsigned tag, int lane, bool dead, long long poll_limit)
{
    unsigned long long pending = n >= 64 ? ~0ull : (1ull << n) - 1ull;
    const unsigned want = tag << 16;
    const long long limit = dead ? 0 : poll_limit;
    for (long long round = 0; pending; ++round) {
        if (round > limit) return false;
        for (unsigned long long m = pending; m; m &= m - 1) {
            const int p = __builtin_ctzll(m);
            const unsigned *from;
            unsigned *to;
            int lanes;
            piece(p, from, to, lanes);
            if (lane < lanes) fetch_piece<true>(from, to);
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        for (unsigned long long m = pending; m; m &= m - 1) {
            const int p = __builtin_ctzll(m);
            const unsigned *from;
            unsigned *to;
            int lanes;
            piece(p, from, to, lanes);
            int ok = 1;
            if (lane < lanes) {
                const uint4 w = lds_load16(to + 4 * lane);
                ok = (int)((w.x & 0xffff0000u) == want) & (int)((w.y & 0xffff0000u) == want) &
                     (int)((w.z & 0xffff0000u) == want) & (int)((w.w & 0xffff0000u) == want);
            }
            if (__all(ok)) pending &= ~(1ull << p);
        }
    }
    return true;
}

// Diagnostic builds (-DSQAP_STEP_STAMPS) record the 100 MHz wall clock of four workgroups at eight points of every
// phase behind the attention trace; product builds compile the macro away.
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
    const bool glue = wave == kStepGlueWave;
    const int block = blockIdx.x;
    const unsigned long long gen0 = *a.gen;            // left by the launch before this one
    auto tag_of = [&](int layer, int what) { return (unsigned)((gen0 + (unsigned long long)(kStepTagsPerLayer * layer + what)) & 0xffffull); };
    const int pos0 = a.pos[0];
    if (block == 0 && t == 0) __hip_atomic_store(a.err, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (t == 0) {
        lds.dead = 0;
        lds.stale[0] = lds.stale[1] = 0;
    }
    if (block < a.H && t < (a.d >> 1)) {               // the rotation's sines and cosines: once per step instead of per layer
        double sn, cs;
        sincos(rope_angle(a.freq, pos0, t, a.d, a.base), &sn, &cs);
        lds.sincos_tab[t] = double2{sn, cs};
    }
    if (glue) {                                        // the token's embedding starts the residual stream
        for (int g0 = 0; g0 < (a.hidden >> 3); g0 += 64)
            if (g0 + lane < (a.hidden >> 3))
                fetch_piece<false>(reinterpret_cast<const uint4 *>(a.x_in) + g0 + lane, lds.resid + g0 * 8);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    lds_barrier();

    StepStream stream = {};
    stream_enter(stream, a, block, wave, lane);        // (the glue wavefront's sequence is empty)
    for (int k = 0; k < kStepRing; ++k) stream_issue(stream, a, lds, block, wave, lane);
    int consumed = 0, cslot = 0;                       // pieces that have left the ring so far; ring slot of the oldest one in it
    v4i park[kStepPark];                               // the oldest pieces not yet multiplied, moved out of the ring
    int park_c = 0, park_n = 0;                        // park[park_c .. park_n) are waiting
    // A streaming wavefront that is about to wait: once the pieces it asked for have landed it moves the oldest
    // into the park registers (when those are empty) and asks for as many new ones.
    auto park_pieces = [&]() {
        if (glue) return;
        if (park_c != park_n) return;
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
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
    // the glue wavefront's wait gave up
    auto give_up = [&](int ph, int what) {
        if (!lds.dead) __hip_atomic_store(a.err, ((unsigned long long)(ph + 1) << 8) | (unsigned long long)what, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        lds.dead = 1;
    };

    for (int ph = 0; ph < a.n_phases; ++ph) {
        const StepPhase P = load_phase(a.phases, ph);
        const StepShare share = step_share(P, block, wave);
        const StepShare all = step_share(P, block, 0);                  // (the group numbers do not depend on the wavefront)
        const bool gate_up = P.kind == kStepGateUp;
        const int n_out = gate_up ? all.n_groups >> 1 : all.n_groups;             // groups of 16 outputs
        const int K = P.K, groups = K >> 3;
        STEP_STAMP(0);
        // ---- the row this linear needs: an update of the residual stream (q|k|v, gate|up, head) or its whole input ----
        // (a layer's rows have addresses of their own: within a launch no address is written twice, so a row can be
        // read through the caches, and a workgroup that fell behind finds nothing newer than it waits for)
        const size_t mine = (size_t)(P.kind == kStepHead ? P.layer - 1 : P.layer) * a.row_stride, before = (size_t)(P.layer > 0 ? P.layer - 1 : 0) * a.row_stride;
        const unsigned *row = nullptr;
        int row_at = 0;                                // where in the step the row is produced: 5 * layer + 1 .. 5
        if (P.kind == kStepQkv) {
            row = P.layer == 0 ? nullptr : a.dn + before;
            row_at = kStepTagsPerLayer * (P.layer - 1) + kTagDown;
        } else if (P.kind == kStepGateUp) {
            row = a.o + mine;
            row_at = kStepTagsPerLayer * P.layer + kTagO;
        } else if (P.kind == kStepHead) {
            row = a.dn + before;
            row_at = kStepTagsPerLayer * (P.layer - 1) + kTagDown;
        } else if (P.kind == kStepO) {
            row = all.n_groups ? a.attn + mine : nullptr;     // (a workgroup with no channels of a linear skips its input)
            row_at = kStepTagsPerLayer * P.layer + kTagAttn;
        } else {
            row = all.n_groups ? a.h + mine : nullptr;
            row_at = kStepTagsPerLayer * P.layer + kTagH;
        }
        __half *st_gamma = reinterpret_cast<__half *>(lds.stage + K);             // the gains, behind the tagged row
        const unsigned want = (unsigned)((gen0 + (unsigned long long)row_at) & 0xffffull) << 16;
        // The glue wavefront waits for the flags, then reads the row once; every thread checks the tags of the words
        // it uses while it starts on the row.  A word that arrived later than its workgroup's flag is rare: then the
        // row is read again (nothing has been written by then: the residual row is updated after the check).
        float v[kStepGpt][8];
        for (int attempt = 0;; ++attempt) {
            if (glue) {
                // 1 KiB per instruction, straight into LDS (lane l's 16 bytes land at l * 16: the rows keep their layout)
                // The weight scales of the workgroup's channels, two per word (padded to whole groups), are not in any
                // cache yet: asked for now, they arrive while the row is waited for.  (The outputs of the phase
                // before may still be reading theirs: two places, by phase parity.)
                if (attempt == 0)
                    for (int it = 0; it < 2; ++it) {
                        const int w = lane + 64 * it;
                        if (w < all.n_groups * 8)
                            __builtin_amdgcn_global_load_lds((const SQAP_GLOBAL unsigned *)(P.sw + step_group(P, all, w >> 3) * 16 + (w & 7) * 2),
                                                             (__attribute__((address_space(3))) void *)(&lds.swl[ph & 1][64 * it]), 4, 0, 0);
                    }
                if (P.gamma && attempt == 0)
                    for (int g0 = 0; g0 < groups; g0 += 64)
                        if (g0 + lane < groups)
                            fetch_piece<false>(reinterpret_cast<const uint4 *>(P.gamma) + g0 + lane, st_gamma + g0 * 8);
                if (row) {
                    if (attempt == 0 && !poll_flags(a.flags, a.blocks, gen0 + (unsigned long long)row_at, lane, lds.dead != 0, a.poll_limit)) give_up(ph, 1);
                    const unsigned *from = row + lane * 4;
                    const int full = K >> 8;
                    // First through the caches (the first workgroup of a chiplet to ask brings a line into the chiplet's
                    // L2 for the other 31): nobody has read these addresses in this launch, and the flags say that the
                    // row has been stored.  A line that was read too early all the same stays stale in the caches: the
                    // tags show it, and the row is read again past the caches (agent scope).
                    if (attempt == 0) {
                        for (int p = 0; p < full; ++p) fetch_piece<false>(from + p * 256, lds.stage + p * 256);
                        if ((K & 255) && lane < ((K & 255) >> 2)) fetch_piece<false>(from + full * 256, lds.stage + full * 256);
                    } else {
                        for (int p = 0; p < full; ++p) fetch_piece<true>(from + p * 256, lds.stage + p * 256);
                        if ((K & 255) && lane < ((K & 255) >> 2)) fetch_piece<true>(from + full * 256, lds.stage + full * 256);
                    }
                }
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            } else if (attempt == 0) {
                park_pieces();
            }
            lds_barrier();
            if (attempt == 0) STEP_STAMP(1);
            unsigned bad = 0;
            unsigned long long hi = 0, lo = 0;
            float amax = 0.f;
#pragma unroll
            for (int gi = 0; gi < kStepGpt; ++gi) {
                const int g = t + gi * kStepThreads;
#pragma unroll
                for (int e = 0; e < 8; ++e) v[gi][e] = 0.f;
                if (g < groups) {
                    float in[8] = {};
                    if (row) {
                        const uint4 w0 = lds_load16(lds.stage + 8 * g), w1 = lds_load16(lds.stage + 8 * g + 4);
                        bad |= (w0.x ^ want) | (w0.y ^ want) | (w0.z ^ want) | (w0.w ^ want) | (w1.x ^ want) | (w1.y ^ want) |
                               (w1.z ^ want) | (w1.w ^ want);
                        const unsigned x[8] = {w0.x, w0.y, w0.z, w0.w, w1.x, w1.y, w1.z, w1.w};
#pragma unroll
                        for (int e = 0; e < 8; ++e) in[e] = __half2float(untag(x[e]));
                    }
                    if (P.gamma) {                     // the row is an update of the residual stream
                        unpack_halves(lds_load16(lds.resid + 8 * g), v[gi]);
                        if (row) {
#pragma unroll
                            for (int e = 0; e < 8; ++e) v[gi][e] = to_half_value(v[gi][e] + in[e]);
                        }
                        add_squares8(v[gi], hi, lo);
                    } else {                           // the row is the linear's input
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            v[gi][e] = in[e];
                            amax = fmaxf(amax, fabsf(in[e]));
                        }
                    }
                }
            }
            if (P.gamma) {
                wave_sum128(hi, lo);
                if (lane == 0) {
                    lds.wsum[2 * wave] = hi;
                    lds.wsum[2 * wave + 1] = lo;
                }
            } else {
                amax = wavefront_max(amax);
                if (lane == 0) lds.wmax[wave] = amax;
            }
            if (__any((bad >> 16) != 0) && lane == 0) lds.stale[attempt & 1] = 1;
            lds_barrier();
            if (t == 0) lds.stale[(attempt + 1) & 1] = 0;      // (its last readers have passed the barrier before this one)
            if (!row || !lds.stale[attempt & 1] || lds.dead) break;
            if (attempt >= a.poll_limit) {
                if (glue) give_up(ph, 3);
                break;
            }
            if (glue) __builtin_amdgcn_s_sleep(8);
        }
        if (P.gamma) {
            const float r = norm_factor(lds.wsum, K, a.eps);
            float amax = 0.f;
#pragma unroll
            for (int gi = 0; gi < kStepGpt; ++gi) {
                const int g = t + gi * kStepThreads;
                if (g < groups) {
                    if (row) {                         // x' is the residual stream from here on
                        uint4 raw;
                        __half2 *h2 = reinterpret_cast<__half2 *>(&raw);
#pragma unroll
                        for (int q = 0; q < 4; ++q) h2[q] = __floats2half2_rn(v[gi][2 * q], v[gi][2 * q + 1]);
                        lds_store16(lds.resid + 8 * g, raw);
                    }
                    float gm[8];
                    unpack_halves(lds_load16(st_gamma + 8 * g), gm);
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const float xr = v[gi][e] * r;
                        v[gi][e] = to_half_value(xr * gm[e]);
                        amax = fmaxf(amax, fabsf(v[gi][e]));
                    }
                }
            }
            amax = wavefront_max(amax);
            if (lane == 0) lds.wmax[wave] = amax;
            lds_barrier();
        }
        {
            float amax = lds.wmax[0];
#pragma unroll
            for (int w = 1; w < kStepWaves; ++w) amax = fmaxf(amax, lds.wmax[w]);
            const float sf = __half2float(row_scale(amax));
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
        }
        // ---- this workgroup's channels: the streaming wavefronts split the reduction axis ----
        for (int i = t; i < kStepMaxGroups * kStepWaves * 16; i += kStepThreads) (&lds.partial[0][0][0])[i] = 0;
        lds_barrier();
        STEP_STAMP(2);
        if (glue) {
            // A workgroup with a head: the cached keys and values it is about to attend over are known since the
            // step began.  One word of every 128-byte line of them is asked for now (and dropped), so that the
            // attention's own loads, which sit in the step's dependency chain, find the lines in the L2 cache.
            if (P.kind == kStepQkv && block < a.H) {
                const int lines_per_row = (a.d * 2 + 127) >> 7;                   // of the head's part of a key or value row
                const int n_lines = min(a.past, kStepWarmKeys) * 2 * lines_per_row;
                for (int i = lane; i < n_lines; i += 64) {
                    const int key = i / (2 * lines_per_row), part = i - key * 2 * lines_per_row;
                    const int kv = part / lines_per_row, line = part - kv * lines_per_row;
                    const __half *at = P.kv + (size_t)key * P.ldkv + (size_t)kv * a.hidden + (size_t)block * a.d + line * 64;
                    // (into a corner of LDS that nothing reads: a load into LDS holds no register, so nothing
                    // has to be kept free until it returns)
                    fetch_piece<false>(at, lds.stage + kStepStageWarm);
                }
            }
        } else {
            int acc = 0;
            int j = share.i0 < share.i1 ? share.i0 / share.Q : 0, q = share.i0 < share.i1 ? share.i0 - j * share.Q : 0;
            auto flush = [&]() {
                const int sum = rows_sum(acc);
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
            if (park_c == 0) {                         // (the usual case: one comparison per piece)
                const int left = share.i1 - i, n_use = park_n < left ? park_n : left;
#pragma unroll
                for (int dd = 0; dd < kStepPark; ++dd)
                    if (dd < n_use) multiply(park[dd]);
                park_c = n_use;
                i += n_use;
            } else {
#pragma unroll
                for (int dd = 0; dd < kStepPark; ++dd)
                    if (dd >= park_c && dd < park_n && i < share.i1) {
                        multiply(park[dd]);
                        ++park_c;
                        ++i;
                    }
            }
            for (; i < share.i1; ++i) {
                // The piece to multiply was asked for kStepRing pieces ago (fewer at the very end of the step): it
                // has landed once at most the younger pieces are still on their way (loads return in order; the
                // wavefront's output stores are in the same queue and at worst make this wait a little longer).
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
        lds_barrier();
        STEP_STAMP(3);
        // ---- outputs: two adjacent channels per thread; nothing waits for the stores ----
        if (t < n_out * 8) {
            const float sxf = lds.sx;
            // (what depends on the thread alone is formed here, from a value the compiler takes as new: hoisted out
            // of the loop over the phases it would sit in registers, in practice in scratch memory, for the whole step)
            int te = t;
            asm volatile("" : "+v"(te));
            const int jo = te >> 3, row2 = (te & 7) * 2;
            auto channel_pair = [&](int j, float (&y)[2]) {       // dequantised outputs of local group j, rows row2, row2 + 1
                int s0 = 0, s1 = 0;
#pragma unroll
                for (int w = 0; w < kStepStreamWaves; ++w) {
                    s0 += lds.partial[j][w][row2];
                    s1 += lds.partial[j][w][row2 + 1];
                }
                const unsigned swb = lds.swl[ph & 1][j * 8 + (te & 7)];
                const __half2 sw2 = *reinterpret_cast<const __half2 *>(&swb);
                float y0 = ((float)s0 * sxf) * __low2float(sw2), y1 = ((float)s1 * sxf) * __high2float(sw2);
                asm volatile("" : "+v"(y0), "+v"(y1));            // two binary32 products, then one rounding to half
                y[0] = __half2float(__float2half_rn(y0));
                y[1] = __half2float(__float2half_rn(y1));
            };
            const int n = (all.u0 + jo) * 16 + row2;
            float y[2];
            if (!gate_up) {
                channel_pair(jo, y);
                if (n < P.N) {
                    if (P.kind == kStepHead) {
                        const __half2 pk = __floats2half2_rn(y[0], y[1]);
                        *(SQAP_GLOBAL unsigned *)(a.logits + n) = *reinterpret_cast<const unsigned *>(&pk);
                    } else if (P.kind == kStepQkv) {
                        store_tagged_pair(a.qkv + mine, n, y[0], y[1], tag_of(P.layer, kTagQkv));
                    } else if (P.kind == kStepO) {
                        store_tagged_pair(a.o + mine, n, y[0], y[1], tag_of(P.layer, kTagO));
                    } else {
                        store_tagged_pair(a.dn + mine, n, y[0], y[1], tag_of(P.layer, kTagDown));
                    }
                }
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
                if (n < (P.N >> 1)) store_tagged_pair(a.h + mine, n, y[0], y[1], tag_of(P.layer, kTagH));
            }
        }
        // how far this workgroup has got (a workgroup without a head has nothing to add to the attention's row)
        const bool attends = P.kind == kStepQkv && block < a.H;
        if (P.kind != kStepHead && !attends && t == (n_out * 8 > 64 ? 64 : 0)) {
            const int at = kStepTagsPerLayer * P.layer + (P.kind == kStepQkv ? kTagAttn : P.kind == kStepO ? kTagO : gate_up ? kTagH : kTagDown);
            __hip_atomic_store(&a.flags[block], gen0 + (unsigned long long)at, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        STEP_STAMP(4);
        if (attends) {
            // attention of the new token over the layer's cache: one workgroup per head; its q, k, v come as three
            // pieces of d tagged words
            if (glue) {
                const bool ok = poll_pieces(3,
                                            [&](int p, const unsigned *&from, unsigned *&to, int &lanes) {
                                                from = a.qkv + mine + (size_t)p * a.hidden + (size_t)block * a.d + lane * 4;
                                                to = lds.stage + kStepStageNew + p * 256;
                                                lanes = a.d >> 2;
                                            },
                                            tag_of(P.layer, kTagQkv), lane, lds.dead != 0, a.poll_limit);
                if (!ok) give_up(ph, 2);
            }
            STEP_STAMP(5);
            decode_attention_head<true>(lds.attn, block, nullptr, pos0, a.H, a.d, a.base, P.kv, P.ldkv, a.past, a.attn + mine,
                                        a.attn_trace ? a.attn_trace + (size_t)P.layer * a.hidden : nullptr, a.freq, lds.sincos_tab,
                                        lds.stage + kStepStageNew, tag_of(P.layer, kTagAttn));
            if (t == 64)
                __hip_atomic_store(&a.flags[block], gen0 + (unsigned long long)(kStepTagsPerLayer * P.layer + kTagAttn), __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
            lds_barrier();                           // its LDS is where the next row lands
            STEP_STAMP(6);
        }
    }
    // The last workgroup to get here moves the generation on for the next launch: by then every workgroup has
    // read it.  (One read-modify-write per workgroup and launch.)
    if (t == 0) {
        const unsigned long long before = __hip_atomic_fetch_add(a.done, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if ((before + 1ull) % (unsigned long long)kStepBlocks == 0ull)
            __hip_atomic_store(a.gen, gen0 + (unsigned long long)(kStepTagsPerLayer * a.n_layers), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// ---------------------------------------------------------------------------------------------
struct Decoder {
    uint32_t magic;
    int device, n_layers, hidden, ffn, H, d, vocab, n_phases, blocks;
    float eps;
    double base;
    StepPhase *phases;          // device
    unsigned *rows;             // device, tagged words: qkv, attn, o, h, dn
    unsigned long long *sync;   // device: generation, error word, count of finished workgroups, flags[256]
    size_t off_attn, off_o, off_h, off_dn, row_stride;
    long long poll_limit;
};
constexpr uint32_t kDecoderMagic = 0x53514443u;  // "SQDC"
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
    if (hidden > kStepMaxHidden) return fail(SQAP_EUNSUPPORTED, "sqap_decoder_create: hidden = %d above %d", hidden, kStepMaxHidden);
    if ((long long)kStepTagsPerLayer * n_layers >= 65536) return fail(SQAP_EUNSUPPORTED, "sqap_decoder_create: %d layers", n_layers);
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
    d->poll_limit = kStepPollLimit;
    d->phases = nullptr;
    d->rows = nullptr;
    d->sync = nullptr;
    auto round64 = [](size_t n) { return (n + 63) & ~(size_t)63; };
    size_t off = round64(3 * (size_t)hidden);       // q|k|v first
    d->off_attn = off; off += round64(hidden);
    d->off_o = off; off += round64(hidden);
    d->off_h = off; off += round64(d->ffn);
    d->off_dn = off; off += round64(hidden);
    d->row_stride = off;                            // every layer has rows of its own
    off *= (size_t)n_layers;
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
    // rows start with tag 0 everywhere, the generation at 1: the first step waits for tags from 2 on
    std::vector<unsigned long long> sync0(3 + kStepBlocks, 0ull);
    sync0[0] = 1ull;
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&d->rows), off * sizeof(unsigned));
    if (e == hipSuccess) e = hipMemset(d->rows, 0, off * sizeof(unsigned));
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&d->sync), sync0.size() * sizeof(unsigned long long));
    if (e == hipSuccess) e = hipMemcpy(d->sync, sync0.data(), sync0.size() * sizeof(unsigned long long), hipMemcpyHostToDevice);
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
    a.n_layers = d->n_layers;
    a.hidden = d->hidden;
    a.ffn = d->ffn;
    a.H = d->H;
    a.d = d->d;
    a.eps = d->eps;
    a.base = d->base;
    a.x_in = reinterpret_cast<const __half *>(x);
    a.pos = pos;
    a.past = past;
    a.qkv = d->rows;
    a.attn = d->rows + d->off_attn;
    a.o = d->rows + d->off_o;
    a.h = d->rows + d->off_h;
    a.dn = d->rows + d->off_dn;
    a.row_stride = d->row_stride;
    a.poll_limit = d->poll_limit;
    a.logits = reinterpret_cast<__half *>(logits);
    a.attn_trace = reinterpret_cast<__half *>(attn_trace);
    a.gen = d->sync;
    a.err = d->sync + 1;
    a.done = d->sync + 2;
    a.flags = d->sync + 3;
    a.freq = rope_frequencies(d->d, d->base);
    hipLaunchKernelGGL(decoder_step_kernel, dim3(d->blocks), dim3(kStepThreads), sizeof(StepLds), st, a);
    SQAP_HIP_CHECK(hipGetLastError());
    return SQAP_OK;
}

sqap_status decoder_error(const Decoder *d, unsigned long long *word_out, hipStream_t st)
{
    SQAP_HIP_CHECK(hipMemcpyAsync(word_out, d->sync + 1, sizeof(unsigned long long), hipMemcpyDeviceToHost, st));
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
void decoder_set_wait_limit(Decoder *d, long long polls) { d->poll_limit = polls < 0 ? kStepPollLimit : polls; }
int decoder_hidden(const Decoder *d) { return d->hidden; }

}  // namespace sqap
