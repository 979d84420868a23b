// Internal helpers of the gfx950 library (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>

#include <atomic>
#include <type_traits>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "sqap.h"

namespace sqap {

// Records the message returned by sqap_last_error() and passes the status through.
sqap_status fail(sqap_status st, const char *fmt, ...);

// Packed weight: device copy in the streaming layout used by the GEMM kernels.
//
// Layout of `data`: rows are grouped by 32 and the reduction axis by chunks of
// 32 codes (16 bytes).  For row group g (rows 32g .. 32g+31) and chunk c the
// 512 bytes at ((g * chunks + c) * 512) hold, for r = 0..31, the 16 packed
// bytes of row 32g + r, codes 32c .. 32c+31, unchanged from the canonical
// layout.  The number of row groups is rounded up to a multiple of 8 (256 rows)
// so that a GEMM tile never needs a guard in N; rows past N are zero.  A wavefront that reads 1 KiB contiguous gets
// two chunks of one row group, which is exactly the B operand of two
// 32x32x32 int8 MFMAs once nibbles are split (low nibbles -> one, high -> other).
struct Weight {
    uint32_t magic;
    int32_t N, K;
    int32_t n_groups;   // ceil(N / 256) * 8
    int32_t chunks;     // K / 32
    uint8_t *data;      // n_groups * chunks * 512 bytes
    __half *scales;     // n_groups * 32 halves (zero padded)
    size_t bytes;
    int device;
};
constexpr uint32_t kWeightMagic = 0x53514150u;  // "SQAP"

// One problem of a small-M launch (see skinny.hip).  rg_begin is the index of the
// problem's first work item (row group) in the launch-wide numbering.
struct SkinnyEntry {
    const uint8_t *Xq;
    const __half *sx;
    const uint8_t *Wd;
    const __half *sw;
    __half *Y;
    int32_t *acc_out;   // nullable
    int64_t ldy;
    int M, N, chunks, rg_begin;
    long long cost_begin;   // sum over earlier problems of row groups * chunks
};
constexpr int kSkinnyInline = 4;
struct SkinnyArgs {
    const SkinnyEntry *table;   // device table, or null to use inline_entries
    int count, total_items, xs_bytes;
    int out_off, out_cap;       // output slots in LDS: byte offset, slots per wavefront (0: outputs are stored at once)
    long long total_cost;
    SkinnyEntry inline_entries[kSkinnyInline];
};
constexpr int kSkinnyMaxM = 8;

// Device-resident table of small-M problems, run by one launch.
struct Group {
    uint32_t magic;
    int count, total_items, max_chunks;
    long long total_cost;
    SkinnyEntry *table;   // device
    int device;
};
constexpr uint32_t kGroupMagic = 0x53514752u;  // "SQGR"

static inline hipStream_t as_stream(void *s) { return reinterpret_cast<hipStream_t>(s); }

// Launcher state that belongs to a device (function attributes set, CU count): one slot per device
// ordinal, atomics so that host threads may race to initialise it (every racer writes the same value).
constexpr int kMaxDeviceSlots = 64;
static inline int device_slot()
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0) dev = 0;
    return dev % kMaxDeviceSlots;
}
static inline int device_cu_count()
{
    static std::atomic<int> cus[kMaxDeviceSlots];
    const int slot = device_slot();
    int v = cus[slot].load(std::memory_order_relaxed);
    if (v == 0) {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0)
            v = 256;
        cus[slot].store(v, std::memory_order_relaxed);
    }
    return v;
}

#define SQAP_HIP_CHECK(expr)                                                          \
    do {                                                                              \
        hipError_t e_ = (expr);                                                       \
        if (e_ != hipSuccess)                                                         \
            return ::sqap::fail(SQAP_EDEVICE, "%s: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

// kernel launchers (defined in the .hip files); all validation is done by the caller
sqap_status launch_attn_scores(const __half *q, const __half *k, int batch, int S, int H, int d,
                               int vis_begin, int n_vis, float *scores, void *workspace, size_t workspace_bytes,
                               hipStream_t st);
size_t attn_scores_workspace_bytes(int batch, int H, int n_vis);
// variant whose scratch is a file-scope device array (prune.hip); limits of that array
sqap_status launch_attn_scores_noalloc(const __half *q, const __half *k, int batch, int S, int H, int d,
                                       int vis_begin, int n_vis, float *scores, hipStream_t st);
sqap_status noalloc_scratch(void **out);
size_t noalloc_max_weights();
int noalloc_max_batch();
sqap_status launch_prune_topk(const float *scores, int batch, int n, int keep_k, int32_t *idx,
                              hipStream_t st);
sqap_status launch_prune_rows(const float *scores, int batch, int n, int keep_k, int seq_len, int vis_begin,
                              int32_t *idx, int32_t *rows, hipStream_t st);
sqap_status launch_prune_select(const float *scores, int batch, int gw, int gh, int k_attn, int keep_total,
                                const double *camera, int radius, int32_t *idx, int cap, int32_t *count,
                                hipStream_t st);
sqap_status launch_kept_rows(const int32_t *idx, int batch, int keep_k, int seq_len,
                             int vis_begin, int n_vis, int32_t *rows, hipStream_t st);
sqap_status launch_gather_rows(const __half *X, int64_t ldx, const int32_t *rows, int M, int K,
                               __half *out, int64_t ldo, hipStream_t st);
sqap_status launch_quantize_rows(const __half *X, int64_t ldx, const int32_t *rows, int M, int K,
                                 bool rotate, uint8_t *Xq, __half *sx, hipStream_t st);
sqap_status launch_quantize_rows_scaled(const __half *X, int64_t ldx, const int32_t *rows, int M, int K,
                                        bool rotate, bool folded, const __half *col_scales, uint8_t *Xq,
                                        __half *sx, hipStream_t st);
// Operation fused in front of the quantizer (quantize.hip) and its operands.
enum PreOp { kPreNone = 0, kPreNorm = 1, kPreSwiglu = 2 };
struct PreArgs {
    const __half *delta;    // kPreNorm: residual update [M, K], nullable
    __half *xsum_out;       // kPreNorm: x + delta [M, K], nullable
    const __half *gamma;    // kPreNorm: [K]
    float eps;              // kPreNorm
    const __half *U;        // kPreSwiglu: up rows, pitch ldu
    int64_t ldu;
    __half *y_out;          // the half-precision result the quantizer sees, [M, K], nullable
};
sqap_status launch_fused_quantize(int pre_op, const __half *X, int64_t ldx, const int32_t *rows, int M, int K,
                                  bool rotate, const __half *col_scales, uint8_t *Xq, __half *sx,
                                  const PreArgs &pre, hipStream_t st);
sqap_status launch_channel_scales(const __half *X, int64_t ldx, const int32_t *rows, int M, int K, bool rotate,
                                  float *amax, bool accumulate, __half *scales, hipStream_t st);
sqap_status launch_weight_pack(const uint8_t *Wq, const __half *sw, const Weight &w,
                               hipStream_t st);
size_t linear_workspace_bytes(int M, int N, int K);
sqap_status launch_w4a4_linear(const uint8_t *Xq, const __half *sx, int M, const Weight &w,
                               __half *Y, int64_t ldy, int32_t *acc_out, void *workspace,
                               hipStream_t st);

// Few hundred token rows, K a multiple of 256: every workgroup owns complete outputs (gemm_rows.hip)
bool rows_kernel_applies(int M, int N, int K);
sqap_status launch_rows_linear(const uint8_t *Xq, const __half *sx, int M, const Weight &w, __half *Y, int64_t ldy,
                               int32_t *acc_out, hipStream_t st);
void set_mid_m_kernel(int which);        // 0: tiles split along K between workgroups, 1: whole outputs per workgroup

sqap_status launch_rope(__half *X, int64_t ld, const int32_t *pos, int S, int H, int d, double base, hipStream_t st);
sqap_status launch_rope_append(__half *QKV, int64_t ld, const int32_t *pos, int S, int H, int d, double base,
                               __half *KV, int64_t ldkv, hipStream_t st);
sqap_status launch_decode_attention(const __half *QKV, const int32_t *pos, int H, int d, double base, __half *KV,
                                    int64_t ldkv, int past, __half *O, uint8_t *Xq, __half *sx,
                                    unsigned int *counter, hipStream_t st);
sqap_status launch_attention(const __half *Q, int64_t ldq, const __half *Kc, int64_t ldk, const __half *V,
                             int64_t ldv, int batch, int Sq, int Sk, int H, int d, __half *O, int64_t ldo, hipStream_t st);
sqap_status launch_residual_add(__half *X, int64_t ldx, const __half *Dl, int64_t ldd, int M, int K, hipStream_t st);
sqap_status launch_quotient_selftest(unsigned long long *mismatches, hipStream_t st);
// Checks once per device how a launch's workgroups are dealt to the XCDs (see gemm.hip); table_out
// (host, 256 words, nullable) receives the XCC id of every workgroup and forces a fresh probe.
sqap_status probe_dispatch(int device, hipStream_t st, uint32_t *table_out);
void set_persistent_kernels(int enabled);
sqap_status plan_linear_shares(int M, int N, int K, int blocks_per_xcd, uint32_t *bounds_out, double *planned_out,
                               double *even_out, int *tile_rows_out, int *tile_cols_out);
// One decode step as one persistent launch (decoder_step.hip)
struct Decoder;
sqap_status decoder_create(const sqap_decoder_layer *layers, int n_layers, int n_heads, int head_dim,
                           const sqap_f16 *gamma_final, const sqap_weight *head, float eps, double rope_base,
                           Decoder **out);
sqap_status decoder_step(Decoder *d, const sqap_f16 *x, const int32_t *pos, int past, sqap_f16 *logits,
                         sqap_f16 *attn_trace, hipStream_t st);
sqap_status decoder_error(const Decoder *d, unsigned long long *word_out, hipStream_t st);
sqap_status decoder_free(Decoder *d);
bool decoder_valid(const Decoder *d);
void decoder_set_wait_limit(Decoder *d, long long polls);
sqap_status launch_skinny(const SkinnyArgs &args, int max_chunks, hipStream_t st);
void skinny_plan(int total_items, int max_chunks, int cus, int *S, int *W, int *out_cap);

// __syncthreads() is a release and an acquire fence around the barrier, and the release waits for every
// load and store of the wavefront, global ones included.  A wavefront that keeps a stream of weight loads in
// flight must not wait for those at every barrier: where the barrier only hands LDS contents from wavefront
// to wavefront, waiting for the wavefront's own LDS operations is enough (they complete in order, and a completed
// LDS write is visible to the whole workgroup).
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }


// Reductions over the wavefront with data-parallel-primitive moves instead of LDS permutes: inside a row of
// 16 lanes the partner is reached by quad permutes (xor 1, xor 2) and the two mirrors (7 - i within 8 lanes,
// 15 - i within 16), each a modifier on the instruction's operand, so after four steps every lane of a row
// holds the row's result; the four rows are read out as scalars.  A step costs a few cycles against the
// LDS round trip of a permute.
template <int CTRL>
__device__ __forceinline__ unsigned dpp_move(unsigned v)
{
    return (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xf, 0xf, false);
}
constexpr int kDppXor1 = 0xB1, kDppXor2 = 0x4E, kDppHalfMirror = 0x141, kDppMirror = 0x140;

// the same for a float, and a row's value (the same in its 16 lanes) of each of the four rows as scalars
template <int CTRL>
__device__ __forceinline__ float dpp_move_f(float v) { return __uint_as_float(dpp_move<CTRL>(__float_as_uint(v))); }
__device__ __forceinline__ float row_value(float v, int row)
{
    return __uint_as_float((unsigned)__builtin_amdgcn_readlane((int)__float_as_uint(v), 16 * row));
}

// the wavefront's maximum of non-negative values, in every lane
__device__ __forceinline__ float wavefront_max(float v)
{
    v = fmaxf(v, __uint_as_float(dpp_move<kDppXor1>(__float_as_uint(v))));
    v = fmaxf(v, __uint_as_float(dpp_move<kDppXor2>(__float_as_uint(v))));
    v = fmaxf(v, __uint_as_float(dpp_move<kDppHalfMirror>(__float_as_uint(v))));
    v = fmaxf(v, __uint_as_float(dpp_move<kDppMirror>(__float_as_uint(v))));
    const unsigned b = __float_as_uint(v);
    const float r0 = __uint_as_float((unsigned)__builtin_amdgcn_readlane((int)b, 0)), r1 = __uint_as_float((unsigned)__builtin_amdgcn_readlane((int)b, 16));
    const float r2 = __uint_as_float((unsigned)__builtin_amdgcn_readlane((int)b, 32)), r3 = __uint_as_float((unsigned)__builtin_amdgcn_readlane((int)b, 48));
    return fmaxf(fmaxf(r0, r1), fmaxf(r2, r3));
}

// the wavefront's 128-bit sum, in every lane
__device__ __forceinline__ void wave_sum128(unsigned long long &hi, unsigned long long &lo)
{
    auto step = [&](auto ctrl_c) {
        constexpr int CTRL = decltype(ctrl_c)::value;
        const unsigned long long olo = (unsigned long long)dpp_move<CTRL>((unsigned)lo) | ((unsigned long long)dpp_move<CTRL>((unsigned)(lo >> 32)) << 32);
        const unsigned long long ohi = (unsigned long long)dpp_move<CTRL>((unsigned)hi) | ((unsigned long long)dpp_move<CTRL>((unsigned)(hi >> 32)) << 32);
        lo += olo;
        hi += ohi + (lo < olo ? 1ull : 0ull);
    };
    step(std::integral_constant<int, kDppXor1>{});
    step(std::integral_constant<int, kDppXor2>{});
    step(std::integral_constant<int, kDppHalfMirror>{});
    step(std::integral_constant<int, kDppMirror>{});
    auto lane64 = [](unsigned long long v, int l) {
        return (unsigned long long)(unsigned)__builtin_amdgcn_readlane((int)(unsigned)v, l) |
               ((unsigned long long)(unsigned)__builtin_amdgcn_readlane((int)(unsigned)(v >> 32), l) << 32);
    };
    unsigned long long h = lane64(hi, 0), l = lane64(lo, 0);
#pragma unroll
    for (int r = 1; r < 4; ++r) {
        const unsigned long long ol = lane64(lo, 16 * r);
        l += ol;
        h += lane64(hi, 16 * r) + (l < ol ? 1ull : 0ull);
    }
    hi = h;
    lo = l;
}

// The sum of an integer over the four rows of 16 lanes (lanes l, l + 16, l + 32, l + 48), in every lane: the
// upper 32 lanes are exchanged with the lower (v_permlane32_swap), then the odd rows with the even
// (v_permlane16_swap); two vector-ALU instructions each, no LDS permute.
__device__ __forceinline__ int rows_sum(int v)
{
    const auto a = __builtin_amdgcn_permlane32_swap(v, v, false, false);
    v = (int)a[0] + (int)a[1];
    const auto b = __builtin_amdgcn_permlane16_swap(v, v, false, false);
    return (int)b[0] + (int)b[1];
}

}  // namespace sqap
