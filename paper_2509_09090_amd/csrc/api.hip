// C ABI of the library: argument validation on the host, then kernel launches.
// Declarations and the meaning of every argument are in include/sqap.h.
#include <stdarg.h>
#include <stdio.h>
#include <new>

#include "common.h"

namespace sqap {

static thread_local char g_error[512] = "";

sqap_status fail(sqap_status st, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof(g_error), fmt, ap);
    va_end(ap);
    return st;
}

static inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

static const Weight *check_weight(const sqap_weight *w)
{
    const Weight *ww = reinterpret_cast<const Weight *>(w);
    if (!ww || ww->magic != kWeightMagic) return nullptr;
    return ww;
}

}  // namespace sqap

using namespace sqap;

extern "C" {

const char *sqap_last_error(void) { return g_error; }

const char *sqap_version(void) { return "sqap-gfx950 0.1"; }

// workspace the fast kernel of the retention score needs for this shape (0: the shape takes the
// one-workgroup kernel, which needs none)
static size_t attn_scores_need(int32_t batch, int32_t S, int32_t H, int32_t d, int32_t n_vis)
{
    if (batch <= 0 || S <= 0 || S > 4096 || H <= 0 || d < 8 || d > 256 || (d & (d - 1)) || n_vis <= 0) return 0;
    return attn_scores_workspace_bytes(batch, H, n_vis);
}

static sqap_status attn_scores_checked(const char *who, const sqap_f16 *q, const sqap_f16 *k, int32_t batch,
                                       int32_t S, int32_t H, int32_t d, int32_t vis_begin, int32_t n_vis,
                                       float *scores_out, void *workspace, size_t workspace_bytes, void *stream)
{
    if (batch < 0) return fail(SQAP_EINVAL, "%s: batch %d < 0", who, batch);
    if (S <= 0 || H <= 0 || d <= 0)
        return fail(SQAP_EINVAL, "%s: S, H, d must be positive (%d, %d, %d)", who, S, H, d);
    if (vis_begin < 0 || n_vis < 0 || (int64_t)vis_begin + n_vis > S)
        return fail(SQAP_EINVAL, "%s: visual span [%d, %d+%d) outside [0, %d)", who, vis_begin, vis_begin, n_vis, S);
    if (batch == 0) return SQAP_OK;
    if (!q || !k) return fail(SQAP_EINVAL, "%s: null q or k", who);
    if (n_vis == 0) return SQAP_OK;
    if (!scores_out) return fail(SQAP_EINVAL, "%s: null scores_out", who);
    if (d > 256 || (d & 1)) return fail(SQAP_EUNSUPPORTED, "%s: d = %d (even, <= 256)", who, d);
    if (S > 16384) return fail(SQAP_EUNSUPPORTED, "%s: S = %d > 16384", who, S);
    if (batch > 4096) return fail(SQAP_EUNSUPPORTED, "%s: batch = %d > 4096", who, batch);
    const size_t need = aligned16(q) && aligned16(k) ? attn_scores_need(batch, S, H, d, n_vis) : 0;
    if (need > 0) {
        if (!workspace || workspace_bytes < need)
            return fail(SQAP_EINVAL, "%s: workspace of %zu bytes needed, %zu given", who, need,
                        workspace ? workspace_bytes : (size_t)0);
        if (!aligned16(workspace)) return fail(SQAP_EINVAL, "%s: workspace must be 16-byte aligned", who);
    }
    return launch_attn_scores(reinterpret_cast<const __half *>(q), reinterpret_cast<const __half *>(k), batch, S, H,
                              d, vis_begin, n_vis, scores_out, need > 0 ? workspace : nullptr, workspace_bytes,
                              as_stream(stream));
}

size_t sqap_attn_scores_workspace_bytes(int32_t batch, int32_t S, int32_t H, int32_t d, int32_t n_vis)
{
    return attn_scores_need(batch, S, H, d, n_vis);
}

sqap_status sqap_attn_scores(const sqap_f16 *q, const sqap_f16 *k, int32_t S, int32_t H,
                             int32_t d, int32_t vis_begin, int32_t n_vis, float *scores_out,
                             void *workspace, size_t workspace_bytes, void *stream)
{
    return attn_scores_checked("sqap_attn_scores", q, k, 1, S, H, d, vis_begin, n_vis, scores_out, workspace,
                               workspace_bytes, stream);
}

sqap_status sqap_attn_scores_batch(const sqap_f16 *q, const sqap_f16 *k, int32_t batch, int32_t S, int32_t H,
                                   int32_t d, int32_t vis_begin, int32_t n_vis, float *scores_out,
                                   void *workspace, size_t workspace_bytes, void *stream)
{
    return attn_scores_checked("sqap_attn_scores_batch", q, k, batch, S, H, d, vis_begin, n_vis, scores_out, workspace,
                               workspace_bytes, stream);
}

sqap_status sqap_attn_scores_noalloc(const sqap_f16 *q, const sqap_f16 *k, int32_t batch, int32_t S, int32_t H,
                                     int32_t d, int32_t vis_begin, int32_t n_vis, float *scores_out, void *stream)
{
    const char *who = "sqap_attn_scores_noalloc";
    if (batch < 0) return fail(SQAP_EINVAL, "%s: batch %d < 0", who, batch);
    if (S <= 0 || H <= 0 || d <= 0)
        return fail(SQAP_EINVAL, "%s: S, H, d must be positive (%d, %d, %d)", who, S, H, d);
    if (vis_begin < 0 || n_vis < 0 || (int64_t)vis_begin + n_vis > S)
        return fail(SQAP_EINVAL, "%s: visual span [%d, %d+%d) outside [0, %d)", who, vis_begin, vis_begin, n_vis, S);
    if (batch == 0) return SQAP_OK;
    if (!q || !k) return fail(SQAP_EINVAL, "%s: null q or k", who);
    if (n_vis == 0) return SQAP_OK;
    if (!scores_out) return fail(SQAP_EINVAL, "%s: null scores_out", who);
    if (d > 256 || (d & 1)) return fail(SQAP_EUNSUPPORTED, "%s: d = %d (even, <= 256)", who, d);
    if (S > 16384) return fail(SQAP_EUNSUPPORTED, "%s: S = %d > 16384", who, S);
    // what the file-scope scratch array holds
    if (batch > noalloc_max_batch())
        return fail(SQAP_EUNSUPPORTED, "%s: batch = %d above the %d observations the built-in scratch array holds", who,
                    batch, noalloc_max_batch());
    if ((uint64_t)batch * (uint64_t)H * (uint64_t)n_vis > noalloc_max_weights())
        return fail(SQAP_EUNSUPPORTED, "%s: batch * H * n_vis = %llu above the %zu per-head weights the built-in scratch "
                    "array holds", who, (unsigned long long)batch * H * n_vis, noalloc_max_weights());
    return launch_attn_scores_noalloc(reinterpret_cast<const __half *>(q), reinterpret_cast<const __half *>(k), batch, S,
                                      H, d, vis_begin, n_vis, scores_out, as_stream(stream));
}

sqap_status sqap_prune_topk(const float *scores, int32_t batch, int32_t n_tokens,
                            int32_t keep_k, int32_t *idx_out, void *stream)
{
    if (batch < 0 || n_tokens < 0 || keep_k < 0)
        return fail(SQAP_EINVAL, "sqap_prune_topk: negative size (batch %d, n %d, keep %d)", batch,
                    n_tokens, keep_k);
    if (keep_k > n_tokens)
        return fail(SQAP_EINVAL, "sqap_prune_topk: keep_k %d > n_tokens %d", keep_k, n_tokens);
    if (batch == 0 || keep_k == 0) return SQAP_OK;
    if (!scores || !idx_out) return fail(SQAP_EINVAL, "sqap_prune_topk: null pointer");
    if (n_tokens > 65536)
        return fail(SQAP_EUNSUPPORTED, "sqap_prune_topk: n_tokens %d > 65536", n_tokens);
    return launch_prune_topk(scores, batch, n_tokens, keep_k, idx_out, as_stream(stream));
}

sqap_status sqap_prune_rows(const float *scores, int32_t batch, int32_t n_vis, int32_t keep_k,
                            int32_t seq_len, int32_t vis_begin, int32_t *idx_out, int32_t *rows_out,
                            void *stream)
{
    if (batch < 0 || n_vis < 0 || keep_k < 0 || seq_len < 0 || vis_begin < 0)
        return fail(SQAP_EINVAL, "sqap_prune_rows: negative size");
    if (keep_k > n_vis) return fail(SQAP_EINVAL, "sqap_prune_rows: keep_k %d > n_vis %d", keep_k, n_vis);
    if ((int64_t)vis_begin + n_vis > seq_len)
        return fail(SQAP_EINVAL, "sqap_prune_rows: visual span [%d, %d+%d) outside [0, %d)", vis_begin,
                    vis_begin, n_vis, seq_len);
    if ((int64_t)batch * seq_len > INT32_MAX)
        return fail(SQAP_EINVAL, "sqap_prune_rows: batch * seq_len overflows int32");
    if (n_vis > 65536) return fail(SQAP_EUNSUPPORTED, "sqap_prune_rows: n_vis %d > 65536", n_vis);
    if (batch == 0 || (int64_t)seq_len - n_vis + keep_k == 0) return SQAP_OK;
    if (!rows_out || (keep_k > 0 && (!scores || !idx_out))) return fail(SQAP_EINVAL, "sqap_prune_rows: null pointer");
    if (keep_k == 0 || n_vis == 0)      // nothing to rank: only the non-visual rows survive
        return launch_kept_rows(idx_out, batch, 0, seq_len, vis_begin, n_vis, rows_out, as_stream(stream));
    return launch_prune_rows(scores, batch, n_vis, keep_k, seq_len, vis_begin, idx_out, rows_out,
                             as_stream(stream));
}

sqap_status sqap_prune_select(const float *scores, int32_t batch, int32_t grid_w, int32_t grid_h,
                              int32_t k_attn, int32_t keep_total, const double *camera, int32_t ring_radius,
                              int32_t *idx_out, int32_t cap, int32_t *count_out, void *stream)
{
    if (batch < 0 || grid_w < 1 || grid_h < 1 || k_attn < 0 || keep_total < 0 || ring_radius < 0 || cap < 0)
        return fail(SQAP_EINVAL, "sqap_prune_select: negative size");
    const int64_t n = (int64_t)grid_w * grid_h;
    if (n > 1024) return fail(SQAP_EUNSUPPORTED, "sqap_prune_select: %lld tokens > 1024", (long long)n);
    if (k_attn > n || keep_total > n)
        return fail(SQAP_EINVAL, "sqap_prune_select: k_attn %d or keep_total %d above %lld tokens", k_attn,
                    keep_total, (long long)n);
    // the union K_attn + K_ring is never cut, so the output must be able to hold it
    const int64_t side = 2 * (int64_t)(ring_radius > 1024 ? 1024 : ring_radius) + 1;
    int64_t most = camera ? (int64_t)k_attn + side * side : k_attn;
    if (most > n) most = n;
    if (most < keep_total) most = keep_total;
    if (cap < most)
        return fail(SQAP_EINVAL, "sqap_prune_select: cap %d below the largest possible set %lld", cap, (long long)most);
    if (batch == 0) return SQAP_OK;
    if (!scores || (cap > 0 && !idx_out)) return fail(SQAP_EINVAL, "sqap_prune_select: null pointer");
    return launch_prune_select(scores, batch, grid_w, grid_h, k_attn, keep_total, camera, ring_radius, idx_out,
                               cap, count_out, as_stream(stream));
}

sqap_status sqap_kept_rows(const int32_t *idx, int32_t batch, int32_t keep_k, int32_t seq_len,
                           int32_t vis_begin, int32_t n_vis, int32_t *rows_out, void *stream)
{
    if (batch < 0 || keep_k < 0 || seq_len < 0 || n_vis < 0 || vis_begin < 0)
        return fail(SQAP_EINVAL, "sqap_kept_rows: negative size");
    if (keep_k > n_vis) return fail(SQAP_EINVAL, "sqap_kept_rows: keep_k %d > n_vis %d", keep_k, n_vis);
    if ((int64_t)vis_begin + n_vis > seq_len)
        return fail(SQAP_EINVAL, "sqap_kept_rows: visual span [%d, %d+%d) outside [0, %d)",
                    vis_begin, vis_begin, n_vis, seq_len);
    int64_t per = (int64_t)seq_len - n_vis + keep_k;
    if ((int64_t)batch * seq_len > INT32_MAX)
        return fail(SQAP_EINVAL, "sqap_kept_rows: batch * seq_len overflows int32");
    if (batch == 0 || per == 0) return SQAP_OK;
    if (!rows_out || (keep_k > 0 && !idx)) return fail(SQAP_EINVAL, "sqap_kept_rows: null pointer");
    return launch_kept_rows(idx, batch, keep_k, seq_len, vis_begin, n_vis, rows_out,
                            as_stream(stream));
}

sqap_status sqap_gather_rows(const sqap_f16 *X, int64_t ldx, const int32_t *rows, int32_t M,
                             int32_t K, sqap_f16 *out, int64_t ldo, void *stream)
{
    if (M < 0 || K <= 0) return fail(SQAP_EINVAL, "sqap_gather_rows: M %d, K %d", M, K);
    if (ldx < K || ldo < K) return fail(SQAP_EINVAL, "sqap_gather_rows: pitch below K");
    if (M == 0) return SQAP_OK;
    if (!X || !rows || !out) return fail(SQAP_EINVAL, "sqap_gather_rows: null pointer");
    if ((K & 7) || (ldx & 7) || (ldo & 7) || !aligned16(X) || !aligned16(out))
        return fail(SQAP_EUNSUPPORTED, "sqap_gather_rows: K and pitches must be multiples of 8, "
                                       "pointers 16-byte aligned");
    return launch_gather_rows(reinterpret_cast<const __half *>(X), ldx, rows, M, K,
                              reinterpret_cast<__half *>(out), ldo, as_stream(stream));
}

static sqap_status quantize_common(const char *who, const sqap_f16 *X, int64_t ldx,
                                   const int32_t *rows, int32_t M, int32_t K, uint32_t flags,
                                   uint8_t *Xq, sqap_f16 *sx, void *stream)
{
    if (M < 0 || K <= 0) return fail(SQAP_EINVAL, "%s: M %d, K %d", who, M, K);
    if (K & 1) return fail(SQAP_EINVAL, "%s: K = %d is odd", who, K);
    if (ldx < K) return fail(SQAP_EINVAL, "%s: pitch %lld below K %d", who, (long long)ldx, K);
    if (flags & ~(uint32_t)SQAP_ROTATE_HADAMARD) return fail(SQAP_EINVAL, "%s: unknown flags 0x%x", who, flags);
    if (M == 0) return SQAP_OK;
    if (!X || !Xq || !sx) return fail(SQAP_EINVAL, "%s: null pointer", who);
    bool rotate = (flags & SQAP_ROTATE_HADAMARD) != 0;
    if (rotate && ((K & -K) < 16))
        return fail(SQAP_EUNSUPPORTED, "%s: rotation needs K a multiple of 16 (K = %d)", who, K);
    if ((K & 7) || K > 16384)
        return fail(SQAP_EUNSUPPORTED, "%s: K = %d (multiple of 8, <= 16384)", who, K);
    if ((ldx & 7) || !aligned16(X) || (reinterpret_cast<uintptr_t>(Xq) & 3u))
        return fail(SQAP_EUNSUPPORTED, "%s: X and its pitch must be 16-byte aligned, Xq 4-byte", who);
    return launch_quantize_rows(reinterpret_cast<const __half *>(X), ldx, rows, M, K, rotate, Xq,
                                reinterpret_cast<__half *>(sx), as_stream(stream));
}

sqap_status sqap_quantize_act(const sqap_f16 *X, int64_t ldx, const int32_t *rows, int32_t M,
                              int32_t K, uint32_t flags, uint8_t *Xq, sqap_f16 *sx, void *stream)
{
    return quantize_common("sqap_quantize_act", X, ldx, rows, M, K, flags, Xq, sx, stream);
}

sqap_status sqap_quantize_weight(const sqap_f16 *W, int32_t N, int32_t K, uint32_t flags,
                                 uint8_t *Wq, sqap_f16 *sw, void *stream)
{
    return quantize_common("sqap_quantize_weight", W, K, nullptr, N, K, flags, Wq, sw, stream);
}

// shared checks of the quantizers with an operation fused in front
static sqap_status fused_common(const char *who, const void *X, int64_t ldx, int32_t M, int32_t K, uint32_t flags,
                                const void *col_scales, const void *y_out, const uint8_t *Xq, const void *sx)
{
    if (M < 0 || K <= 0) return fail(SQAP_EINVAL, "%s: M %d, K %d", who, M, K);
    if (ldx < K) return fail(SQAP_EINVAL, "%s: pitch %lld below K %d", who, (long long)ldx, K);
    if (flags & ~(uint32_t)SQAP_ROTATE_HADAMARD) return fail(SQAP_EINVAL, "%s: unknown flags 0x%x", who, flags);
    if (!Xq && !y_out && M > 0) return fail(SQAP_EINVAL, "%s: neither Xq nor a half-precision output asked for", who);
    if (Xq && !sx) return fail(SQAP_EINVAL, "%s: null sx", who);
    if (M > 0 && !X) return fail(SQAP_EINVAL, "%s: null input", who);
    const bool rotate = (flags & SQAP_ROTATE_HADAMARD) != 0;
    if (rotate && ((K & -K) < 16))
        return fail(SQAP_EUNSUPPORTED, "%s: rotation needs K a multiple of 16 (K = %d)", who, K);
    if ((K & 7) || K > 16384) return fail(SQAP_EUNSUPPORTED, "%s: K = %d (multiple of 8, <= 16384)", who, K);
    if ((ldx & 7) || !aligned16(X) || !aligned16(col_scales) || !aligned16(y_out) ||
        (reinterpret_cast<uintptr_t>(Xq) & 3u))
        return fail(SQAP_EUNSUPPORTED, "%s: half operands and pitches must be 16-byte aligned, Xq 4-byte", who);
    return SQAP_OK;
}

sqap_status sqap_rmsnorm_quantize_act(const sqap_f16 *X, int64_t ldx, const int32_t *rows, int32_t M, int32_t K,
                                      const sqap_f16 *delta, const sqap_f16 *gamma, float eps, uint32_t flags,
                                      const sqap_f16 *col_scales, sqap_f16 *xsum_out, sqap_f16 *y_out,
                                      uint8_t *Xq, sqap_f16 *sx, void *stream)
{
    const char *who = "sqap_rmsnorm_quantize_act";
    sqap_status s = fused_common(who, X, ldx, M, K, flags, col_scales, y_out, Xq, sx);
    if (s != SQAP_OK) return s;
    if (!(eps >= 0.0f)) return fail(SQAP_EINVAL, "%s: eps must be >= 0", who);
    if (M == 0) return SQAP_OK;
    if (!gamma) return fail(SQAP_EINVAL, "%s: null gamma", who);
    if (!aligned16(gamma) || !aligned16(delta) || !aligned16(xsum_out))
        return fail(SQAP_EUNSUPPORTED, "%s: gamma, delta and xsum_out must be 16-byte aligned", who);
    PreArgs pre = {};
    pre.delta = reinterpret_cast<const __half *>(delta);
    pre.xsum_out = reinterpret_cast<__half *>(xsum_out);
    pre.gamma = reinterpret_cast<const __half *>(gamma);
    pre.eps = eps;
    pre.y_out = reinterpret_cast<__half *>(y_out);
    return launch_fused_quantize(kPreNorm, reinterpret_cast<const __half *>(X), ldx, rows, M, K,
                                 (flags & SQAP_ROTATE_HADAMARD) != 0, reinterpret_cast<const __half *>(col_scales),
                                 Xq, reinterpret_cast<__half *>(sx), pre, as_stream(stream));
}

sqap_status sqap_swiglu_quantize_act(const sqap_f16 *G, int64_t ldg, const sqap_f16 *U, int64_t ldu, int32_t M,
                                     int32_t F, const sqap_f16 *col_scales, sqap_f16 *h_out, uint8_t *Xq,
                                     sqap_f16 *sx, void *stream)
{
    const char *who = "sqap_swiglu_quantize_act";
    sqap_status s = fused_common(who, G, ldg, M, F, 0, col_scales, h_out, Xq, sx);
    if (s != SQAP_OK) return s;
    if (ldu < F) return fail(SQAP_EINVAL, "%s: pitch %lld below F %d", who, (long long)ldu, F);
    if (M == 0) return SQAP_OK;
    if (!U) return fail(SQAP_EINVAL, "%s: null U", who);
    if ((ldu & 7) || !aligned16(U)) return fail(SQAP_EUNSUPPORTED, "%s: U and its pitch must be 16-byte aligned", who);
    PreArgs pre = {};
    pre.U = reinterpret_cast<const __half *>(U);
    pre.ldu = ldu;
    pre.y_out = reinterpret_cast<__half *>(h_out);
    return launch_fused_quantize(kPreSwiglu, reinterpret_cast<const __half *>(G), ldg, nullptr, M, F, false,
                                 reinterpret_cast<const __half *>(col_scales), Xq, reinterpret_cast<__half *>(sx), pre,
                                 as_stream(stream));
}

sqap_status sqap_rope(sqap_f16 *X, int64_t ld, const int32_t *pos, int32_t S, int32_t H, int32_t d, double base,
                      void *stream)
{
    if (S < 0 || H <= 0 || d <= 0 || (d & 1)) return fail(SQAP_EINVAL, "sqap_rope: S %d, H %d, d %d", S, H, d);
    if (ld < (int64_t)H * d) return fail(SQAP_EINVAL, "sqap_rope: pitch %lld below H * d", (long long)ld);
    if (!(base > 0.0)) return fail(SQAP_EINVAL, "sqap_rope: base must be positive");
    if (S == 0) return SQAP_OK;
    if (!X || !pos) return fail(SQAP_EINVAL, "sqap_rope: null pointer");
    return launch_rope(reinterpret_cast<__half *>(X), ld, pos, S, H, d, base, as_stream(stream));
}

sqap_status sqap_rope_append(sqap_f16 *QKV, int64_t ld, const int32_t *pos, int32_t S, int32_t H, int32_t d,
                             double base, sqap_f16 *KV, int64_t ldkv, void *stream)
{
    if (S < 0 || H <= 0 || d <= 0 || (d & 1)) return fail(SQAP_EINVAL, "sqap_rope_append: S %d, H %d, d %d", S, H, d);
    if (ld < (int64_t)3 * H * d || ldkv < (int64_t)2 * H * d)
        return fail(SQAP_EINVAL, "sqap_rope_append: pitch below 3 H d (q|k|v) or 2 H d (cache)");
    if (!(base > 0.0)) return fail(SQAP_EINVAL, "sqap_rope_append: base must be positive");
    if (S == 0) return SQAP_OK;
    if (!QKV || !pos || !KV) return fail(SQAP_EINVAL, "sqap_rope_append: null pointer");
    return launch_rope_append(reinterpret_cast<__half *>(QKV), ld, pos, S, H, d, base, reinterpret_cast<__half *>(KV),
                              ldkv, as_stream(stream));
}

sqap_status sqap_attention(const sqap_f16 *Q, int64_t ldq, const sqap_f16 *K, int64_t ldk, const sqap_f16 *V,
                           int64_t ldv, int32_t batch, int32_t Sq, int32_t Sk, int32_t H, int32_t d, sqap_f16 *O,
                           int64_t ldo, void *stream)
{
    if (batch < 0 || Sq < 0 || Sk < Sq || H <= 0 || d <= 0)
        return fail(SQAP_EINVAL, "sqap_attention: batch %d, Sq %d, Sk %d (>= Sq), H %d, d %d", batch, Sq, Sk, H, d);
    const int64_t width = (int64_t)H * d;
    if (ldq < width || ldk < width || ldv < width || ldo < width)
        return fail(SQAP_EINVAL, "sqap_attention: a pitch is below H * d");
    if (d != 16 && d != 32 && d != 64 && d != 128)
        return fail(SQAP_EUNSUPPORTED, "sqap_attention: head size %d (16, 32, 64 or 128)", d);
    if (batch > 65535) return fail(SQAP_EUNSUPPORTED, "sqap_attention: batch = %d", batch);
    if (Sq == 0 || batch == 0) return SQAP_OK;
    if (!Q || !K || !V || !O) return fail(SQAP_EINVAL, "sqap_attention: null pointer");
    if (((ldq | ldk | ldv | ldo) & 7) || !aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O))
        return fail(SQAP_EUNSUPPORTED, "sqap_attention: operands and pitches must be 16-byte aligned");
    return launch_attention(reinterpret_cast<const __half *>(Q), ldq, reinterpret_cast<const __half *>(K), ldk,
                            reinterpret_cast<const __half *>(V), ldv, batch, Sq, Sk, H, d, reinterpret_cast<__half *>(O), ldo,
                            as_stream(stream));
}

sqap_status sqap_decode_attention(const sqap_f16 *QKV, const int32_t *pos, int32_t H, int32_t d, double base,
                                  sqap_f16 *KV, int64_t ldkv, int32_t past, sqap_f16 *O, uint8_t *Xq, sqap_f16 *sx,
                                  uint32_t *counter, void *stream)
{
    if (H <= 0 || d <= 0 || past < 0) return fail(SQAP_EINVAL, "sqap_decode_attention: H %d, d %d, past %d", H, d, past);
    if (ldkv < (int64_t)2 * H * d) return fail(SQAP_EINVAL, "sqap_decode_attention: cache pitch below 2 H d");
    if (!(base > 0.0)) return fail(SQAP_EINVAL, "sqap_decode_attention: base must be positive");
    if (!QKV || !pos || !KV || !O) return fail(SQAP_EINVAL, "sqap_decode_attention: null pointer");
    if (Xq && (!sx || !counter)) return fail(SQAP_EINVAL, "sqap_decode_attention: Xq needs sx and counter");
    if ((d & 7) || d > 128) return fail(SQAP_EUNSUPPORTED, "sqap_decode_attention: head size %d (multiple of 8, <= 128)", d);
    if ((ldkv & 7) || !aligned16(KV) || !aligned16(O))
        return fail(SQAP_EUNSUPPORTED, "sqap_decode_attention: cache, its pitch and the output must be 16-byte aligned");
    if (Xq && (int64_t)H * d > 8192)
        return fail(SQAP_EUNSUPPORTED, "sqap_decode_attention: H * d = %lld above 8192 with the quantizer folded in",
                    (long long)H * d);
    if (Xq && ((reinterpret_cast<uintptr_t>(Xq) | reinterpret_cast<uintptr_t>(counter)) & 3u))
        return fail(SQAP_EUNSUPPORTED, "sqap_decode_attention: Xq and counter must be 4-byte aligned");
    return launch_decode_attention(reinterpret_cast<const __half *>(QKV), pos, H, d, base, reinterpret_cast<__half *>(KV),
                                   ldkv, past, reinterpret_cast<__half *>(O), Xq, reinterpret_cast<__half *>(sx), counter,
                                   as_stream(stream));
}

sqap_status sqap_residual_add(sqap_f16 *X, int64_t ldx, const sqap_f16 *delta, int64_t ldd, int32_t M, int32_t K,
                              void *stream)
{
    if (M < 0 || K < 0) return fail(SQAP_EINVAL, "sqap_residual_add: M %d, K %d", M, K);
    if (ldx < K || ldd < K) return fail(SQAP_EINVAL, "sqap_residual_add: pitch below K");
    if (M == 0 || K == 0) return SQAP_OK;
    if (!X || !delta) return fail(SQAP_EINVAL, "sqap_residual_add: null pointer");
    if ((K & 7) || (ldx & 7) || (ldd & 7) || !aligned16(X) || !aligned16(delta))
        return fail(SQAP_EUNSUPPORTED, "sqap_residual_add: K and pitches multiples of 8, pointers 16-byte aligned");
    return launch_residual_add(reinterpret_cast<__half *>(X), ldx, reinterpret_cast<const __half *>(delta), ldd, M, K,
                               as_stream(stream));
}

// shared checks of the entry points that take per-channel scales
static sqap_status scaled_common(const char *who, const sqap_f16 *X, int64_t ldx, int32_t M, int32_t K,
                                 uint32_t flags, const void *col_scales)
{
    if (M < 0 || K <= 0) return fail(SQAP_EINVAL, "%s: M %d, K %d", who, M, K);
    if (K & 1) return fail(SQAP_EINVAL, "%s: K = %d is odd", who, K);
    if (ldx < K) return fail(SQAP_EINVAL, "%s: pitch %lld below K %d", who, (long long)ldx, K);
    if (flags & ~(uint32_t)SQAP_ROTATE_HADAMARD) return fail(SQAP_EINVAL, "%s: unknown flags 0x%x", who, flags);
    if ((flags & SQAP_ROTATE_HADAMARD) && ((K & -K) < 16))
        return fail(SQAP_EUNSUPPORTED, "%s: rotation needs K a multiple of 16 (K = %d)", who, K);
    if ((K & 7) || K > 16384) return fail(SQAP_EUNSUPPORTED, "%s: K = %d (multiple of 8, <= 16384)", who, K);
    if (M > 0 && (!X || !col_scales)) return fail(SQAP_EINVAL, "%s: null pointer", who);
    if (M > 0 && ((ldx & 7) || !aligned16(X) || !aligned16(col_scales)))
        return fail(SQAP_EUNSUPPORTED, "%s: X, its pitch and the channel scales must be 16-byte aligned", who);
    return SQAP_OK;
}

sqap_status sqap_channel_scales(const sqap_f16 *X, int64_t ldx, const int32_t *rows, int32_t M, int32_t K,
                                uint32_t flags, float *amax, int32_t accumulate, sqap_f16 *scales_out,
                                void *stream)
{
    if (!amax || !scales_out) return fail(SQAP_EINVAL, "sqap_channel_scales: null pointer");
    sqap_status st = scaled_common("sqap_channel_scales", X, ldx, M, K, flags, scales_out);
    if (st != SQAP_OK) return st;
    return launch_channel_scales(reinterpret_cast<const __half *>(X), ldx, rows, M, K,
                                 (flags & SQAP_ROTATE_HADAMARD) != 0, amax, accumulate != 0,
                                 reinterpret_cast<__half *>(scales_out), as_stream(stream));
}

sqap_status sqap_quantize_act_channelwise(const sqap_f16 *X, int64_t ldx, const int32_t *rows, int32_t M,
                                          int32_t K, uint32_t flags, const sqap_f16 *col_scales, uint8_t *Xq,
                                          sqap_f16 *sx, void *stream)
{
    sqap_status st = scaled_common("sqap_quantize_act_channelwise", X, ldx, M, K, flags, col_scales);
    if (st != SQAP_OK) return st;
    if (M == 0) return SQAP_OK;
    if (!Xq || !sx) return fail(SQAP_EINVAL, "sqap_quantize_act_channelwise: null pointer");
    if (reinterpret_cast<uintptr_t>(Xq) & 3u)
        return fail(SQAP_EUNSUPPORTED, "sqap_quantize_act_channelwise: Xq must be 4-byte aligned");
    return launch_quantize_rows_scaled(reinterpret_cast<const __half *>(X), ldx, rows, M, K,
                                       (flags & SQAP_ROTATE_HADAMARD) != 0, false,
                                       reinterpret_cast<const __half *>(col_scales), Xq,
                                       reinterpret_cast<__half *>(sx), as_stream(stream));
}

sqap_status sqap_quantize_weight_folded(const sqap_f16 *W, int32_t N, int32_t K, uint32_t flags,
                                        const sqap_f16 *col_scales, uint8_t *Wq, sqap_f16 *sw, void *stream)
{
    sqap_status st = scaled_common("sqap_quantize_weight_folded", W, K, N, K, flags, col_scales);
    if (st != SQAP_OK) return st;
    if (N == 0) return SQAP_OK;
    if (!Wq || !sw) return fail(SQAP_EINVAL, "sqap_quantize_weight_folded: null pointer");
    if (reinterpret_cast<uintptr_t>(Wq) & 3u)
        return fail(SQAP_EUNSUPPORTED, "sqap_quantize_weight_folded: Wq must be 4-byte aligned");
    return launch_quantize_rows_scaled(reinterpret_cast<const __half *>(W), K, nullptr, N, K,
                                       (flags & SQAP_ROTATE_HADAMARD) != 0, true,
                                       reinterpret_cast<const __half *>(col_scales), Wq,
                                       reinterpret_cast<__half *>(sw), as_stream(stream));
}

sqap_status sqap_weight_pack(const uint8_t *Wq, const sqap_f16 *sw, int32_t N, int32_t K,
                             sqap_weight **out, void *stream)
{
    if (out) *out = nullptr;
    if (N <= 0 || K <= 0) return fail(SQAP_EINVAL, "sqap_weight_pack: N %d, K %d", N, K);
    if (!Wq || !sw || !out) return fail(SQAP_EINVAL, "sqap_weight_pack: null pointer");
    if (K % 32 != 0) return fail(SQAP_EUNSUPPORTED, "sqap_weight_pack: K = %d is not a multiple of 32", K);
    if (!aligned16(Wq)) return fail(SQAP_EUNSUPPORTED, "sqap_weight_pack: Wq must be 16-byte aligned");
    Weight *w = new (std::nothrow) Weight();
    if (!w) return fail(SQAP_ENOMEM, "sqap_weight_pack: host allocation failed");
    w->magic = kWeightMagic;
    w->N = N;
    w->K = K;
    w->n_groups = ((N + 255) / 256) * 8;
    w->chunks = K / 32;
    size_t data_bytes = (size_t)w->n_groups * w->chunks * 512;
    size_t scale_bytes = (size_t)w->n_groups * 32 * sizeof(__half);
    w->bytes = data_bytes + scale_bytes;
    w->data = nullptr;
    w->scales = nullptr;
    hipError_t e = hipGetDevice(&w->device);
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&w->data), data_bytes);
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&w->scales), scale_bytes);
    if (e != hipSuccess) {
        if (w->data) (void)hipFree(w->data);
        delete w;
        return fail(e == hipErrorOutOfMemory ? SQAP_ENOMEM : SQAP_EDEVICE, "sqap_weight_pack: %s",
                    hipGetErrorString(e));
    }
    sqap_status st = launch_weight_pack(Wq, reinterpret_cast<const __half *>(sw), *w, as_stream(stream));
    if (st != SQAP_OK) {
        (void)hipFree(w->data);
        (void)hipFree(w->scales);
        delete w;
        return st;
    }
    // first weight on this device: find out whether the persistent GEMM kernels may be used on it
    st = probe_dispatch(w->device, as_stream(stream), nullptr);
    if (st != SQAP_OK) {
        (void)hipFree(w->data);
        (void)hipFree(w->scales);
        delete w;
        return st;
    }
    *out = reinterpret_cast<sqap_weight *>(w);
    return SQAP_OK;
}

sqap_status sqap_weight_free(sqap_weight *w)
{
    if (!w) return SQAP_OK;
    Weight *ww = reinterpret_cast<Weight *>(w);
    if (ww->magic != kWeightMagic) return fail(SQAP_EINVAL, "sqap_weight_free: not a weight handle");
    ww->magic = 0;
    hipError_t e1 = hipFree(ww->data);
    hipError_t e2 = hipFree(ww->scales);
    delete ww;
    if (e1 != hipSuccess) return fail(SQAP_EDEVICE, "sqap_weight_free: %s", hipGetErrorString(e1));
    if (e2 != hipSuccess) return fail(SQAP_EDEVICE, "sqap_weight_free: %s", hipGetErrorString(e2));
    return SQAP_OK;
}

sqap_status sqap_weight_info(const sqap_weight *w, int32_t *N, int32_t *K, size_t *device_bytes)
{
    const Weight *ww = check_weight(w);
    if (!ww) return fail(SQAP_EINVAL, "sqap_weight_info: not a weight handle");
    if (N) *N = ww->N;
    if (K) *K = ww->K;
    if (device_bytes) *device_bytes = ww->bytes;
    return SQAP_OK;
}

sqap_status sqap_init(void *stream)
{
    int dev = 0;
    SQAP_HIP_CHECK(hipGetDevice(&dev));
    void *scratch_ptr = nullptr;               // device address of the built-in scratch array, looked up once per device
    sqap_status s = noalloc_scratch(&scratch_ptr);
    if (s != SQAP_OK) return s;
    return probe_dispatch(dev, as_stream(stream), nullptr);
}

sqap_status sqap_set_persistent_kernels(int32_t enabled)
{
    set_persistent_kernels(enabled);
    return SQAP_OK;
}

sqap_status sqap_set_mid_m_kernel(int32_t which)
{
    set_mid_m_kernel(which);
    return SQAP_OK;
}

sqap_status sqap_selftest_dispatch(uint32_t *xcc_of_block_out, void *stream)
{
    if (!xcc_of_block_out) return fail(SQAP_EINVAL, "sqap_selftest_dispatch: null pointer");
    int dev = 0;
    SQAP_HIP_CHECK(hipGetDevice(&dev));
    return probe_dispatch(dev, as_stream(stream), xcc_of_block_out);
}

sqap_status sqap_plan_linear_shares(int32_t M, int32_t N, int32_t K, int32_t blocks_per_xcd, uint32_t *bounds_out,
                                    double *planned_steps_out, double *even_steps_out, int32_t *tile_rows_out,
                                    int32_t *tile_cols_out)
{
    if (!bounds_out || !planned_steps_out || !even_steps_out || !tile_rows_out || !tile_cols_out)
        return fail(SQAP_EINVAL, "sqap_plan_linear_shares: null pointer");
    if (M <= 0 || N <= 0 || K <= 0) return fail(SQAP_EINVAL, "sqap_plan_linear_shares: M, N, K must be positive");
    return plan_linear_shares(M, N, K, blocks_per_xcd, bounds_out, planned_steps_out, even_steps_out, tile_rows_out,
                              tile_cols_out);
}

sqap_status sqap_selftest_quotient(uint64_t *mismatches_out, void *stream)
{
    if (!mismatches_out) return fail(SQAP_EINVAL, "sqap_selftest_quotient: null pointer");
    return launch_quotient_selftest(reinterpret_cast<unsigned long long *>(mismatches_out), as_stream(stream));
}

size_t sqap_workspace_bytes(int32_t M, int32_t N, int32_t K)
{
    if (M <= 0 || N <= 0 || K <= 0) return 0;
    return linear_workspace_bytes(M, N, K);
}

sqap_status sqap_w4a4_linear(const uint8_t *Xq, const sqap_f16 *sx, int32_t M,
                             const sqap_weight *W, sqap_f16 *Y, int64_t ldy, int32_t *acc_out,
                             void *workspace, size_t workspace_bytes, void *stream)
{
    const Weight *w = check_weight(W);
    if (!w) return fail(SQAP_EINVAL, "sqap_w4a4_linear: W is not a weight handle");
    if (M < 0) return fail(SQAP_EINVAL, "sqap_w4a4_linear: M = %d", M);
    if (ldy < w->N) return fail(SQAP_EINVAL, "sqap_w4a4_linear: ldy %lld below N %d", (long long)ldy, w->N);
    if (M == 0) return SQAP_OK;
    if (!Xq || !sx || !Y) return fail(SQAP_EINVAL, "sqap_w4a4_linear: null pointer");
    if (!aligned16(Xq)) return fail(SQAP_EUNSUPPORTED, "sqap_w4a4_linear: Xq must be 16-byte aligned");
    size_t need = linear_workspace_bytes(M, w->N, w->K);
    if (need > 0) {
        if (!workspace || workspace_bytes < need)
            return fail(SQAP_EINVAL, "sqap_w4a4_linear: workspace of %zu bytes needed, %zu given", need,
                        workspace ? workspace_bytes : (size_t)0);
        if (reinterpret_cast<uintptr_t>(workspace) & 255u)
            return fail(SQAP_EINVAL, "sqap_w4a4_linear: workspace must be 256-byte aligned");
    }
    if (M <= kSkinnyMaxM && w->K % 64 == 0) {
        SkinnyArgs a = {};
        a.table = nullptr;
        a.count = 1;
        a.total_items = (w->N + 31) / 32;
        SkinnyEntry &e = a.inline_entries[0];
        e.Xq = Xq;
        e.sx = reinterpret_cast<const __half *>(sx);
        e.Wd = w->data;
        e.sw = w->scales;
        e.Y = reinterpret_cast<__half *>(Y);
        e.acc_out = acc_out;
        e.ldy = ldy;
        e.M = M;
        e.N = w->N;
        e.chunks = w->chunks;
        e.rg_begin = 0;
        e.cost_begin = 0;
        a.total_cost = (long long)a.total_items * w->chunks;
        return launch_skinny(a, w->chunks, as_stream(stream));
    }
    return launch_w4a4_linear(Xq, reinterpret_cast<const __half *>(sx), M, *w,
                              reinterpret_cast<__half *>(Y), ldy, acc_out, workspace,
                              as_stream(stream));
}

sqap_status sqap_decoder_create(const sqap_decoder_layer *layers, int32_t n_layers, int32_t n_heads, int32_t head_dim,
                                const sqap_f16 *gamma_final, const sqap_weight *head, float eps, double rope_base,
                                sqap_decoder **out)
{
    if (out) *out = nullptr;
    if (!layers || !out) return fail(SQAP_EINVAL, "sqap_decoder_create: null pointer");
    if (!(eps >= 0.0f) || !(rope_base > 0.0)) return fail(SQAP_EINVAL, "sqap_decoder_create: eps must be >= 0, rope_base > 0");
    Decoder *d = nullptr;
    sqap_status s = decoder_create(layers, n_layers, n_heads, head_dim, gamma_final, head, eps, rope_base, &d);
    if (s == SQAP_OK) *out = reinterpret_cast<sqap_decoder *>(d);
    return s;
}

sqap_status sqap_decoder_step(sqap_decoder *d, const sqap_f16 *x, const int32_t *pos, int32_t past, sqap_f16 *logits,
                              sqap_f16 *attn_trace, void *stream)
{
    Decoder *dd = reinterpret_cast<Decoder *>(d);
    if (!decoder_valid(dd)) return fail(SQAP_EINVAL, "sqap_decoder_step: not a decoder handle");
    if (!x || !pos || !logits) return fail(SQAP_EINVAL, "sqap_decoder_step: null pointer");
    if (past < 0) return fail(SQAP_EINVAL, "sqap_decoder_step: past = %d", past);
    if ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(logits) | reinterpret_cast<uintptr_t>(attn_trace)) & 15u)
        return fail(SQAP_EUNSUPPORTED, "sqap_decoder_step: x, logits and attn_trace must be 16-byte aligned");
    return decoder_step(dd, x, pos, past, logits, attn_trace, as_stream(stream));
}

sqap_status sqap_decoder_status(const sqap_decoder *d, uint64_t *error_word_out, void *stream)
{
    const Decoder *dd = reinterpret_cast<const Decoder *>(d);
    if (!decoder_valid(dd)) return fail(SQAP_EINVAL, "sqap_decoder_status: not a decoder handle");
    if (!error_word_out) return fail(SQAP_EINVAL, "sqap_decoder_status: null pointer");
    unsigned long long w = 0;
    sqap_status s = decoder_error(dd, &w, as_stream(stream));
    *error_word_out = w;
    return s;
}

sqap_status sqap_decoder_set_wait_limit(sqap_decoder *d, int64_t polls)
{
    Decoder *dd = reinterpret_cast<Decoder *>(d);
    if (!decoder_valid(dd)) return fail(SQAP_EINVAL, "sqap_decoder_set_wait_limit: not a decoder handle");
    decoder_set_wait_limit(dd, (long long)polls);
    return SQAP_OK;
}

sqap_status sqap_decoder_free(sqap_decoder *d)
{
    if (!d) return SQAP_OK;
    Decoder *dd = reinterpret_cast<Decoder *>(d);
    if (!decoder_valid(dd)) return fail(SQAP_EINVAL, "sqap_decoder_free: not a decoder handle");
    return decoder_free(dd);
}

sqap_status sqap_group_create(const sqap_linear_desc *descs, int32_t count, sqap_group **out)
{
    if (out) *out = nullptr;
    if (!descs || !out) return fail(SQAP_EINVAL, "sqap_group_create: null pointer");
    if (count <= 0) return fail(SQAP_EINVAL, "sqap_group_create: count = %d", count);
    SkinnyEntry *host = new (std::nothrow) SkinnyEntry[count];
    if (!host) return fail(SQAP_ENOMEM, "sqap_group_create: host allocation failed");
    int total = 0, max_chunks = 0;
    long long cost = 0;
    for (int i = 0; i < count; ++i) {
        const sqap_linear_desc &d = descs[i];
        const Weight *w = check_weight(d.W);
        sqap_status st = SQAP_OK;
        if (!w) st = fail(SQAP_EINVAL, "sqap_group_create: problem %d: W is not a weight handle", i);
        else if (!d.Xq || !d.sx || !d.Y) st = fail(SQAP_EINVAL, "sqap_group_create: problem %d: null pointer", i);
        else if (d.M < 1) st = fail(SQAP_EINVAL, "sqap_group_create: problem %d: M = %d", i, d.M);
        else if (d.ldy < w->N) st = fail(SQAP_EINVAL, "sqap_group_create: problem %d: ldy below N", i);
        else if (d.M > kSkinnyMaxM) st = fail(SQAP_EUNSUPPORTED, "sqap_group_create: problem %d: M = %d > %d", i, d.M, kSkinnyMaxM);
        else if (w->K % 64 != 0) st = fail(SQAP_EUNSUPPORTED, "sqap_group_create: problem %d: K = %d is not a multiple of 64", i, w->K);
        else if (!aligned16(d.Xq)) st = fail(SQAP_EUNSUPPORTED, "sqap_group_create: problem %d: Xq must be 16-byte aligned", i);
        if (st != SQAP_OK) {
            delete[] host;
            return st;
        }
        SkinnyEntry &e = host[i];
        e.Xq = d.Xq;
        e.sx = reinterpret_cast<const __half *>(d.sx);
        e.Wd = w->data;
        e.sw = w->scales;
        e.Y = reinterpret_cast<__half *>(d.Y);
        e.acc_out = d.acc_out;
        e.ldy = d.ldy;
        e.M = d.M;
        e.N = w->N;
        e.chunks = w->chunks;
        e.rg_begin = total;
        e.cost_begin = cost;
        total += (w->N + 31) / 32;
        cost += (long long)((w->N + 31) / 32) * w->chunks;
        if (w->chunks > max_chunks) max_chunks = w->chunks;
    }
    Group *g = new (std::nothrow) Group();
    if (!g) {
        delete[] host;
        return fail(SQAP_ENOMEM, "sqap_group_create: host allocation failed");
    }
    g->magic = kGroupMagic;
    g->count = count;
    g->total_items = total;
    g->max_chunks = max_chunks;
    g->total_cost = cost;
    g->table = nullptr;
    hipError_t e = hipGetDevice(&g->device);
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&g->table), sizeof(SkinnyEntry) * count);
    if (e == hipSuccess) e = hipMemcpy(g->table, host, sizeof(SkinnyEntry) * count, hipMemcpyHostToDevice);
    delete[] host;
    if (e != hipSuccess) {
        if (g->table) (void)hipFree(g->table);
        delete g;
        return fail(e == hipErrorOutOfMemory ? SQAP_ENOMEM : SQAP_EDEVICE, "sqap_group_create: %s",
                    hipGetErrorString(e));
    }
    *out = reinterpret_cast<sqap_group *>(g);
    return SQAP_OK;
}

sqap_status sqap_group_run(const sqap_group *g, void *stream)
{
    const Group *gg = reinterpret_cast<const Group *>(g);
    if (!gg || gg->magic != kGroupMagic) return fail(SQAP_EINVAL, "sqap_group_run: not a group handle");
    SkinnyArgs a = {};
    a.table = gg->table;
    a.count = gg->count;
    a.total_items = gg->total_items;
    a.total_cost = gg->total_cost;
    return launch_skinny(a, gg->max_chunks, as_stream(stream));
}

sqap_status sqap_group_info(const sqap_group *g, int32_t compute_units, int32_t *problems_out, int32_t *row_groups_out,
                            int32_t *wavefronts_per_row_group_out, int32_t *wavefronts_per_workgroup_out,
                            int32_t *output_slots_out)
{
    const Group *gg = reinterpret_cast<const Group *>(g);
    if (!gg || gg->magic != kGroupMagic) return fail(SQAP_EINVAL, "sqap_group_info: not a group handle");
    if (compute_units < 0) return fail(SQAP_EINVAL, "sqap_group_info: compute_units = %d", compute_units);
    int S, W, cap;
    skinny_plan(gg->total_items, gg->max_chunks, compute_units > 0 ? compute_units : device_cu_count(), &S, &W, &cap);
    if (problems_out) *problems_out = gg->count;
    if (row_groups_out) *row_groups_out = gg->total_items;
    if (wavefronts_per_row_group_out) *wavefronts_per_row_group_out = S;
    if (wavefronts_per_workgroup_out) *wavefronts_per_workgroup_out = W;
    if (output_slots_out) *output_slots_out = cap;
    return SQAP_OK;
}

sqap_status sqap_group_free(sqap_group *g)
{
    if (!g) return SQAP_OK;
    Group *gg = reinterpret_cast<Group *>(g);
    if (gg->magic != kGroupMagic) return fail(SQAP_EINVAL, "sqap_group_free: not a group handle");
    gg->magic = 0;
    hipError_t e = hipFree(gg->table);
    delete gg;
    if (e != hipSuccess) return fail(SQAP_EDEVICE, "sqap_group_free: %s", hipGetErrorString(e));
    return SQAP_OK;
}

}  // extern "C"
