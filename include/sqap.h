/*
 * sqap.h: C ABI of the MI355X (gfx950) library for the hot path of SQAP-VLA
 * (arXiv 2509.09090): W4A4 linear layers run over the tokens that survive the
 * paper's pruning criterion.
 *
 *   prune_topk -> kept_rows -> (gather) -> quantize_act -> w4a4_linear
 *
 * Conventions that hold for every call unless stated otherwise
 *   - Data pointers are DEVICE pointers owned by the caller.  The library
 *     never frees or keeps them.  The only library-owned objects are
 *     sqap_weight and sqap_group handles.
 *   - Half precision crosses the ABI as IEEE binary16 bit patterns (sqap_f16).
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).
 *     Calls enqueue work on it and return; they never synchronise the host.
 *   - Arguments are validated on the host before any device work.  A failed
 *     validation returns a negative status, enqueues nothing, and leaves a
 *     message for sqap_last_error().
 *   - Sizes of zero (M = 0, keep_k = 0, batch = 0) are legal and do nothing.
 *   - Packed int4 ("canonical") layout: row-major, K/2 bytes per row; byte j
 *     holds element 2j in bits 0-3 and element 2j+1 in bits 4-7, each a 4-bit
 *     two's-complement code in [-8, 7].
 *   - No C++ exception crosses this boundary.
 */
#ifndef SQAP_H
#define SQAP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t sqap_status;
typedef uint16_t sqap_f16; /* IEEE binary16 bit pattern */

enum {
    SQAP_OK = 0,
    SQAP_EINVAL = -1,       /* null pointer, negative size, odd K, keep_k > n, ld < K ... */
    SQAP_EUNSUPPORTED = -2, /* legal request outside what the kernels cover */
    SQAP_EDEVICE = -3,      /* a HIP call failed; message holds hipGetErrorString */
    SQAP_ENOMEM = -4
};

/* flags */
enum {
    SQAP_ROTATE_HADAMARD = 1u /* rotate each row by the orthonormal Hadamard matrix first */
};

/* Opaque packed weight: device-resident, library-private layout. */
typedef struct sqap_weight sqap_weight;

/* Message of the last failed call on this thread (static storage, never NULL). */
const char *sqap_last_error(void);

/* Library version string (static storage). */
const char *sqap_version(void);

/*
 * One-time set-up of the current device: finds out how the hardware deals the
 * workgroups of a launch to the XCDs, which decides whether sqap_w4a4_linear
 * may use its persistent kernels there (see sqap_selftest_dispatch).  This is
 * the one call of the library that SYNCHRONISES the stream (a probe launch
 * and a read-back of 1 KiB); later calls on the same device return at once.
 * A device that has not been set up is set up by the first sqap_weight_pack
 * on it, which then synchronises its stream once in the same way; when that
 * stream is being captured into a graph the set-up is put off and
 * sqap_w4a4_linear uses its slower one-tile-per-workgroup kernels on the
 * device until a later sqap_init or sqap_weight_pack has probed it.
 * EDEVICE: a HIP call failed.
 */
sqap_status sqap_init(void *stream);

/*
 * Retention score a_q (Strategy 1, text under Eq. 1; Section 3.3 defines the
 * Q and K it is computed from).  For a task-query token with per-head query
 * q[H,d] and the key cache k[S,H,d] (both half, row-major), computes for each
 * head the softmax over all S keys of (q.k)/sqrt(d) and writes the mean over
 * heads of the weights of the visual span:
 *   scores_out[j] = (1/H) sum_h softmax_s(l[h,:])[vis_begin + j],  j < n_vis.
 * Arithmetic in binary32.  scores_out: n_vis floats.  All pointers are device
 * pointers owned by the caller.  The heads are added in head order, so the
 * result is the same bits on every call.
 * workspace: device scratch of at least sqap_attn_scores_workspace_bytes(1, S, H,
 * d, n_vis) bytes, 16-byte aligned (may be NULL when that is 0): one workgroup
 * per head leaves the head's weights there and the workgroup that finishes last,
 * told by a counter at the start of the workspace, adds them.  The first
 * 256 * batch bytes (the counters) must be ZERO before the first call that uses
 * a workspace; every call leaves them zero, so clearing once is enough.  The
 * rest needs no initialisation.  Calls that share a workspace must be ordered
 * on one stream; calls on different streams need a workspace each.
 * EINVAL: null pointer, S/H/d <= 0, span outside [0,S), workspace missing, too
 * small or misaligned.  EUNSUPPORTED: d > 256, d odd or S > 16384.
 */
sqap_status sqap_attn_scores(const sqap_f16 *q, const sqap_f16 *k, int32_t S, int32_t H,
                             int32_t d, int32_t vis_begin, int32_t n_vis, float *scores_out,
                             void *workspace, size_t workspace_bytes, void *stream);

/*
 * The same score for `batch` observations in one launch: q[batch,H,d],
 * k[batch,S,H,d], scores_out[batch,n_vis] (row-major, dense); observation b
 * gets exactly what sqap_attn_scores gives for q[b], k[b].  batch = 0 is a
 * no-op.  workspace: sqap_attn_scores_workspace_bytes(batch, ...) bytes, as above.
 * Errors as above; EINVAL for batch < 0, EUNSUPPORTED for batch > 4096.
 */
sqap_status sqap_attn_scores_batch(const sqap_f16 *q, const sqap_f16 *k, int32_t batch, int32_t S,
                                   int32_t H, int32_t d, int32_t vis_begin, int32_t n_vis,
                                   float *scores_out, void *workspace, size_t workspace_bytes,
                                   void *stream);

/*
 * Bytes of workspace the two calls above need for this shape: 256 per observation
 * for the counters plus 4 * batch * H * n_vis for the per-head weights; 0 for
 * shapes that run in a single workgroup and need none (head size not a power of
 * two in 8 .. 256, or S > 4096) and for empty shapes.
 */
size_t sqap_attn_scores_workspace_bytes(int32_t batch, int32_t S, int32_t H, int32_t d, int32_t n_vis);

/*
 * sqap_attn_scores_batch for callers that cannot allocate device memory or pass
 * a workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments without the workspace, same kernels, same
 * bits in scores_out.  The scratch memory is an array built into the library,
 * 2 MiB + 16 KiB of device memory that every GPU the library runs on holds
 * until the process ends; it serves at most 64 observations per call and
 * batch * H * n_vis <= 524288 per-head weights (16 observations of 32 heads x
 * 256 visual tokens use a quarter of it).  The call itself allocates and frees
 * nothing, on the host or on the device; the array's device address is looked
 * up at sqap_init, or else at the first call on a device.  All calls on one GPU
 * share the array: calls that overlap in time there (two streams, two host
 * threads) race, calls ordered on one stream do not.  What must be zero at the
 * start of a call is zero when the library is loaded and is put back to zero by
 * the kernel before it ends, so a call that runs to its end leaves the array
 * ready for the next one whatever that one's size.  Shapes that run in a single
 * workgroup (see sqap_attn_scores_workspace_bytes) use no scratch memory at all.
 * EINVAL / EUNSUPPORTED as sqap_attn_scores_batch; EUNSUPPORTED also for
 * batch > 64 or batch * H * n_vis > 524288 (the message says which).
 */
sqap_status sqap_attn_scores_noalloc(const sqap_f16 *q, const sqap_f16 *k, int32_t batch, int32_t S,
                                     int32_t H, int32_t d, int32_t vis_begin, int32_t n_vis,
                                     float *scores_out, void *stream);

/*
 * Eq. 1: K_attn = Top_k(a_q, k).  For each of `batch` rows of `scores`
 * ([batch, n_tokens] floats) writes the indices of the keep_k largest values
 * to idx_out ([batch, keep_k] int32), in ascending index order.  The kept set
 * is unique: larger score first, equal scores -> lower index first, -0 == +0,
 * NaN ranks below every number (lower index first among NaN).
 * EINVAL: null pointer (when the size is non-zero), negative size,
 * keep_k > n_tokens.  EUNSUPPORTED: n_tokens > 65536.
 */
sqap_status sqap_prune_topk(const float *scores, int32_t batch, int32_t n_tokens,
                            int32_t keep_k, int32_t *idx_out, void *stream);

/*
 * Section 3.2 (final paragraph: the retained tokens form the shortened
 * sequence).  Turns kept visual indices into row numbers of the token matrix:
 * every token outside the visual span [vis_begin, vis_begin + n_vis) survives,
 * visual token v survives iff v is in idx[b,:]; original order is preserved.
 * idx: [batch, keep_k] ascending (as sqap_prune_topk writes it).
 * rows_out: [batch * (seq_len - n_vis + keep_k)] int32; observation b's rows
 * are offset by b * seq_len.
 * EINVAL: null pointer, negative size, keep_k > n_vis, span outside the sequence.
 */
sqap_status sqap_kept_rows(const int32_t *idx, int32_t batch, int32_t keep_k, int32_t seq_len,
                           int32_t vis_begin, int32_t n_vis, int32_t *rows_out, void *stream);

/*
 * The full selection rule of Section 3.2: K_final = K_attn + K_ring + K_fps.
 *
 * The visual tokens form a grid_w x grid_h grid, token (t_u, t_v) has index
 * t_v * grid_w + t_u (at most 1024 tokens).  For each of `batch` observations:
 *   K_attn = the k_attn highest scores (Eq. 1, same ranking as sqap_prune_topk);
 *   K_ring = tokens within Chebyshev distance ring_radius of the token that the
 *            observation's world point projects to (Eq. 2-4): a filled square
 *            clipped to the grid; empty if `camera` is null or the point is not
 *            in front of the camera;
 *   K_fps  = farthest point sampling (Eq. 5) of m = keep_total - |K_attn + K_ring|
 *            further tokens (none if that is not positive: the union is never
 *            cut), on token coordinates with squared Euclidean distance, the
 *            distance of a candidate being its minimum over everything kept so
 *            far, starting from K_attn + K_ring; largest distance first, lowest
 *            index among equals.
 *
 * scores    device, [batch, grid_w * grid_h] binary32.
 * camera    device or null, [batch, 26] binary64 per observation: the intrinsic
 *           matrix K (3 x 3, row-major), the extrinsic [R|t] (3 x 4, row-major),
 *           the world point (x, y, z), the patch width and height in pixels.
 *           The projection is evaluated in binary64: cam = R p + t, h = K cam
 *           (each dot product summed left to right), u = h0 / h2, v = h1 / h2,
 *           t_u = floor(u / patch_w), t_v = floor(v / patch_h).
 * idx_out   device, [batch, cap] int32: the members in ascending order, then -1.
 * cap       row pitch of idx_out; must hold the largest possible set:
 *           max(keep_total, min(tokens, k_attn + (2 ring_radius + 1)^2)).
 * count_out device or null, [batch] int32: size of each final set (keep_total
 *           whenever the union did not already exceed it).
 * EINVAL: null pointer, negative size, k_attn or keep_total above the token
 * count, cap too small.  EUNSUPPORTED: more than 1024 tokens.
 */
sqap_status sqap_prune_select(const float *scores, int32_t batch, int32_t grid_w, int32_t grid_h,
                              int32_t k_attn, int32_t keep_total, const double *camera,
                              int32_t ring_radius, int32_t *idx_out, int32_t cap, int32_t *count_out,
                              void *stream);

/*
 * sqap_prune_topk followed by sqap_kept_rows in one launch (Eq. 1 and the
 * shortened sequence of Section 3.2): scores [batch, n_vis] -> idx_out
 * [batch, keep_k] and rows_out [batch * (seq_len - n_vis + keep_k)], both exactly
 * as the two separate calls write them.  Same errors as those calls.
 */
sqap_status sqap_prune_rows(const float *scores, int32_t batch, int32_t n_vis, int32_t keep_k,
                            int32_t seq_len, int32_t vis_begin, int32_t *idx_out, int32_t *rows_out,
                            void *stream);

/*
 * Token gather (same passage): out[i, 0..K) = X[rows[i], 0..K), a bit copy of
 * half rows.  ldx / ldo are row pitches in elements (>= K).  K must be a
 * multiple of 8 and both base pointers and pitches 16-byte aligned
 * (EUNSUPPORTED otherwise).  Row numbers are not range-checked.
 */
sqap_status sqap_gather_rows(const sqap_f16 *X, int64_t ldx, const int32_t *rows, int32_t M,
                             int32_t K, sqap_f16 *out, int64_t ldo, void *stream);

/*
 * 4-bit activation quantizer, one scale per token (Section 3.3; Implementation
 * Details: W4A4).  For output row i, taken from X[rows[i], :] (or X[i, :] when
 * rows is NULL, which fuses the gather):
 *   v     = the row in binary32; with SQAP_ROTATE_HADAMARD, v <- (H/sqrt(K)) v
 *           (Eq. 6; butterflies at distance 1, 2, 4, ... in that order); when
 *           K is not a power of two, H is block diagonal with one matrix of
 *           order B per aligned run of B channels, B the largest power of two
 *           dividing K (256 for K = 11008), scaled by 1/sqrt(B)
 *   sx[i] = binary16(max|v| / 7), raised to 2^-24 when that rounds to 0
 *   code  = clamp(rint(v / sx[i]), -8, 7), round-half-even, IEEE division
 * Xq: [M, K/2] canonical packed int4.  sx: [M] half.
 * EINVAL: null pointer, M < 0, K <= 0, K odd, ldx < K.
 * EUNSUPPORTED: K not a multiple of 8, K > 16384, X/ldx not 16-byte aligned,
 * rotation with K not a multiple of 16.
 */
sqap_status sqap_quantize_act(const sqap_f16 *X, int64_t ldx, const int32_t *rows, int32_t M,
                              int32_t K, uint32_t flags, uint8_t *Xq, sqap_f16 *sx,
                              void *stream);

/*
 * 4-bit weight quantizer, one scale per output channel, round to nearest
 * (the paper's "tensor-wise", i.e. not group-wise, W4; offline step).  Same
 * arithmetic as sqap_quantize_act applied to the rows of W [N, K] (dense,
 * pitch K).  With SQAP_ROTATE_HADAMARD the rows are rotated first, which is
 * the (W^T H^T) factor of Eq. 6.  Wq: [N, K/2] canonical.  sw: [N] half.
 */
sqap_status sqap_quantize_weight(const sqap_f16 *W, int32_t N, int32_t K, uint32_t flags,
                                 uint8_t *Wq, sqap_f16 *sw, void *stream);

/*
 * Channel-wise activation quantization (Section 3.3: one activation scale per
 * input channel instead of one per token, so that a few large channels do not
 * flatten the others).  The scales are static: taken once from calibration
 * rows and folded into the weight, since a scale that varies along the
 * reduction axis cannot leave an integer dot product:
 *   x_k ~ c_k q_k,   y_n = sum_k x_k W_nk ~ sw_n sum_k q_k qw_nk,
 *   with qw, sw the per-output-channel quantization of W_nk * c_k.
 *
 * sqap_channel_scales: c_k = binary16(max over the M rows of |v_k| / 7), raised
 * to 2^-24 when that rounds to 0; v as in sqap_quantize_act (rotated first with
 * SQAP_ROTATE_HADAMARD).  amax: device, [K] binary32 running maxima, cleared by
 * the call unless accumulate != 0 (several calibration batches); scales_out:
 * device, [K] half, 16-byte aligned.
 *
 * sqap_quantize_act_channelwise: code = clamp(rint(v_k / c_k), -8, 7) (IEEE
 * division, round-half-even); Xq as sqap_quantize_act; sx[i] = 1 for every row,
 * so that sqap_w4a4_linear applies unchanged.
 *
 * sqap_quantize_weight_folded: the rows of W [N, K] (rotated first with the
 * flag), multiplied elementwise by c_k in binary32, then quantized per output
 * channel exactly as sqap_quantize_weight does.
 *
 * Errors as sqap_quantize_act; col_scales / scales_out must be 16-byte aligned.
 */
sqap_status sqap_channel_scales(const sqap_f16 *X, int64_t ldx, const int32_t *rows, int32_t M,
                                int32_t K, uint32_t flags, float *amax, int32_t accumulate,
                                sqap_f16 *scales_out, void *stream);
sqap_status sqap_quantize_act_channelwise(const sqap_f16 *X, int64_t ldx, const int32_t *rows,
                                          int32_t M, int32_t K, uint32_t flags,
                                          const sqap_f16 *col_scales, uint8_t *Xq, sqap_f16 *sx,
                                          void *stream);
sqap_status sqap_quantize_weight_folded(const sqap_f16 *W, int32_t N, int32_t K, uint32_t flags,
                                        const sqap_f16 *col_scales, uint8_t *Wq, sqap_f16 *sw,
                                        void *stream);

/*
 * Re-lays canonical packed weights [N, K/2] and their scales [N] into the
 * library's streaming layout and returns a handle that owns a device copy
 * (allocated with hipMalloc on the current device).  The inputs may be freed
 * once the stream has run past this call.  K must be a multiple of 32.
 * The first call on a device that sqap_init has not set up does that set-up
 * and so synchronises the stream once (see sqap_init).
 * EINVAL: null pointer, N/K <= 0.  EUNSUPPORTED: K % 32 != 0.  ENOMEM.
 */
sqap_status sqap_weight_pack(const uint8_t *Wq, const sqap_f16 *sw, int32_t N, int32_t K,
                             sqap_weight **out, void *stream);

/* Frees a handle (NULL is allowed).  The caller makes sure no kernel still uses it. */
sqap_status sqap_weight_free(sqap_weight *w);

/* Shape and device footprint of a handle; any out pointer may be NULL. */
sqap_status sqap_weight_info(const sqap_weight *w, int32_t *N, int32_t *K, size_t *device_bytes);

/*
 * Bytes of device workspace sqap_w4a4_linear needs for this shape (may be 0).
 * The workspace is scratch: contents before and after a call are unspecified.
 */
size_t sqap_workspace_bytes(int32_t M, int32_t N, int32_t K);

/*
 * W4A4 linear (the q/k/v/o, gate/up/down and lm_head layers of the quantized
 * backbone; Section 4.3 names them as where the time goes):
 *   acc[m,n] = sum_k xq[m,k] * wq[n,k]          exact, int32
 *   Y[m,n]   = binary16( ((float)acc * sx[m]) * sw[n] )
 * Xq: [M, K/2] canonical (pitch K/2, 16-byte aligned), sx: [M] half, W: a packed
 * handle with the same K, Y: [M, N] half with pitch ldy >= N elements.
 * acc_out: NULL, or [M, N] int32 (pitch N) that receives the accumulators.
 * workspace: at least sqap_workspace_bytes(M, N, K) bytes, 256-byte aligned
 * (may be NULL when that is 0); its contents need no initialisation.  Calls
 * that share a workspace must be ordered on one stream.  The large- and mid-M
 * kernels are persistent (one workgroup per compute unit) and split tiles
 * between workgroups, which exchange partial sums through the workspace; a
 * wait that does not end within a few seconds (two million polls) gives up, and
 * the result is then wrong.  Such a launch can be told from a good one whatever
 * the workspace held before: the launch's first workgroup clears the 64-bit
 * word at byte 4000 of the workspace when it starts and a wait that gives up
 * writes a nonzero value there, so after the launch the word is zero or the
 * output is wrong.  A launch may be captured in a HIP graph and replayed: every flag it
 * raises in the workspace is cleared again before it ends.  One entry point
 * serves prefill (large M) and decode (M <= 8); the kernel is chosen from M
 * inside.
 * EINVAL: null pointer, M < 0, ldy < N, workspace too small.
 */
sqap_status sqap_w4a4_linear(const uint8_t *Xq, const sqap_f16 *sx, int32_t M,
                             const sqap_weight *W, sqap_f16 *Y, int64_t ldy, int32_t *acc_out,
                             void *workspace, size_t workspace_bytes, void *stream);

/*
 * Decoder glue between the linears.  The paper runs its W4A4 linears inside a
 * Llama-2-7B decoder (Implementation Details; Section 3.3 takes Q and K from
 * it) and does not restate that architecture; the calls below follow the
 * published one: RMSNorm in front of each group of linears, rotary position
 * embedding, causal softmax attention, SwiGLU feed-forward, residual adds.
 * Every result that a quantizer consumes is rounded to binary16 first, so each
 * fused call equals the unfused sequence bit for bit.
 *
 * sqap_rmsnorm_quantize_act: for output row i taken from X[rows[i], :] (or
 * X[i, :] when rows is NULL):
 *   x' = binary16(x + delta[i, :])      when delta is given ([M, K] dense);
 *                                        xsum_out[i, :] = x' when asked for
 *   S  = sum_k x'_k^2, exact (128-bit integer arithmetic on the half values)
 *   r  = (float)(1 / sqrt(S / K + eps)) in binary64, S rounded to binary64 once
 *   y  = binary16((float(x') * r) * float(gamma))     two binary32 products
 * y_out[i, :] = y when asked for; then, when Xq is given, y is quantized as by
 * sqap_quantize_act (col_scales NULL: one scale per token, written to sx) or as
 * by sqap_quantize_act_channelwise (col_scales given).  flags as there.  Rows
 * must be finite.  delta, xsum_out, y_out: [M, K] dense halves, 16-byte
 * aligned; gamma: [K].  xsum_out may be X itself when rows is NULL and
 * ldx = K (update in place).  EINVAL: null X/gamma, neither Xq nor y_out, eps < 0.
 *
 * sqap_swiglu_quantize_act: h = binary16(silu(g) * float(u)) elementwise over
 * G, U [M, F] (pitches ldg, ldu), silu(g) = (float)(g / (1 + exp(-g)))
 * evaluated in binary64; h_out[i, :] = h when asked for; then quantized as
 * above (no rotation).
 */
sqap_status sqap_rmsnorm_quantize_act(const sqap_f16 *X, int64_t ldx, const int32_t *rows, int32_t M,
                                      int32_t K, const sqap_f16 *delta, const sqap_f16 *gamma, float eps,
                                      uint32_t flags, const sqap_f16 *col_scales, sqap_f16 *xsum_out,
                                      sqap_f16 *y_out, uint8_t *Xq, sqap_f16 *sx, void *stream);
sqap_status sqap_swiglu_quantize_act(const sqap_f16 *G, int64_t ldg, const sqap_f16 *U, int64_t ldu,
                                     int32_t M, int32_t F, const sqap_f16 *col_scales, sqap_f16 *h_out,
                                     uint8_t *Xq, sqap_f16 *sx, void *stream);

/*
 * Rotary position embedding, in place, half-split pairing: for token s, head h
 * and i < d/2, with a = pos[s] * base^(-2i/d),
 *   v'_i = v_i cos a - v_{i+d/2} sin a,   v'_{i+d/2} = v_{i+d/2} cos a + v_i sin a,
 * evaluated in binary64, rounded to binary32 and then to half (two roundings).
 * X: [S, H*d] with row pitch ld
 * (elements), so a slice of a fused q/k/v output can be rotated where it lies.
 * pos: [S] int32 device.  EINVAL: null pointer, d odd, ld < H*d, base <= 0.
 *
 * sqap_rope_append: the same rotation for a block of fused q|k|v rows [S, 3*H*d] (pitch ld) with the
 * key/value cache append folded in: queries are rotated in place; keys are rotated into KV[s, 0 .. H*d) and
 * values copied into KV[s, H*d .. 2*H*d) (KV: the cache rows these S tokens occupy, pitch ldkv >= 2*H*d); the
 * key and value columns of QKV are left as they were.  Bit-identical to sqap_rope on the q and k slices
 * followed by a row copy.  EINVAL: null pointer, d odd, a pitch too small, base <= 0.
 *
 * sqap_attention: causal softmax attention.  Query i (of Sq) sits at position
 * Sk - Sq + i of the key sequence and sees keys 0 .. Sk - Sq + i:
 *   o[i,h,:] = sum_t softmax_t((q[i,h,:] . k[t,h,:]) / sqrt(d)) v[t,h,:]
 * in binary32 (online softmax over tiles of 64 keys), rounded to half.
 * Q [Sq, H*d], K, V [Sk, H*d], O [Sq, H*d] with row pitches in elements; a
 * batch of independent sequences is a stack of such row blocks (sequence b
 * owns rows b*Sq .. of Q and O and rows b*Sk .. of K and V).
 * EINVAL: null pointer, Sk < Sq, pitch < H*d.  EUNSUPPORTED: d not in
 * {16, 32, 64, 128}, operands or pitches not 16-byte aligned.
 *
 * sqap_decode_attention: the attention of ONE new token of one sequence (a decode step) in a single
 * launch: sqap_rope_append of the token's fused q|k|v row QKV [3*H*d] into cache row `past`
 * (KV [>= past + 1, ldkv]: rotated key | value per position), sqap_attention of the rotated query
 * over cache rows 0 .. past into O [H*d], and, when Xq is given, sqap_quantize_act of O (flags 0)
 * into Xq [H*d/2], sx [1].  QKV is only read (the rotated query is not written back).  pos: [1]
 * int32 device, the token's position.  The cache row and Xq, sx hold the same bits as the three
 * separate calls give on the same O; O agrees with sqap_attention within the fp16 tolerance (the
 * order of the binary32 sums differs).  counter: one device uint32 the quantizer needs (the
 * workgroup that finishes last does it); zero before the first call, left zero by every call;
 * calls that share it must not overlap.  EINVAL: null pointer, H, d <= 0, past < 0, pitch below
 * 2*H*d, base <= 0, Xq without sx or counter.  EUNSUPPORTED: d not a multiple of 8 or above 128,
 * KV, ldkv or O not 16-byte aligned, H*d > 8192 with Xq.
 *
 * sqap_residual_add: X[i, :] <- binary16(float(X[i, :]) + float(delta[i, :])),
 * K a multiple of 8, 16-byte aligned rows.
 */
sqap_status sqap_rope(sqap_f16 *X, int64_t ld, const int32_t *pos, int32_t S, int32_t H, int32_t d,
                      double base, void *stream);
sqap_status sqap_rope_append(sqap_f16 *QKV, int64_t ld, const int32_t *pos, int32_t S, int32_t H, int32_t d,
                             double base, sqap_f16 *KV, int64_t ldkv, void *stream);
sqap_status sqap_attention(const sqap_f16 *Q, int64_t ldq, const sqap_f16 *K, int64_t ldk,
                           const sqap_f16 *V, int64_t ldv, int32_t batch, int32_t Sq, int32_t Sk, int32_t H,
                           int32_t d, sqap_f16 *O, int64_t ldo, void *stream);
sqap_status sqap_decode_attention(const sqap_f16 *QKV, const int32_t *pos, int32_t H, int32_t d, double base,
                                  sqap_f16 *KV, int64_t ldkv, int32_t past, sqap_f16 *O, uint8_t *Xq,
                                  sqap_f16 *sx, uint32_t *counter, void *stream);
sqap_status sqap_residual_add(sqap_f16 *X, int64_t ldx, const sqap_f16 *delta, int64_t ldd, int32_t M,
                              int32_t K, void *stream);

/*
 * Self-test of the quantizer's arithmetic.  The quantizer divides every element
 * of a row by the same scale; it does so with a reciprocal and two fused
 * corrections that give the correctly rounded binary32 quotient.  This call
 * checks that claim on the device for every pair (v, s) of finite half values,
 * s > 0, both signs of v, against the division operator, and ADDS the number of
 * differing bit patterns to *mismatches_out (a device uint64 the caller has
 * zeroed).  Expected result: 0.  EINVAL: null pointer.
 */
sqap_status sqap_selftest_quotient(uint64_t *mismatches_out, void *stream);

/*
 * Self-test of the dispatch order the persistent GEMM kernels rely on.  They
 * pass partial sums between workgroups b and b' of one launch with
 * b % 8 == b' % 8 through ordinary stores, which requires both to run behind
 * the same L2 (workgroup b on XCD b % 8, or a device with one L2).  The library
 * checks this once per device (sqap_init, or the first sqap_weight_pack), and uses
 * one-tile-per-workgroup kernels on a device where it does not hold.  This call
 * repeats the probe and writes the XCC id of each of the 256 workgroups of a
 * probe launch to xcc_of_block_out (HOST memory, 256 words); it synchronises
 * the stream.  Expected: out[b] == out[b % 8] for every b.  EINVAL: null.
 * Setting SQAP_DISABLE_PERSISTENT=1 in the environment selects the fallback
 * kernels on any device (read once per process, at the first sqap_w4a4_linear
 * call that could use a persistent kernel).  sqap_set_persistent_kernels is
 * the same switch at run time, process wide, for tests and diagnosis: 0 selects
 * the fallback kernels, anything else lets the library choose per device again
 * (and overrides the environment variable).  Always SQAP_OK.
 */
sqap_status sqap_selftest_dispatch(uint32_t *xcc_of_block_out, void *stream);
sqap_status sqap_set_persistent_kernels(int32_t enabled);

/*
 * Which kernel sqap_w4a4_linear uses for 8 < M < 512 with K a multiple of 256 (and at least 1024): 1, the
 * default, the kernel in which every workgroup owns complete outputs and nothing passes between
 * workgroups (it needs no workspace); 0 the tile kernels that split K between workgroups and exchange
 * partial sums through the workspace (which other shapes always use).  Same results bit for bit; process
 * wide; for tests and measurement.  sqap_workspace_bytes reports what the second kind needs either way.
 * Always SQAP_OK.
 */
sqap_status sqap_set_mid_m_kernel(int32_t which);

/*
 * The work split of the stream-K linear (M > 8, K a multiple of 128), as a
 * host-side computation: no GPU is touched.  A launch runs 8 x blocks_per_xcd
 * persistent workgroups; the output tiles (256 x 256 from M = 512 on, 96 or
 * 160 rows x 128 columns below: *tile_rows_out, *tile_cols_out) are dealt to
 * the 8 XCDs in contiguous runs and workgroup j of XCD x runs main-loop steps
 * [bounds[x][j], bounds[x][j + 1]) of its XCD's run (tile after tile, K / 128
 * steps each), so a tile can be shared along K; the workgroup holding a
 * tile's last step adds the others' partial sums and stores the tile.  The
 * bounds are planned from measured costs (epilogues, partial exchange, the
 * shorter steps of a ragged last tile row) so that the workgroups finish
 * together.  (Launches with at most 64 narrow tiles use another kernel, whose
 * contributors finish a tile jointly from equal step counts; the plan is
 * reported for them all the same.)  bounds_out: HOST, 8 x 33 words, row x =
 * XCD x (entries past blocks_per_xcd repeat the total).  planned_steps_out /
 * even_steps_out: HOST, 8 doubles each: the finishing time the cost model
 * predicts for the planned shares and for equal step counts, in units of one
 * main-loop step.  blocks_per_xcd: 1 ... 32 (a 256-CU device uses 32).
 * EINVAL: null pointers, sizes <= 0, blocks_per_xcd out of range;
 * EUNSUPPORTED: M <= 8, K not a multiple of 128 or above the K limit.
 */
sqap_status sqap_plan_linear_shares(int32_t M, int32_t N, int32_t K, int32_t blocks_per_xcd,
                                    uint32_t *bounds_out, double *planned_steps_out,
                                    double *even_steps_out, int32_t *tile_rows_out,
                                    int32_t *tile_cols_out);

/*
 * Grouped small-M linears (autoregressive decode, M <= 8).  Decode streams
 * every weight once per step and a single linear moves only a few megabytes,
 * so launching linears one by one leaves the memory system idle between them.
 * A group is a device-resident table of INDEPENDENT problems (for example
 * q/k/v of one layer, which share an input, or gate/up) that one launch
 * streams through back to back; each problem computes exactly what
 * sqap_w4a4_linear computes.  Build the group once, run it every step.
 *
 * descs is a HOST array; the device pointers inside it are captured, not
 * copied, and must stay valid while the group is used.  That includes the
 * packed weights: a group keeps the device addresses of each problem's
 * sqap_weight, not a reference to the handle, so every weight must outlive
 * (not be freed before) every group built from it.  Outputs of different
 * problems must not overlap.
 * EINVAL: null pointers, count <= 0, M < 1, ldy < N, bad weight handle.
 * EUNSUPPORTED: some M > 8 or some K not a multiple of 64.  ENOMEM / EDEVICE.
 */
typedef struct sqap_linear_desc {
    const uint8_t *Xq;      /* [M, K/2] canonical, 16-byte aligned */
    const sqap_f16 *sx;     /* [M] */
    int32_t M;
    const sqap_weight *W;
    sqap_f16 *Y;            /* [M, N], pitch ldy */
    int64_t ldy;
    int32_t *acc_out;       /* NULL or [M, N] int32 */
} sqap_linear_desc;

typedef struct sqap_group sqap_group;

sqap_status sqap_group_create(const sqap_linear_desc *descs, int32_t count, sqap_group **out);

/* Enqueues the whole group on `stream` as one launch.  No host synchronisation. */
sqap_status sqap_group_run(const sqap_group *g, void *stream);

/*
 * How sqap_group_run will launch a group (host arithmetic only; no GPU work): the number of problems and of
 * row groups (32 output channels each) in it, and the form of the small-M kernel the launch takes on a
 * device with `compute_units` compute units (0: the current device): wavefronts that share one row
 * group along K (1, 2, 4 or 8), wavefronts per workgroup (8, or 16 for launches in which every wavefront
 * streams four or more row groups: outputs then wait in LDS slots, output_slots_out per wavefront, 0
 * otherwise).  Any out pointer may be NULL.  EINVAL: not a group handle, compute_units < 0.
 */
sqap_status sqap_group_info(const sqap_group *g, int32_t compute_units, int32_t *problems_out,
                            int32_t *row_groups_out, int32_t *wavefronts_per_row_group_out,
                            int32_t *wavefronts_per_workgroup_out, int32_t *output_slots_out);

/* Frees a group (NULL allowed); the caller makes sure no launch still uses it. */
sqap_status sqap_group_free(sqap_group *g);

/*
 * One decode step as ONE launch (autoregressive action-token decode at batch 1: the memory-bound
 * regime of Section 4.3's linears, where every weight is streamed once per token).  A decoder is a device-
 * resident description of a Llama-shaped model: per layer the packed q|k|v ([3 hidden, hidden]), o, gate|up
 * ([2 ffn, hidden], gate rows first) and down weights, the two norm gains and the layer's key/value cache
 * ([capacity, ldkv] halves: rotated key | value per position, as sqap_rope_append and
 * sqap_decode_attention keep it); plus the final norm gain and the vocabulary head.  A step runs, for the
 * token with embedding x [hidden] at position pos[0] and `past` positions already in the caches, exactly
 * the chain
 *   sqap_rmsnorm_quantize_act -> sqap_w4a4_linear(q|k|v) -> sqap_decode_attention (appends cache row `past`)
 *   -> sqap_quantize_act -> sqap_w4a4_linear(o) -> sqap_rmsnorm_quantize_act (residual add fused)
 *   -> sqap_w4a4_linear(gate|up) -> sqap_swiglu_quantize_act -> sqap_w4a4_linear(down)
 * for every layer (each layer's trailing residual add fused into the next norm), then the final norm and the
 * head, in one persistent kernel of 256 workgroups that hand the small rows between the linears to each
 * other on the device and keep the weight stream running across those hand-overs.  Same bits as the chain
 * wherever the chain is exact (everything but the attention output, which agrees within the fp16
 * tolerance: the order of its binary32 sums is that of sqap_decode_attention).
 *
 * The handle owns the device memory of the rows in flight (4 * (7 hidden + ffn) bytes per layer) and of the
 * workgroups' progress flags; the weights, gains and caches are captured by address and must outlive it.  One step at a time per decoder (steps are
 * ordered on one stream).  A step writes row `past` of every layer's cache: the caller makes sure that
 * past < capacity (the library does not know the caches' sizes).  logits: [vocab] halves.  attn_trace: NULL, or [n_layers, hidden] halves that
 * receive every layer's attention output (tests feed it to the reference).  The kernel needs all its 256
 * workgroups resident at once (a device with at least 256 compute units; EUNSUPPORTED otherwise).  A
 * workgroup's wait for another's output that does not end within a second or so gives up: the step's outputs
 * are then wrong and sqap_decoder_status reports a nonzero word (it copies 8 bytes back and SYNCHRONISES the
 * stream; the word is cleared when a step starts).  The decoder stays usable.
 * A captured step can be replayed from a HIP graph.
 * EINVAL: null pointer, a handle that is not a weight, shapes that do not fit each other, negative
 * past.  EUNSUPPORTED: head size not a multiple of 8 or above 128, hidden above 4096, ffn above 12288, either not a
 * multiple of 128, more than 256 heads, a linear with more than 16 groups of 16 channels per compute unit
 * (N above 65536), operands not 16-byte aligned.  ENOMEM / EDEVICE.
 */
typedef struct sqap_decoder sqap_decoder;
typedef struct sqap_decoder_layer {
    const sqap_weight *qkv, *o, *gate_up, *down;
    const sqap_f16 *gamma_attn, *gamma_mlp;   /* device, [hidden] each, 16-byte aligned */
    sqap_f16 *kv;                             /* device, this layer's cache */
    int64_t ldkv;                             /* cache row pitch in elements, >= 2 * hidden */
} sqap_decoder_layer;

sqap_status sqap_decoder_create(const sqap_decoder_layer *layers, int32_t n_layers, int32_t n_heads,
                                int32_t head_dim, const sqap_f16 *gamma_final, const sqap_weight *head,
                                float eps, double rope_base, sqap_decoder **out);
sqap_status sqap_decoder_step(sqap_decoder *d, const sqap_f16 *x, const int32_t *pos, int32_t past,
                              sqap_f16 *logits, sqap_f16 *attn_trace, void *stream);
sqap_status sqap_decoder_status(const sqap_decoder *d, uint64_t *error_word_out, void *stream);
/* How many times a workgroup of the step kernel looks for another's output before it gives up (default: a
 * negative value restores it; about 200 000 looks, a few tenths of a second).  Applies to the steps enqueued
 * afterwards.  With 0 a step never waits: it ends at once with a nonzero status word and wrong outputs, which
 * is how the tests exercise the give-up path without a kernel that waits for long.  EINVAL: not a decoder. */
sqap_status sqap_decoder_set_wait_limit(sqap_decoder *d, int64_t polls);
sqap_status sqap_decoder_free(sqap_decoder *d);

#ifdef __cplusplus
}
#endif
#endif /* SQAP_H */
