/*
 * CPU oracle for the SQAP-VLA hot path: TEST INFRASTRUCTURE ONLY.
 *
 * Plain C, one loop nest per definition, no blocking, no fusion.  It exists so
 * that the HIP library can be checked element by element; it shares no code,
 * header, table or helper with that library and must never be called by it.
 * Only the test-suite, the smoke check and the benchmark's cpu_baseline leg
 * may load this object.
 *
 * Every function names the passage of the paper (arXiv 2509.09090) it follows.
 * Where the paper leaves arithmetic open (int4 range, rounding, scale format)
 * the reading taken is written next to the code.
 *
 * Half-precision values cross this interface as IEEE binary16 bit patterns in
 * uint16_t, because the host compiler has no half type.
 *
 * Parity pins: every function below is pinned by tests that do not re-type its
 * formula (stable library sort, numpy integer matmul, numpy half conversion,
 * dense Sylvester matrix product, closed forms, brute force).  The one
 * exception is oracle_attn_scores: its arithmetic is pinned (generic softmax
 * attention row), but WHICH layer, query token and head aggregation define
 * the retention score is not fixed by the paper: "parity unpinned" for that
 * choice.  Likewise for Eq. 5: farthest point sampling itself is pinned (a
 * hand-worked sequence, the max-min property step by step, a running-minimum
 * formulation), but the set it starts from, the metric and the tie-break are
 * readings the paper does not fix: "parity unpinned" for those choices.
 * The decoder glue at the end of the file (RMSNorm, rotary embedding, causal
 * attention, SwiGLU, residual add) is not described by the paper at all; it
 * follows the published Llama-2 architecture and is pinned by closed forms
 * (constant rows, zero queries, position 0), exact rational arithmetic for the
 * sum of squares, 50-digit decimal evaluation of silu, complex multiplication
 * for the rotation and a matrix formulation of attention with library softmax.
 */
#include <limits.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ */
/* binary16 <-> binary32, written out bit by bit                       */
/* ------------------------------------------------------------------ */

float oracle_f16_to_f32(uint16_t h)
{
    uint32_t sign = (uint32_t)(h >> 15) & 1u;
    uint32_t exp = (uint32_t)(h >> 10) & 0x1fu;
    uint32_t man = (uint32_t)h & 0x3ffu;
    double v;
    if (exp == 0x1fu) {
        if (man != 0) return sign ? -NAN : NAN;
        v = INFINITY;
    } else if (exp == 0) {
        v = ldexp((double)man, -24);            /* subnormal: man * 2^-24 */
    } else {
        v = ldexp((double)(man + 1024u), (int)exp - 25);
    }
    return (float)(sign ? -v : v);              /* exact: 11 significant bits */
}

/* round-to-nearest-even conversion, subnormals kept, overflow to infinity */
uint16_t oracle_f32_to_f16(float f)
{
    uint32_t bits;
    memcpy(&bits, &f, 4);
    uint16_t sign = (uint16_t)((bits >> 16) & 0x8000u);
    if (isnan(f)) return (uint16_t)(sign | 0x7e00u);
    double a = fabs((double)f);
    if (a >= 65520.0) return (uint16_t)(sign | 0x7c00u);   /* rounds to inf */
    if (a == 0.0) return sign;
    int e;
    (void)frexp(a, &e);                         /* a = m * 2^e, m in [0.5,1) */
    int ulp_exp = e - 11;                       /* 11 significant bits        */
    if (ulp_exp < -24) ulp_exp = -24;           /* subnormal spacing          */
    double q = ldexp(a, -ulp_exp);              /* exact scaling              */
    double r = nearbyint(q);                    /* default mode: ties to even */
    double rounded = ldexp(r, ulp_exp);
    /* re-encode the rounded value (it is representable by construction) */
    if (rounded >= 65520.0) return (uint16_t)(sign | 0x7c00u);
    if (rounded < ldexp(1.0, -14)) {
        return (uint16_t)(sign | (uint16_t)ldexp(rounded, 24));
    }
    int e2;
    double m2 = frexp(rounded, &e2);            /* m2 in [0.5,1) */
    uint32_t man = (uint32_t)ldexp(m2, 11) - 1024u;
    uint32_t ex = (uint32_t)(e2 - 1 + 15);
    return (uint16_t)(sign | (ex << 10) | man);
}

/* ------------------------------------------------------------------ */
/* Strategy 1, Eq. 1: K_attn = Top_k(a_q, k)                           */
/* ------------------------------------------------------------------ */
/*
 * Reading of what Eq. 1 leaves open: the set is made unique by the total
 * order "larger score first, equal scores: lower index first"; -0 equals +0;
 * NaN ranks below every number; the kept indices are returned ascending.
 */
static int ranks_before(float sa, int ia, float sb, int ib)
{
    int na = isnan(sa), nb = isnan(sb);
    if (na || nb) {
        if (na && nb) return ia < ib;
        return nb;                     /* a number ranks before a NaN */
    }
    if (sa > sb) return 1;
    if (sa < sb) return 0;
    return ia < ib;
}

int oracle_prune_topk(const float *scores, int batch, int n_tokens, int keep_k,
                      int32_t *idx_out)
{
    if (batch < 0 || n_tokens < 0 || keep_k < 0 || keep_k > n_tokens) return -1;
    int32_t *order = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n_tokens > 0 ? n_tokens : 1));
    if (!order) return -4;
    for (int b = 0; b < batch; ++b) {
        const float *s = scores + (size_t)b * n_tokens;
        /* full insertion sort into descending rank order */
        for (int i = 0; i < n_tokens; ++i) {
            int j = i;
            while (j > 0 && ranks_before(s[i], i, s[order[j - 1]], order[j - 1])) {
                order[j] = order[j - 1];
                --j;
            }
            order[j] = i;
        }
        /* first keep_k of that order, reported by ascending index */
        int32_t *out = idx_out + (size_t)b * keep_k;
        for (int i = 0; i < keep_k; ++i) {
            int j = i;
            while (j > 0 && out[j - 1] > order[i]) {
                out[j] = out[j - 1];
                --j;
            }
            out[j] = order[i];
        }
    }
    free(order);
    return 0;
}

/* ------------------------------------------------------------------ */
/* Section 3.2, strategies 2 and 3: Eq. 2-5 and the final union         */
/* ------------------------------------------------------------------ */
/*
 * Eq. 2 and Eq. 3: a world point is taken into the camera frame by [R|t],
 * onto the image plane by K, and the pixel is mapped to its patch.
 * cam = R p + t, h = K cam, (u, v) = (h0/h2, h1/h2), t_u = floor(u/P_w),
 * t_v = floor(v/P_h).  Reading (the paper fixes no precision): binary64,
 * every dot product summed left to right, no fused multiply-add.  Kmat is
 * 3x3 and Rt is 3x4, both row-major.  Returns 1 and the token coordinates if
 * the point is in front of the camera (h2 > 0) and u, v are finite and within
 * +-2^30 patches; 0 otherwise (then there is no ring).
 */
int oracle_project_token(const double *Kmat, const double *Rt, const double *xyz,
                         double patch_w, double patch_h, int32_t *tu, int32_t *tv)
{
    double cam[3], h[3];
    for (int i = 0; i < 3; ++i)
        cam[i] = ((Rt[4 * i] * xyz[0] + Rt[4 * i + 1] * xyz[1]) + Rt[4 * i + 2] * xyz[2]) + Rt[4 * i + 3];
    for (int i = 0; i < 3; ++i)
        h[i] = (Kmat[3 * i] * cam[0] + Kmat[3 * i + 1] * cam[1]) + Kmat[3 * i + 2] * cam[2];
    if (!(h[2] > 0.0)) return 0;
    double fu = floor((h[0] / h[2]) / patch_w), fv = floor((h[1] / h[2]) / patch_h);
    if (!(fabs(fu) <= 1073741824.0) || !(fabs(fv) <= 1073741824.0)) return 0;
    *tu = (int32_t)fu;
    *tv = (int32_t)fv;
    return 1;
}

/*
 * Eq. 4: the protected set is every token of the grid whose Chebyshev distance
 * from the centre token is at most R_t.  Reading: a filled square, clipped to
 * the grid (the centre itself may lie outside the image).  Token (t_u, t_v)
 * has index t_v * grid_w + t_u.  flags[i] = 1 for members.
 */
int oracle_ring(int grid_w, int grid_h, int cu, int cv, int radius, uint8_t *flags)
{
    if (grid_w <= 0 || grid_h <= 0 || radius < 0) return -1;
    for (int v = 0; v < grid_h; ++v)
        for (int u = 0; u < grid_w; ++u) {
            long du = labs((long)u - cu), dv = labs((long)v - cv);
            flags[v * grid_w + u] = (uint8_t)((du > dv ? du : dv) <= radius);
        }
    return 0;
}

/*
 * Eq. 5: farthest point sampling of m tokens from the tokens not yet kept.
 * Reading (the paper names FPS only): points are the token coordinates on the
 * grid, distance is squared Euclidean in integers, a candidate's distance is
 * its minimum over the tokens kept so far, the set it starts from being
 * K_attn + K_ring (so that the FINAL set is spread out, as the text asks),
 * and each step takes the candidate with the largest such distance, the lowest
 * index among equals.  With nothing kept yet every distance is infinite and
 * the first pick is token 0.  kept[] is updated; picks_out gets the m picks in
 * the order they were made.  Written as the definition: every step recomputes
 * every minimum from scratch.
 */
int oracle_fps(int grid_w, int grid_h, uint8_t *kept, int m, int32_t *picks_out)
{
    const int n = grid_w * grid_h;
    if (grid_w <= 0 || grid_h <= 0 || m < 0) return -1;
    for (int step = 0; step < m; ++step) {
        long best_d = -1;
        int best = -1;
        for (int c = 0; c < n; ++c) {
            if (kept[c]) continue;
            long dmin = LONG_MAX;
            for (int s = 0; s < n; ++s) {
                if (!kept[s]) continue;
                long du = (c % grid_w) - (s % grid_w), dv = (c / grid_w) - (s / grid_w);
                long d = du * du + dv * dv;
                if (d < dmin) dmin = d;
            }
            if (dmin > best_d) {          /* strict: the lowest index among equals stays */
                best_d = dmin;
                best = c;
            }
        }
        if (best < 0) return -2;          /* fewer than m candidates */
        kept[best] = 1;
        picks_out[step] = best;
    }
    return 0;
}

/*
 * Final set: K_attn + K_ring + K_fps.  K_attn = Top_k(scores, k_attn) over all
 * tokens (Eq. 1), K_ring as above (absent when have_ring = 0), and the quota
 * left, m = keep_total - |K_attn + K_ring|, is filled by FPS (none if the two
 * sets already reach the total: the union is never cut).  idx_out receives the
 * members in ascending order (capacity: grid_w * grid_h); returns their number,
 * or a negative status.
 */
int oracle_prune_select(const float *scores, int grid_w, int grid_h, int k_attn, int keep_total,
                        int have_ring, int cu, int cv, int radius, int32_t *idx_out)
{
    const int n = grid_w * grid_h;
    if (grid_w <= 0 || grid_h <= 0 || k_attn < 0 || k_attn > n || keep_total < 0 || keep_total > n ||
        radius < 0)
        return -1;
    uint8_t *kept = (uint8_t *)calloc((size_t)n, 1);
    int32_t *tmp = (int32_t *)malloc(sizeof(int32_t) * (size_t)n);
    if (!kept || !tmp) {
        free(kept);
        free(tmp);
        return -4;
    }
    int rc = oracle_prune_topk(scores, 1, n, k_attn, tmp);
    for (int i = 0; rc == 0 && i < k_attn; ++i) kept[tmp[i]] = 1;
    if (rc == 0 && have_ring) {
        uint8_t *ring = (uint8_t *)malloc((size_t)n);
        if (!ring) rc = -4;
        if (rc == 0) rc = oracle_ring(grid_w, grid_h, cu, cv, radius, ring);
        for (int i = 0; rc == 0 && i < n; ++i) kept[i] |= ring[i];
        free(ring);
    }
    int count = 0;
    for (int i = 0; i < n; ++i) count += kept[i];
    if (rc == 0 && keep_total > count) {
        rc = oracle_fps(grid_w, grid_h, kept, keep_total - count, tmp);
        count = keep_total;
    }
    int o = 0;
    for (int i = 0; rc == 0 && i < n; ++i)
        if (kept[i]) idx_out[o++] = i;
    free(kept);
    free(tmp);
    return rc == 0 ? count : rc;
}

/*
 * Section 3.2, last paragraph: the kept visual tokens shorten the sequence.
 * Reading: the surviving sequence keeps the original order; every token
 * outside the visual span [vis_begin, vis_begin+n_vis) is kept.  Row numbers
 * are global over the batch: observation b starts at row b*seq_len.
 * rows_out has batch*(seq_len-n_vis+keep_k) entries.
 */
int oracle_kept_rows(const int32_t *idx, int batch, int keep_k, int seq_len,
                     int vis_begin, int n_vis, int32_t *rows_out)
{
    if (batch < 0 || keep_k < 0 || keep_k > n_vis || vis_begin < 0 ||
        vis_begin + n_vis > seq_len)
        return -1;
    size_t o = 0;
    for (int b = 0; b < batch; ++b) {
        for (int s = 0; s < seq_len; ++s) {
            int keep = 1;
            if (s >= vis_begin && s < vis_begin + n_vis) {
                keep = 0;
                for (int i = 0; i < keep_k; ++i)
                    if (idx[(size_t)b * keep_k + i] == s - vis_begin) keep = 1;
            }
            if (keep) rows_out[o++] = b * seq_len + s;
        }
    }
    return 0;
}

/* gather: out[i,:] = X[rows[i],:], a bit copy of half-precision rows */
int oracle_gather_rows(const uint16_t *X, int64_t ldx, const int32_t *rows, int M,
                       int K, uint16_t *out, int64_t ldo)
{
    for (int i = 0; i < M; ++i)
        for (int k = 0; k < K; ++k)
            out[(size_t)i * ldo + k] = X[(size_t)rows[i] * ldx + k];
    return 0;
}

/* ------------------------------------------------------------------ */
/* Section 3.3, Eq. 6: rotation by the Hadamard matrix H               */
/* ------------------------------------------------------------------ */
/*
 * Reading: H is the Sylvester (natural-order) Walsh-Hadamard matrix scaled by
 * 1/sqrt(K) so that H^T H = I as Eq. 6 needs.  Arithmetic fixed so that a
 * parallel implementation can agree to the bit: binary32 butterflies, stage
 * distance h = 1, 2, 4, ..., K/2 in that order, (a,b) -> (a+b, a-b) with a
 * the lower index, then one multiply by (float)(1/sqrt(K)).
 */
int oracle_fwht_f32(float *v, int K)
{
    if (K <= 0 || (K & (K - 1)) != 0) return -2;
    for (int h = 1; h < K; h *= 2) {
        for (int base = 0; base < K; base += 2 * h) {
            for (int j = base; j < base + h; ++j) {
                float a = v[j], b = v[j + h];
                v[j] = a + b;
                v[j + h] = a - b;
            }
        }
    }
    float c = (float)(1.0 / sqrt((double)K));
    for (int j = 0; j < K; ++j) v[j] = v[j] * c;
    return 0;
}

/*
 * Rotation of a row whose length is not a power of two (the feed-forward width
 * 11008 = 43 * 256).  Eq. 6 only needs H orthogonal.  Reading: H is block
 * diagonal, one orthonormal Sylvester matrix of order B per aligned block of B
 * consecutive channels, B the largest power of two that divides K (for a power
 * of two this is the single matrix above).  Outlier energy is then spread over
 * the 256 channels of its block instead of over the whole row.
 */
int oracle_rotation_block(int K)
{
    int B = 1;
    while (K > 0 && (K % (2 * B)) == 0) B *= 2;
    return B;
}

int oracle_rotate_f32(float *v, int K)
{
    if (K <= 0) return -2;
    int B = oracle_rotation_block(K);
    for (int base = 0; base < K; base += B) {
        int rc = oracle_fwht_f32(v + base, B);
        if (rc) return rc;
    }
    return 0;
}

/* ------------------------------------------------------------------ */
/* 4-bit symmetric quantizer, one scale per row                        */
/* (Section 3.3 / Implementation Details: W4A4; the arithmetic is a    */
/* reading: divisor 7, ties-to-even, binary16 scale, no zero point)    */
/* ------------------------------------------------------------------ */
/*
 * For each output row i (a token for activations, an output channel for
 * weights), taken from source row rows[i] (or i when rows is NULL):
 *   v      = binary32 of the row, rotated by oracle_rotate_f32 when rotate != 0
 *   amax   = max_k |v_k|
 *   scale  = binary16(amax / 7), raised to the smallest subnormal 2^-24 if 0
 *   q_k    = clamp(rint(v_k / (float)scale), -8, 7)
 *   byte j = (q_{2j} & 15) | (q_{2j+1} & 15) << 4        (two's complement)
 *   rowsum = sum_k q_k
 */
int oracle_quantize_rows(const uint16_t *X, int64_t ldx, const int32_t *rows, int M,
                         int K, int rotate, uint8_t *Xq, uint16_t *scale_out,
                         int32_t *rowsum_out)
{
    if (M < 0 || K <= 0 || (K & 1)) return -1;
    if (rotate && oracle_rotation_block(K) < 16) return -2;
    int status = 0;
#pragma omp parallel for schedule(static)
    for (int i = 0; i < M; ++i) {
        float *v = (float *)malloc(sizeof(float) * (size_t)K);
        if (!v) {
#pragma omp atomic write
            status = -4;
            continue;
        }
        size_t src = rows ? (size_t)rows[i] : (size_t)i;
        for (int k = 0; k < K; ++k) v[k] = oracle_f16_to_f32(X[src * ldx + k]);
        if (rotate) oracle_rotate_f32(v, K);
        float amax = 0.0f;
        for (int k = 0; k < K; ++k) {
            float a = fabsf(v[k]);
            if (a > amax) amax = a;
        }
        uint16_t sh = oracle_f32_to_f16(amax / 7.0f);
        if (sh == 0) sh = 1;                     /* 2^-24: keeps the scale positive */
        float sf = oracle_f16_to_f32(sh);
        int32_t sum = 0;
        for (int k = 0; k < K; k += 2) {
            int q[2];
            for (int t = 0; t < 2; ++t) {
                float r = rintf(v[k + t] / sf);
                if (r > 7.0f) r = 7.0f;
                if (r < -8.0f) r = -8.0f;
                q[t] = (int)r;
                sum += q[t];
            }
            Xq[(size_t)i * (K / 2) + k / 2] =
                (uint8_t)((q[0] & 15) | ((q[1] & 15) << 4));
        }
        scale_out[i] = sh;
        if (rowsum_out) rowsum_out[i] = sum;
        free(v);
    }
    return status;
}

/* ------------------------------------------------------------------ */
/* Section 3.3: channel-wise quantization of activations               */
/* ------------------------------------------------------------------ */
/*
 * The paper proposes one activation scale per input channel instead of one per
 * token, so that a few large channels do not flatten all the others.  Reading
 * (the paper gives no formula): the scales are static, taken from calibration
 * rows,
 *   c_k = binary16(max_rows |v_k| / 7), raised to 2^-24 if 0,
 * with v the row in binary32, rotated first when rotate != 0.  A scale that
 * varies along the reduction axis cannot leave an integer dot product, so it
 * is folded into the weight before the weight is quantized:
 *   x_k ~ c_k q_k,   y_n = sum_k x_k W_nk ~ sum_k q_k (c_k W_nk).
 */
int oracle_channel_scales(const uint16_t *X, int64_t ldx, const int32_t *rows, int M, int K,
                          int rotate, uint16_t *scales_out)
{
    if (M < 0 || K <= 0) return -1;
    if (rotate && oracle_rotation_block(K) < 16) return -2;
    float *amax = (float *)calloc((size_t)K, sizeof(float));
    float *v = (float *)malloc(sizeof(float) * (size_t)K);
    if (!amax || !v) {
        free(amax);
        free(v);
        return -4;
    }
    for (int i = 0; i < M; ++i) {
        size_t src = rows ? (size_t)rows[i] : (size_t)i;
        for (int k = 0; k < K; ++k) v[k] = oracle_f16_to_f32(X[src * ldx + k]);
        if (rotate) oracle_rotate_f32(v, K);
        for (int k = 0; k < K; ++k)
            if (fabsf(v[k]) > amax[k]) amax[k] = fabsf(v[k]);
    }
    for (int k = 0; k < K; ++k) {
        uint16_t sh = oracle_f32_to_f16(amax[k] / 7.0f);
        scales_out[k] = sh == 0 ? 1 : sh;
    }
    free(amax);
    free(v);
    return 0;
}

/*
 * Activations with the static channel scales: q_k = clamp(rint(v_k / (float)c_k), -8, 7),
 * packed as in oracle_quantize_rows.  The per-token scale that the linear's
 * epilogue multiplies by is 1 for every token (binary16 0x3c00).
 */
int oracle_quantize_rows_channelwise(const uint16_t *X, int64_t ldx, const int32_t *rows, int M,
                                     int K, int rotate, const uint16_t *col_scales, uint8_t *Xq,
                                     uint16_t *scale_out)
{
    if (M < 0 || K <= 0 || (K & 1)) return -1;
    if (rotate && oracle_rotation_block(K) < 16) return -2;
    int status = 0;
#pragma omp parallel for schedule(static)
    for (int i = 0; i < M; ++i) {
        float *v = (float *)malloc(sizeof(float) * (size_t)K);
        if (!v) {
#pragma omp atomic write
            status = -4;
            continue;
        }
        size_t src = rows ? (size_t)rows[i] : (size_t)i;
        for (int k = 0; k < K; ++k) v[k] = oracle_f16_to_f32(X[src * ldx + k]);
        if (rotate) oracle_rotate_f32(v, K);
        for (int k = 0; k < K; k += 2) {
            int q[2];
            for (int t = 0; t < 2; ++t) {
                float r = rintf(v[k + t] / oracle_f16_to_f32(col_scales[k + t]));
                if (r > 7.0f) r = 7.0f;
                if (r < -8.0f) r = -8.0f;
                q[t] = (int)r;
            }
            Xq[(size_t)i * (K / 2) + k / 2] = (uint8_t)((q[0] & 15) | ((q[1] & 15) << 4));
        }
        scale_out[i] = 0x3c00;
        free(v);
    }
    return status;
}

/*
 * Weight with the channel scales folded in: row n of W (rotated first when
 * rotate != 0) is multiplied elementwise by (float)c_k in binary32, then
 * quantized per output channel exactly as oracle_quantize_rows does.
 */
int oracle_quantize_rows_folded(const uint16_t *W, int64_t ldw, int N, int K, int rotate,
                                const uint16_t *col_scales, uint8_t *Wq, uint16_t *scale_out)
{
    if (N < 0 || K <= 0 || (K & 1)) return -1;
    if (rotate && oracle_rotation_block(K) < 16) return -2;
    int status = 0;
#pragma omp parallel for schedule(static)
    for (int i = 0; i < N; ++i) {
        float *v = (float *)malloc(sizeof(float) * (size_t)K);
        if (!v) {
#pragma omp atomic write
            status = -4;
            continue;
        }
        for (int k = 0; k < K; ++k) v[k] = oracle_f16_to_f32(W[(size_t)i * ldw + k]);
        if (rotate) oracle_rotate_f32(v, K);
        float amax = 0.0f;
        for (int k = 0; k < K; ++k) {
            v[k] = v[k] * oracle_f16_to_f32(col_scales[k]);
            if (fabsf(v[k]) > amax) amax = fabsf(v[k]);
        }
        uint16_t sh = oracle_f32_to_f16(amax / 7.0f);
        if (sh == 0) sh = 1;
        float sf = oracle_f16_to_f32(sh);
        for (int k = 0; k < K; k += 2) {
            int q[2];
            for (int t = 0; t < 2; ++t) {
                float r = rintf(v[k + t] / sf);
                if (r > 7.0f) r = 7.0f;
                if (r < -8.0f) r = -8.0f;
                q[t] = (int)r;
            }
            Wq[(size_t)i * (K / 2) + k / 2] = (uint8_t)((q[0] & 15) | ((q[1] & 15) << 4));
        }
        scale_out[i] = sh;
        free(v);
    }
    return status;
}

/* signed value of nibble number k of a packed row */
static inline int nibble(const uint8_t *row, int k)
{
    int b = row[k >> 1];
    int u = (k & 1) ? (b >> 4) : (b & 15);
    return u >= 8 ? u - 16 : u;
}

/* unpack a packed row matrix to one int8 per code (helper for the GEMM) */
int oracle_unpack_int4(const uint8_t *Q, int R, int K, int8_t *out)
{
    for (int r = 0; r < R; ++r)
        for (int k = 0; k < K; ++k)
            out[(size_t)r * K + k] = (int8_t)nibble(Q + (size_t)r * (K / 2), k);
    return 0;
}

/* ------------------------------------------------------------------ */
/* W4A4 linear: exact integer contraction, then dequantisation         */
/* ------------------------------------------------------------------ */
/*
 * acc[m,n] = sum_k xq[m,k] * wq[n,k], accumulated both in int32 and in int64;
 * returns the number of entries where the two disagree (must be 0).
 */
int64_t oracle_int_gemm(const uint8_t *Xq, const uint8_t *Wq, int M, int N, int K,
                        int32_t *acc)
{
    int8_t *x = (int8_t *)malloc((size_t)(M > 0 ? M : 1) * K);
    int8_t *w = (int8_t *)malloc((size_t)(N > 0 ? N : 1) * K);
    if (!x || !w) {
        free(x);
        free(w);
        return -4;
    }
    oracle_unpack_int4(Xq, M, K, x);
    oracle_unpack_int4(Wq, N, K, w);
    int64_t bad = 0;
#pragma omp parallel for schedule(static) reduction(+ : bad)
    for (int n = 0; n < N; ++n) {
        for (int m = 0; m < M; ++m) {
            int32_t s32 = 0;
            int64_t s64 = 0;
            const int8_t *xr = x + (size_t)m * K, *wr = w + (size_t)n * K;
            for (int k = 0; k < K; ++k) {
                int p = (int)xr[k] * (int)wr[k];
                s32 += p;
                s64 += p;
            }
            if ((int64_t)s32 != s64) ++bad;
            acc[(size_t)m * N + n] = s32;
        }
    }
    free(x);
    free(w);
    return bad;
}

/* Y[m,n] = binary16( ((float)acc * sx[m]) * sw[n] ), two binary32 products */
int oracle_dequant(const int32_t *acc, const uint16_t *sx, const uint16_t *sw, int M,
                   int N, uint16_t *Y, int64_t ldy)
{
    for (int m = 0; m < M; ++m) {
        float a = oracle_f16_to_f32(sx[m]);
        for (int n = 0; n < N; ++n) {
            float t = (float)acc[(size_t)m * N + n] * a;
            float y = t * oracle_f16_to_f32(sw[n]);
            Y[(size_t)m * ldy + n] = oracle_f32_to_f16(y);
        }
    }
    return 0;
}

/*
 * The same two definitions evaluated only at chosen output positions
 * (ms[i], ns[i]); used where the full product is too slow to form.
 */
int oracle_linear_samples(const uint8_t *Xq, const uint16_t *sx, const uint8_t *Wq,
                          const uint16_t *sw, int K, const int32_t *ms,
                          const int32_t *ns, int count, int32_t *acc_out,
                          uint16_t *y_out)
{
    for (int i = 0; i < count; ++i) {
        const uint8_t *xr = Xq + (size_t)ms[i] * (K / 2);
        const uint8_t *wr = Wq + (size_t)ns[i] * (K / 2);
        int64_t s = 0;
        for (int k = 0; k < K; ++k) s += (int64_t)nibble(xr, k) * nibble(wr, k);
        acc_out[i] = (int32_t)s;
        float t = (float)(int32_t)s * oracle_f16_to_f32(sx[ms[i]]);
        y_out[i] = oracle_f32_to_f16(t * oracle_f16_to_f32(sw[ns[i]]));
    }
    return 0;
}

/* ------------------------------------------------------------------ */
/* Retention score a_q (Strategy 1 text; Section 3.3: Q, K from X)     */
/* ------------------------------------------------------------------ */
/*
 * Reading: the task-query token is one query vector per head q[h,:]; the
 * score of visual token j is its softmax attention weight over all S keys,
 * averaged over the H heads.  Double precision throughout.
 *   l[h,s] = (q[h,:] . k[s,h,:]) / sqrt(d)
 *   p[h,:] = softmax_s(l[h,:])
 *   score[j] = (1/H) sum_h p[h, vis_begin + j]
 */
int oracle_attn_scores(const uint16_t *q, const uint16_t *k, int S, int H, int d,
                       int vis_begin, int n_vis, float *scores_out)
{
    if (S <= 0 || H <= 0 || d <= 0 || vis_begin < 0 || n_vis < 0 ||
        vis_begin + n_vis > S)
        return -1;
    double *p = (double *)malloc(sizeof(double) * (size_t)S);
    double *acc = (double *)calloc((size_t)(n_vis > 0 ? n_vis : 1), sizeof(double));
    if (!p || !acc) {
        free(p);
        free(acc);
        return -4;
    }
    for (int h = 0; h < H; ++h) {
        double lmax = -INFINITY;
        for (int s = 0; s < S; ++s) {
            double dot = 0.0;
            for (int i = 0; i < d; ++i)
                dot += (double)oracle_f16_to_f32(q[(size_t)h * d + i]) *
                       (double)oracle_f16_to_f32(k[((size_t)s * H + h) * d + i]);
            p[s] = dot / sqrt((double)d);
            if (p[s] > lmax) lmax = p[s];
        }
        double z = 0.0;
        for (int s = 0; s < S; ++s) {
            p[s] = exp(p[s] - lmax);
            z += p[s];
        }
        for (int j = 0; j < n_vis; ++j) acc[j] += p[vis_begin + j] / z;
    }
    for (int j = 0; j < n_vis; ++j) scores_out[j] = (float)(acc[j] / (double)H);
    free(p);
    free(acc);
    return 0;
}

/* ------------------------------------------------------------------ */
/* Decoder glue between the linears                                    */
/* ------------------------------------------------------------------ */
/*
 * The paper runs its W4A4 linears inside a Llama-2-7B decoder (Implementation
 * Details; Section 3.3 takes Q = W_q^T X and K = W_k^T X from it) and does not
 * restate that architecture.  What follows is the published one, written out:
 * pre-normalisation by RMSNorm (Zhang & Sennrich 2019), rotary position
 * embedding in the half-split pairing (Su et al. 2021 as used by Llama),
 * causal softmax attention, and the SwiGLU feed-forward (Shazeer 2020).  Each
 * result that a later quantizer consumes is rounded to binary16 here, so that
 * the fused device kernels (norm + quantize, SwiGLU + quantize) are the
 * composition of one of these functions with oracle_quantize_rows.
 */

/*
 * RMSNorm of rows of halves, with an optional residual update first:
 *   x'_k = binary16(float(x_k) + float(delta_k))          (delta != NULL)
 *   S    = sum_k x'_k^2                                    exactly
 *   r    = (float)(1 / sqrt(S / K + eps))                  binary64, one rounding
 *   y_k  = binary16((float(x'_k) * r) * float(gamma_k))    two binary32 products
 * S is exact: a half is an integer m (|m| < 2^11) times 2^e with e >= -24, so
 * x^2 * 2^48 is an integer below 2^80 and the row sum fits 128 bits; it is
 * rounded to binary64 once.  Source row rows[i] (or i); delta, xsum_out and y_out
 * are dense [M, K] indexed by the output row.  xsum_out (nullable) receives x'.
 */
int oracle_rmsnorm_rows(const uint16_t *X, int64_t ldx, const int32_t *rows, int M, int K,
                        const uint16_t *delta, const uint16_t *gamma, float eps,
                        uint16_t *xsum_out, uint16_t *y_out)
{
    if (M < 0 || K <= 0 || !(eps >= 0.0f)) return -1;
    for (int i = 0; i < M; ++i) {
        size_t src = rows ? (size_t)rows[i] : (size_t)i;
        unsigned __int128 S = 0;
        for (int k = 0; k < K; ++k) {
            uint16_t h = X[src * ldx + k];
            if (delta) {
                float s = oracle_f16_to_f32(h) + oracle_f16_to_f32(delta[(size_t)i * K + k]);
                h = oracle_f32_to_f16(s);
            }
            if (xsum_out) xsum_out[(size_t)i * K + k] = h;
            y_out[(size_t)i * K + k] = h;                    /* parked: x' */
            uint32_t ex = (h >> 10) & 0x1fu, man = h & 0x3ffu;
            if (ex == 0x1fu) return -3;                       /* infinity or NaN in the row */
            uint32_t m = ex ? man + 1024u : man;
            int e = ex ? (int)ex - 25 : -24;                  /* |x| = m * 2^e */
            S += (unsigned __int128)((uint64_t)m * m) << (2 * e + 48);
        }
        double Sd = ldexp((double)S, -48);                    /* one rounding to nearest even */
        float r = (float)(1.0 / sqrt(Sd / (double)K + (double)eps));
        for (int k = 0; k < K; ++k) {
            float xv = oracle_f16_to_f32(y_out[(size_t)i * K + k]);
            float t = xv * r;
            float y = t * oracle_f16_to_f32(gamma[k]);
            y_out[(size_t)i * K + k] = oracle_f32_to_f16(y);
        }
    }
    return 0;
}

/*
 * SwiGLU gate: h = binary16(silu(g) * float(u)),
 *   silu(g) = (float)(g / (1 + exp(-g)))   evaluated in binary64, one rounding,
 * then one binary32 product and one rounding to half.  G, U: [M, F] halves
 * with row pitches ldg, ldu; H_out dense [M, F].
 */
int oracle_swiglu(const uint16_t *G, int64_t ldg, const uint16_t *U, int64_t ldu, int M, int F,
                  uint16_t *H_out)
{
    if (M < 0 || F < 0) return -1;
    for (int i = 0; i < M; ++i)
        for (int k = 0; k < F; ++k) {
            double g = (double)oracle_f16_to_f32(G[(size_t)i * ldg + k]);
            float s = (float)(g / (1.0 + exp(-g)));
            float h = s * oracle_f16_to_f32(U[(size_t)i * ldu + k]);
            H_out[(size_t)i * F + k] = oracle_f32_to_f16(h);
        }
    return 0;
}

/*
 * Rotary position embedding, half-split pairing: for a head vector v of even
 * size d at position p and i < d/2, with angle a = p * base^(-2i/d),
 *   v'_i       = v_i cos a - v_{i+d/2} sin a
 *   v'_{i+d/2} = v_{i+d/2} cos a + v_i sin a
 * in binary64; each result is rounded to binary32 and that to binary16 (two
 * roundings).  X: [S, H, d] halves, in place.
 */
int oracle_rope(uint16_t *X, const int32_t *pos, int S, int H, int d, double base)
{
    if (S < 0 || H <= 0 || d <= 0 || (d & 1)) return -1;
    for (int s = 0; s < S; ++s)
        for (int h = 0; h < H; ++h) {
            uint16_t *v = X + ((size_t)s * H + h) * d;
            for (int i = 0; i < d / 2; ++i) {
                double a = (double)pos[s] * pow(base, -2.0 * (double)i / (double)d);
                double lo = (double)oracle_f16_to_f32(v[i]);
                double hi = (double)oracle_f16_to_f32(v[i + d / 2]);
                v[i] = oracle_f32_to_f16((float)(lo * cos(a) - hi * sin(a)));
                v[i + d / 2] = oracle_f32_to_f16((float)(hi * cos(a) + lo * sin(a)));
            }
        }
    return 0;
}

/*
 * Causal softmax attention, one head at a time, binary64 throughout.  The Sq
 * queries are the last Sq positions of a sequence of Sk keys: query s sits at
 * position Sk - Sq + s and sees keys t <= Sk - Sq + s.
 *   l[s,t] = (q[s,h,:] . k[t,h,:]) / sqrt(d),   p[s,:] = softmax_t(l[s,:]),
 *   o[s,h,:] = sum_t p[s,t] v[t,h,:]  -> binary32 -> binary16 (two roundings).
 * Q, O: [Sq, H, d] halves; K, V: [Sk, H, d].  Queries and keys are taken as
 * given (rotate them with oracle_rope first).
 */
int oracle_attention(const uint16_t *Q, const uint16_t *Kc, const uint16_t *V, int Sq, int Sk, int H,
                     int d, uint16_t *O)
{
    if (Sq < 0 || Sk < Sq || H <= 0 || d <= 0) return -1;
    double *p = (double *)malloc(sizeof(double) * (size_t)(Sk > 0 ? Sk : 1));
    double *o = (double *)malloc(sizeof(double) * (size_t)d);
    if (!p || !o) {
        free(p);
        free(o);
        return -4;
    }
    for (int h = 0; h < H; ++h)
        for (int s = 0; s < Sq; ++s) {
            int last = Sk - Sq + s;
            double lmax = -INFINITY;
            for (int t = 0; t <= last; ++t) {
                double dot = 0.0;
                for (int i = 0; i < d; ++i)
                    dot += (double)oracle_f16_to_f32(Q[((size_t)s * H + h) * d + i]) *
                           (double)oracle_f16_to_f32(Kc[((size_t)t * H + h) * d + i]);
                p[t] = dot / sqrt((double)d);
                if (p[t] > lmax) lmax = p[t];
            }
            double z = 0.0;
            for (int t = 0; t <= last; ++t) {
                p[t] = exp(p[t] - lmax);
                z += p[t];
            }
            for (int i = 0; i < d; ++i) o[i] = 0.0;
            for (int t = 0; t <= last; ++t)
                for (int i = 0; i < d; ++i)
                    o[i] += (p[t] / z) * (double)oracle_f16_to_f32(V[((size_t)t * H + h) * d + i]);
            for (int i = 0; i < d; ++i)
                O[((size_t)s * H + h) * d + i] = oracle_f32_to_f16((float)o[i]);
        }
    free(p);
    free(o);
    return 0;
}

/* Residual update of the hidden state: x_k <- binary16(float(x_k) + float(delta_k)), [M, K] dense. */
int oracle_residual_add(uint16_t *X, const uint16_t *delta, int M, int K)
{
    if (M < 0 || K < 0) return -1;
    for (size_t j = 0; j < (size_t)M * (size_t)K; ++j)
        X[j] = oracle_f32_to_f16(oracle_f16_to_f32(X[j]) + oracle_f16_to_f32(delta[j]));
    return 0;
}
