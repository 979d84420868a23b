// Token selection kernels: retention score, top-k (Eq. 1 of the paper), the
// surviving row list and the row gather.
#include "common.h"

namespace sqap {

// Monotone map from a score to an unsigned key: larger score <=> larger key,
// -0 and +0 share a key, every NaN maps to 0 (below -inf, whose key is 0x007fffff).
__device__ __forceinline__ uint32_t score_key(float s)
{
    uint32_t b = __float_as_uint(s);
    if ((b & 0x7fffffffu) > 0x7f800000u) return 0u;
    if (b == 0x80000000u) b = 0u;
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

// Exclusive prefix sum of one 0/1 flag per thread over a 256-thread block.
// Returns the thread's offset; *total receives the block sum.  `wave_sums`
// is 4 ints of LDS.  Contains two barriers.
__device__ __forceinline__ int block_scan_flags(bool flag, int *wave_sums, int *total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    unsigned long long m = __ballot(flag);
    int before = __popcll(m & ((1ull << lane) - 1ull));
    __syncthreads();                       // previous users of wave_sums are done
    if (lane == 0) wave_sums[wave] = __popcll(m);
    __syncthreads();
    int off = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        int c = wave_sums[w];
        if (w < wave) off += c;
        tot += c;
    }
    *total = tot;
    return off + before;
}

constexpr int kTopkSmallMax = 2048;

// n <= 2048: every element counts how many rank ahead of it (larger key, or the
// same key at a lower index); it is kept iff that count is below keep_k.
// With rows_out the same launch also writes the surviving sequence rows (see
// kept_rows_kernel), saving a dependent launch.
__global__ __launch_bounds__(256) void topk_rank_kernel(const float *__restrict__ scores, int n,
                                                        int keep_k, int32_t *__restrict__ idx_out,
                                                        int seq_len, int vis_begin,
                                                        int32_t *__restrict__ rows_out)
{
    __shared__ __attribute__((aligned(16))) uint32_t keys[kTopkSmallMax];
    __shared__ uint8_t kept[kTopkSmallMax];
    __shared__ int wave_sums[4];
    const int t = threadIdx.x;
    const float *s = scores + (size_t)blockIdx.x * n;
    int32_t *out = idx_out + (size_t)blockIdx.x * keep_k;
    const int n4 = (n + 3) & ~3;
    for (int i = t; i < n4; i += 256) keys[i] = i < n ? score_key(s[i]) : 0u;
    __syncthreads();
    int base = 0;
    for (int c = 0; c < n; c += 256) {
        const int i = c + t;
        bool keep = false;
        if (i < n) {
            const uint32_t ki = keys[i];
            int ahead = 0;
            for (int j = 0; j < n4; j += 4) {
                uint4 kj = *reinterpret_cast<const uint4 *>(&keys[j]);
                ahead += (kj.x > ki) || (kj.x == ki && j + 0 < i);
                ahead += (kj.y > ki) || (kj.y == ki && j + 1 < i);
                ahead += (kj.z > ki) || (kj.z == ki && j + 2 < i);
                ahead += (kj.w > ki) || (kj.w == ki && j + 3 < i);
            }
            keep = ahead < keep_k;
            kept[i] = keep;
        }
        int total;
        int pos = block_scan_flags(keep, wave_sums, &total);
        if (keep) out[base + pos] = i;
        base += total;
    }
    if (rows_out) {
        int32_t *rows = rows_out + (size_t)blockIdx.x * (seq_len - n + keep_k);
        __syncthreads();
        base = 0;
        for (int c = 0; c < seq_len; c += 256) {
            const int sq = c + t, v = sq - vis_begin;
            const bool keep = sq < seq_len && (v < 0 || v >= n || kept[v]);
            int total;
            int pos = block_scan_flags(keep, wave_sums, &total);
            if (keep) rows[base + pos] = blockIdx.x * seq_len + sq;
            base += total;
        }
    }
}

// n <= 1024 and a sequence of at most 2048 positions: one wavefront per observation, no
// barriers and no LDS traffic in the ranking.  Lane l owns tokens l, l + 64, ...: tokens
// 64 r .. 64 r + 63 sit in lane order, so "lower index first" is "lower row, then lower lane".
// The keep_k-th largest key T is built bit by bit from the top (T is the largest value that at
// least keep_k keys reach) with wave ballots; keys above T are kept, and of the keys equal to T
// the first ones by index.  Outputs are compacted with ballot prefixes.  PL = tokens per lane.
template <int PL>
__global__ __launch_bounds__(64) void topk_wave_kernel(const float *__restrict__ scores, int n, int keep_k,
                                                       int32_t *__restrict__ idx_out, int seq_len, int vis_begin,
                                                       int32_t *__restrict__ rows_out)
{
    __shared__ uint8_t keptf[1024];
    const int lane = threadIdx.x, b = blockIdx.x;
    const float *s = scores + (size_t)b * n;
    const unsigned long long below = (1ull << lane) - 1ull;
    bool valid[PL], kept[PL];
    uint32_t key[PL];
#pragma unroll
    for (int r = 0; r < PL; ++r) {
        const int i = lane + 64 * r;
        valid[r] = i < n;
        key[r] = valid[r] ? score_key(s[i]) : 0u;
    }
    uint32_t T = 0;
    for (int bit = 31; bit >= 0; --bit) {
        const uint32_t cand = T | (1u << bit);
        int reach = 0;
#pragma unroll
        for (int r = 0; r < PL; ++r) reach += __popcll(__ballot(valid[r] && key[r] >= cand));
        if (reach >= keep_k) T = cand;
    }
    int above = 0;
#pragma unroll
    for (int r = 0; r < PL; ++r) above += __popcll(__ballot(valid[r] && key[r] > T));
    const int need_eq = keep_k - above;
    int32_t *out = idx_out + (size_t)b * keep_k;
    int eq_seen = 0, base = 0;
#pragma unroll
    for (int r = 0; r < PL; ++r) {
        const bool eq = valid[r] && key[r] == T;
        const unsigned long long me = __ballot(eq);
        kept[r] = valid[r] && (key[r] > T || (eq && eq_seen + __popcll(me & below) < need_eq));
        eq_seen += __popcll(me);
        const unsigned long long mk = __ballot(kept[r]);
        if (kept[r]) out[base + __popcll(mk & below)] = lane + 64 * r;
        base += __popcll(mk);
        if (rows_out && valid[r]) keptf[lane + 64 * r] = kept[r];
    }
    if (rows_out) {
        // LDS operations of one wavefront complete in order: the flags written above are visible
        __builtin_amdgcn_wave_barrier();
        int32_t *rows = rows_out + (size_t)b * (seq_len - n + keep_k);
        int rbase = 0;
        for (int c = 0; c < seq_len; c += 64) {
            const int sq = c + lane, v = sq - vis_begin;
            const bool keep = sq < seq_len && (v < 0 || v >= n || keptf[v]);
            const unsigned long long mk = __ballot(keep);
            if (keep) rows[rbase + __popcll(mk & below)] = b * seq_len + sq;
            rbase += __popcll(mk);
        }
    }
}

static bool launch_topk_wave(const float *scores, int batch, int n, int keep_k, int32_t *idx, int seq_len,
                             int vis_begin, int32_t *rows, hipStream_t st)
{
    if (n > 1024 || seq_len > 2048) return false;
    if (n <= 256)
        hipLaunchKernelGGL(topk_wave_kernel<4>, dim3(batch), dim3(64), 0, st, scores, n, keep_k, idx, seq_len,
                           vis_begin, rows);
    else if (n <= 512)
        hipLaunchKernelGGL(topk_wave_kernel<8>, dim3(batch), dim3(64), 0, st, scores, n, keep_k, idx, seq_len,
                           vis_begin, rows);
    else
        hipLaunchKernelGGL(topk_wave_kernel<16>, dim3(batch), dim3(64), 0, st, scores, n, keep_k, idx, seq_len,
                           vis_begin, rows);
    return true;
}

// Any n: radix select, 8 bits per pass from the top, finds the key T of the
// keep_k-th ranked element and how many elements equal to T are kept; a last
// pass in index order keeps key > T and the first `need_eq` with key == T.
__global__ __launch_bounds__(256) void topk_radix_kernel(const float *__restrict__ scores, int n,
                                                         int keep_k, int32_t *__restrict__ idx_out)
{
    __shared__ int hist[256];
    __shared__ int wave_sums[4];
    __shared__ int sel_digit, sel_remaining;
    const int t = threadIdx.x;
    const float *s = scores + (size_t)blockIdx.x * n;
    int32_t *out = idx_out + (size_t)blockIdx.x * keep_k;
    uint32_t prefix = 0, mask = 0;
    int remaining = keep_k;
    for (int shift = 24; shift >= 0; shift -= 8) {
        hist[t] = 0;
        __syncthreads();
        for (int i = t; i < n; i += 256) {
            uint32_t k = score_key(s[i]);
            if ((k & mask) == prefix) atomicAdd(&hist[(k >> shift) & 255u], 1);
        }
        __syncthreads();
        int above = 0;
        for (int d = t + 1; d < 256; ++d) above += hist[d];
        if (above < remaining && above + hist[t] >= remaining) {
            sel_digit = t;
            sel_remaining = remaining - above;
        }
        __syncthreads();
        prefix |= (uint32_t)sel_digit << shift;
        mask |= 0xffu << shift;
        remaining = sel_remaining;
        __syncthreads();
    }
    const uint32_t T = prefix;
    const int need_eq = remaining;
    int base = 0, eq_seen = 0;
    for (int c = 0; c < n; c += 256) {
        const int i = c + t;
        uint32_t k = i < n ? score_key(s[i]) : 0u;
        bool gt = i < n && k > T, eq = i < n && k == T;
        int eq_total;
        int eq_rank = eq_seen + block_scan_flags(eq, wave_sums, &eq_total);
        bool keep = gt || (eq && eq_rank < need_eq);
        int total;
        int pos = block_scan_flags(keep, wave_sums, &total);
        if (keep) out[base + pos] = i;
        base += total;
        eq_seen += eq_total;
    }
}

sqap_status launch_prune_topk(const float *scores, int batch, int n, int keep_k, int32_t *idx,
                              hipStream_t st)
{
    if (launch_topk_wave(scores, batch, n, keep_k, idx, 0, 0, nullptr, st)) {
    } else if (n <= kTopkSmallMax)
        hipLaunchKernelGGL(topk_rank_kernel, dim3(batch), dim3(256), 0, st, scores, n, keep_k, idx, 0, 0,
                           (int32_t *)nullptr);
    else
        hipLaunchKernelGGL(topk_radix_kernel, dim3(batch), dim3(256), 0, st, scores, n, keep_k, idx);
    SQAP_HIP_CHECK(hipGetLastError());
    return SQAP_OK;
}

sqap_status launch_kept_rows(const int32_t *idx, int batch, int keep_k, int seq_len,
                             int vis_begin, int n_vis, int32_t *rows, hipStream_t st);

// top-k and the surviving rows; one launch when the scores fit the rank kernel
sqap_status launch_prune_rows(const float *scores, int batch, int n, int keep_k, int seq_len, int vis_begin,
                              int32_t *idx, int32_t *rows, hipStream_t st)
{
    if (launch_topk_wave(scores, batch, n, keep_k, idx, seq_len, vis_begin, rows, st)) {
        SQAP_HIP_CHECK(hipGetLastError());
        return SQAP_OK;
    }
    if (n <= kTopkSmallMax) {
        hipLaunchKernelGGL(topk_rank_kernel, dim3(batch), dim3(256), 0, st, scores, n, keep_k, idx, seq_len,
                           vis_begin, rows);
        SQAP_HIP_CHECK(hipGetLastError());
        return SQAP_OK;
    }
    sqap_status stt = launch_prune_topk(scores, batch, n, keep_k, idx, st);
    if (stt != SQAP_OK) return stt;
    return launch_kept_rows(idx, batch, keep_k, seq_len, vis_begin, n, rows, st);
}

// ---------------------------------------------------------------------------
// Full selection rule of Section 3.2: K_attn (Eq. 1) + K_ring (Eq. 2-4) + K_fps
// (Eq. 5).  One wavefront per observation; lane l owns tokens l, l + 64, ...
// (at most 1024 tokens, 16 per lane).  Everything after the projection is
// integer work, so the result is exact.
constexpr int kSelectCamera = 26;          // doubles per observation: K (9), [R|t] (12), point (3), patch w, h
constexpr uint32_t kFarAway = 1u << 20;    // above any squared distance on a grid of <= 1024 tokens

// Eq. 2-3 in binary64, dot products summed left to right, no contraction.
__device__ __forceinline__ bool project_token(const double *c, int &tu, int &tv)
{
    const double *Km = c, *Rt = c + 9, *p = c + 21;
    double cam[3], h[3];
#pragma unroll
    for (int i = 0; i < 3; ++i)
        cam[i] = ((Rt[4 * i] * p[0] + Rt[4 * i + 1] * p[1]) + Rt[4 * i + 2] * p[2]) + Rt[4 * i + 3];
#pragma unroll
    for (int i = 0; i < 3; ++i) h[i] = (Km[3 * i] * cam[0] + Km[3 * i + 1] * cam[1]) + Km[3 * i + 2] * cam[2];
    if (!(h[2] > 0.0)) return false;
    const double fu = floor((h[0] / h[2]) / c[24]), fv = floor((h[1] / h[2]) / c[25]);
    if (!(fabs(fu) <= 1073741824.0) || !(fabs(fv) <= 1073741824.0)) return false;
    tu = (int)fu;
    tv = (int)fv;
    return true;
}

// Maximum over the 64 lanes, returned in every lane.  Row-shift steps fold each row of 16
// lanes into its lane 15, two row broadcasts fold the four rows into lane 63; lanes whose
// source does not exist take 0, the identity here.
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v)
{
#define SQAP_DPP_MAX(ctrl, row_mask, bank_mask)                                                      \
    {                                                                                                \
        const uint32_t o = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, ctrl, row_mask, bank_mask, false); \
        v = o > v ? o : v;                                                                           \
    }
    SQAP_DPP_MAX(0x111, 0xf, 0xf)    // row_shr:1
    SQAP_DPP_MAX(0x112, 0xf, 0xf)    // row_shr:2
    SQAP_DPP_MAX(0x114, 0xf, 0xe)    // row_shr:4, lanes 4-15 of a row
    SQAP_DPP_MAX(0x118, 0xf, 0xc)    // row_shr:8, lanes 8-15 of a row
    SQAP_DPP_MAX(0x142, 0xa, 0xf)    // lane 15 of rows 0 and 2 into rows 1 and 3
    SQAP_DPP_MAX(0x143, 0xc, 0xf)    // lane 31 into rows 2 and 3
#undef SQAP_DPP_MAX
    return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}

template <int PL>     // tokens per lane: at most 64 * PL tokens
__global__ __launch_bounds__(64) void prune_select_kernel(const float *__restrict__ scores, int gw, int gh,
                                                          int k_attn, int keep_total,
                                                          const double *__restrict__ camera, int radius,
                                                          int32_t *__restrict__ idx_out, int cap,
                                                          int32_t *__restrict__ count_out)
{
    const int lane = threadIdx.x, b = blockIdx.x;
    const int n = gw * gh;
    const float *s = scores + (size_t)b * n;
    const unsigned long long below = (1ull << lane) - 1ull;      // lanes with a lower number

    int cu = 0, cv = 0;
    bool have_ring = false;
    if (camera) have_ring = project_token(camera + (size_t)b * kSelectCamera, cu, cv);

    // own tokens: lane + 64 r.  Tokens 64 r .. 64 r + 63 sit in lane order, so "lower index
    // first" is "lower row first, then lower lane".
    bool valid[PL], kept[PL];
    uint32_t key[PL];
    int tu[PL], tv[PL];
#pragma unroll
    for (int r = 0; r < PL; ++r) {
        const int i = lane + 64 * r;
        valid[r] = i < n;
        key[r] = valid[r] ? score_key(s[i]) : 0u;
        tu[r] = valid[r] ? i % gw : 0;
        tv[r] = valid[r] ? i / gw : 0;
    }

    // Eq. 1: the k_attn-th largest key T, found bit by bit from the top (T is the largest value
    // that at least k_attn keys reach), then keys above T and the first tokens equal to T.
    uint32_t T = 0;
    for (int bit = 31; bit >= 0; --bit) {
        const uint32_t cand = T | (1u << bit);
        int reach = 0;
#pragma unroll
        for (int r = 0; r < PL; ++r) reach += __popcll(__ballot(valid[r] && key[r] >= cand));
        if (reach >= k_attn) T = cand;
    }
    int above = 0;
#pragma unroll
    for (int r = 0; r < PL; ++r) above += __popcll(__ballot(valid[r] && key[r] > T));
    const int need_eq = k_attn - above;          // (k_attn = 0 ends with T = all ones: nothing above, nothing needed)
    int eq_seen = 0;
#pragma unroll
    for (int r = 0; r < PL; ++r) {
        const bool eq = valid[r] && key[r] == T;
        const unsigned long long mk = __ballot(eq);
        bool keep = valid[r] && (key[r] > T || (eq && eq_seen + __popcll(mk & below) < need_eq));
        eq_seen += __popcll(mk);
        // Eq. 4 by the distance itself
        if (have_ring && valid[r]) {
            const int du = abs(tu[r] - cu), dv = abs(tv[r] - cv);
            keep = keep || (du > dv ? du : dv) <= radius;
        }
        kept[r] = keep;
    }
    int count = 0;
#pragma unroll
    for (int r = 0; r < PL; ++r) count += __popcll(__ballot(kept[r]));

    // Eq. 5: distance of every candidate to the set kept so far, then one pick per step
    const int m = keep_total > count ? keep_total - count : 0;
    uint32_t mind[PL];
#pragma unroll
    for (int r = 0; r < PL; ++r) mind[r] = kFarAway;
    if (m > 0) {
#pragma unroll
        for (int rr = 0; rr < PL; ++rr) {
            unsigned long long mk = __ballot(kept[rr]);     // kept tokens 64 rr .. 64 rr + 63, one at a time
            while (mk) {
                const int src = __builtin_ctzll(mk);
                mk &= mk - 1;
                const int ju = __builtin_amdgcn_readlane(tu[rr], src), jv = __builtin_amdgcn_readlane(tv[rr], src);
#pragma unroll
                for (int r = 0; r < PL; ++r) {
                    const int du = tu[r] - ju, dv = tv[r] - jv;
                    const uint32_t d = (uint32_t)(du * du + dv * dv);
                    mind[r] = d < mind[r] ? d : mind[r];
                }
            }
        }
    }
    for (int step = 0; step < m; ++step) {
        // largest distance, lowest index among equals: the index enters the key inverted
        uint32_t best = 0;
#pragma unroll
        for (int r = 0; r < PL; ++r) {
            const uint32_t k2 = (valid[r] && !kept[r]) ? (mind[r] << 11) + (uint32_t)(2047 - (lane + 64 * r)) : 0u;
            best = k2 > best ? k2 : best;
        }
        best = wave_max_u32(best);
        const int w = 2047 - (int)(best & 2047u);
        const int wl = w & 63, wr = w >> 6;
        int wu = 0, wv = 0;
#pragma unroll
        for (int r = 0; r < PL; ++r)
            if (r == wr) {                                   // uniform
                wu = __builtin_amdgcn_readlane(tu[r], wl);
                wv = __builtin_amdgcn_readlane(tv[r], wl);
            }
#pragma unroll
        for (int r = 0; r < PL; ++r) {
            if (lane + 64 * r == w) kept[r] = true;
            const int du = tu[r] - wu, dv = tv[r] - wv;
            const uint32_t d = (uint32_t)(du * du + dv * dv);
            mind[r] = d < mind[r] ? d : mind[r];
        }
    }

    // ascending output
    int32_t *out = idx_out + (size_t)b * cap;
    int base = 0;
#pragma unroll
    for (int r = 0; r < PL; ++r) {
        const unsigned long long mk = __ballot(kept[r]);
        if (kept[r]) out[base + __popcll(mk & below)] = lane + 64 * r;
        base += __popcll(mk);
    }
    for (int i = base + lane; i < cap; i += 64) out[i] = -1;
    if (count_out && lane == 0) count_out[b] = base;
}

sqap_status launch_prune_select(const float *scores, int batch, int gw, int gh, int k_attn, int keep_total,
                                const double *camera, int radius, int32_t *idx, int cap, int32_t *count,
                                hipStream_t st)
{
    const int n = gw * gh;
    if (n <= 256)
        hipLaunchKernelGGL(prune_select_kernel<4>, dim3(batch), dim3(64), 0, st, scores, gw, gh, k_attn, keep_total,
                           camera, radius, idx, cap, count);
    else if (n <= 512)
        hipLaunchKernelGGL(prune_select_kernel<8>, dim3(batch), dim3(64), 0, st, scores, gw, gh, k_attn, keep_total,
                           camera, radius, idx, cap, count);
    else
        hipLaunchKernelGGL(prune_select_kernel<16>, dim3(batch), dim3(64), 0, st, scores, gw, gh, k_attn,
                           keep_total, camera, radius, idx, cap, count);
    SQAP_HIP_CHECK(hipGetLastError());
    return SQAP_OK;
}

// One block per observation: walks the sequence in order, keeps every token
// outside the visual span and the visual tokens listed (ascending) in idx.
__global__ __launch_bounds__(256) void kept_rows_kernel(const int32_t *__restrict__ idx, int keep_k,
                                                        int seq_len, int vis_begin, int n_vis,
                                                        int32_t *__restrict__ rows)
{
    __shared__ int wave_sums[4];
    const int b = blockIdx.x, t = threadIdx.x;
    const int32_t *my = idx + (size_t)b * keep_k;
    int32_t *out = rows + (size_t)b * (seq_len - n_vis + keep_k);
    int base = 0;
    for (int c = 0; c < seq_len; c += 256) {
        const int s = c + t;
        bool keep = false;
        if (s < seq_len) {
            const int v = s - vis_begin;
            if (v < 0 || v >= n_vis) {
                keep = true;
            } else {                     // binary search in the ascending list
                int lo = 0, hi = keep_k;
                while (lo < hi) {
                    int mid = (lo + hi) >> 1;
                    if (my[mid] < v) lo = mid + 1; else hi = mid;
                }
                keep = lo < keep_k && my[lo] == v;
            }
        }
        int total;
        int pos = block_scan_flags(keep, wave_sums, &total);
        if (keep) out[base + pos] = b * seq_len + s;
        base += total;
    }
}

sqap_status launch_kept_rows(const int32_t *idx, int batch, int keep_k, int seq_len,
                             int vis_begin, int n_vis, int32_t *rows, hipStream_t st)
{
    hipLaunchKernelGGL(kept_rows_kernel, dim3(batch), dim3(256), 0, st, idx, keep_k, seq_len,
                       vis_begin, n_vis, rows);
    SQAP_HIP_CHECK(hipGetLastError());
    return SQAP_OK;
}

// out[i,:] = X[rows[i],:]; one 16-byte piece per thread, rows of a block contiguous.
__global__ __launch_bounds__(256) void gather_rows_kernel(const __half *__restrict__ X, int64_t ldx,
                                                          const int32_t *__restrict__ rows, int M,
                                                          int pieces, __half *__restrict__ out,
                                                          int64_t ldo)
{
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t row = gid / pieces;
    const int p = (int)(gid % pieces);
    if (row >= M) return;
    const uint4 *src = reinterpret_cast<const uint4 *>(X + (int64_t)rows[row] * ldx) + p;
    uint4 *dst = reinterpret_cast<uint4 *>(out + row * ldo) + p;
    *dst = *src;
}

sqap_status launch_gather_rows(const __half *X, int64_t ldx, const int32_t *rows, int M, int K,
                               __half *out, int64_t ldo, hipStream_t st)
{
    const int pieces = K / 8;
    const int64_t total = (int64_t)M * pieces;
    const int64_t blocks = (total + 255) / 256;
    if (blocks > 0x7fffffff) return fail(SQAP_EUNSUPPORTED, "sqap_gather_rows: too large");
    hipLaunchKernelGGL(gather_rows_kernel, dim3((unsigned)blocks), dim3(256), 0, st, X, ldx, rows, M,
                       pieces, out, ldo);
    SQAP_HIP_CHECK(hipGetLastError());
    return SQAP_OK;
}

// Retention score.  One block of 8 wavefronts; wavefront w takes heads w, w+8, ...
// For its head every lane owns keys lane, lane+64, ...: pass 1 builds the
// running (max, sum) of the softmax, pass 2 recomputes the logits of the
// visual span and turns them into weights.  Heads are then added into the
// LDS accumulator in wavefront order, so the sum order is fixed.
__device__ __forceinline__ float dot_qk(const __half *__restrict__ qh, const __half *__restrict__ kh, int d)
{
    float acc = 0.f;
    for (int i = 0; i < d; i += 2) {
        float2 a = __half22float2(*reinterpret_cast<const __half2 *>(qh + i));
        float2 b = __half22float2(*reinterpret_cast<const __half2 *>(kh + i));
        acc = fmaf(a.x, b.x, acc);
        acc = fmaf(a.y, b.y, acc);
    }
    return acc;
}

constexpr int kScoreWaves = 8;

__global__ __launch_bounds__(64 * kScoreWaves) void attn_scores_kernel(
    const __half *__restrict__ q, const __half *__restrict__ k, int S, int H, int d, int vis_begin,
    int n_vis, float *__restrict__ scores)
{
    extern __shared__ float acc_lds[];   // n_vis floats
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int j = threadIdx.x; j < n_vis; j += blockDim.x) acc_lds[j] = 0.f;
    __syncthreads();
    const float inv_sqrt_d = 1.0f / sqrtf((float)d);
    const int rounds = (H + kScoreWaves - 1) / kScoreWaves;
    for (int r = 0; r < rounds; ++r) {
        const int h = r * kScoreWaves + wave;
        float m = -INFINITY, z = 0.f;
        if (h < H) {
            const __half *qh = q + (size_t)h * d;
            for (int s = lane; s < S; s += 64) {
                float l = dot_qk(qh, k + ((size_t)s * H + h) * d, d) * inv_sqrt_d;
                float mn = fmaxf(m, l);
                z = z * expf(m - mn) + expf(l - mn);
                m = mn;
            }
            for (int o = 32; o > 0; o >>= 1) {
                float m2 = __shfl_xor(m, o), z2 = __shfl_xor(z, o);
                float mn = fmaxf(m, m2);
                float za = (m == -INFINITY) ? 0.f : z * expf(m - mn);
                float zb = (m2 == -INFINITY) ? 0.f : z2 * expf(m2 - mn);
                z = za + zb;
                m = mn;
            }
        }
        // add this round's heads in wavefront order
        for (int w = 0; w < kScoreWaves; ++w) {
            if (w == wave && h < H) {
                const __half *qh = q + (size_t)h * d;
                for (int j = lane; j < n_vis; j += 64) {
                    const int s = vis_begin + j;
                    float l = dot_qk(qh, k + ((size_t)s * H + h) * d, d) * inv_sqrt_d;
                    acc_lds[j] += expf(l - m) / z;
                }
            }
            __syncthreads();
        }
    }
    for (int j = threadIdx.x; j < n_vis; j += blockDim.x) scores[j] = acc_lds[j] / (float)H;
}

// Fast path of the retention score: one workgroup per head.  A group of d/8 lanes reads one
// key row piece (16 bytes per lane: a coalesced run of 2d bytes), the logits of the head go to
// LDS, the workgroup takes their maximum and the sum of exponentials, and writes the head's
// softmax weights of the visual span to the workspace.  The workgroup that finishes last (a
// counter in the workspace tells) adds the heads in head order, so the result does not depend on
// the order in which the workgroups ran, and puts the counter back to zero.
// A batch of observations runs as one launch (grid: heads x observations); each observation has
// its own counter and its own piece of the weight array.
// Workspace: [batch counters, one 256-byte line each (atomics on one line serialise)]
//            [batch * H * n_vis floats].
constexpr int kScoreMaxSeq = 4096;                // logits of one head sit in LDS
constexpr int kCounterStride = 64;                // 32-bit words per counter line
static size_t score_counter_bytes(int batch) { return (size_t)batch * kCounterStride * sizeof(unsigned int); }

__device__ __forceinline__ float block_reduce_256(float v, bool take_max, float *scratch4)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int o = 32; o > 0; o >>= 1) {
        const float u = __shfl_xor(v, o);
        v = take_max ? fmaxf(v, u) : v + u;
    }
    __syncthreads();                              // previous users of scratch4 are done
    if (lane == 0) scratch4[wave] = v;
    __syncthreads();
    return take_max ? fmaxf(fmaxf(scratch4[0], scratch4[1]), fmaxf(scratch4[2], scratch4[3]))
                    : (scratch4[0] + scratch4[1]) + (scratch4[2] + scratch4[3]);
}

__global__ __launch_bounds__(256) void attn_head_kernel(const __half *__restrict__ q, const __half *__restrict__ k,
                                                        int S, int H, int d, int vis_begin, int n_vis,
                                                        float *__restrict__ scores, unsigned int *heads_done,
                                                        float *all_head_weights)
{
    __shared__ float logits[kScoreMaxSeq];
    __shared__ float red[4];
    __shared__ bool is_last;
    const int t = threadIdx.x, h = blockIdx.x, b = blockIdx.y;
    q += (size_t)b * H * d;
    k += (size_t)b * S * H * d;
    scores += (size_t)b * n_vis;
    float *head_weights = all_head_weights + (size_t)b * H * n_vis;
    const int lp = d >> 3;                        // lanes per key row: a power of two, 1 .. 32
    const int sub = t & (lp - 1), grp = t / lp, groups = 256 / lp;
    float qf[8];
    {
        const uint4 raw = *reinterpret_cast<const uint4 *>(q + (size_t)h * d + sub * 8);
        const __half2 *h2 = reinterpret_cast<const __half2 *>(&raw);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float2 f = __half22float2(h2[i]);
            qf[2 * i] = f.x;
            qf[2 * i + 1] = f.y;
        }
    }
    const float inv_sqrt_d = 1.0f / sqrtf((float)d);
    constexpr int kRowsInFlight = 8;              // key rows a lane group loads before it reduces any
    for (int s0 = 0; s0 < S; s0 += groups * kRowsInFlight) {
        uint4 raw[kRowsInFlight];
#pragma unroll
        for (int r = 0; r < kRowsInFlight; ++r) {
            const int s = s0 + r * groups + grp;
            raw[r] = make_uint4(0u, 0u, 0u, 0u);
            if (s < S) raw[r] = *reinterpret_cast<const uint4 *>(k + ((size_t)s * H + h) * d + sub * 8);
        }
#pragma unroll
        for (int r = 0; r < kRowsInFlight; ++r) {
            const int s = s0 + r * groups + grp;
            const __half2 *h2 = reinterpret_cast<const __half2 *>(&raw[r]);
            float acc = 0.f;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float2 f = __half22float2(h2[i]);
                acc = fmaf(qf[2 * i], f.x, acc);
                acc = fmaf(qf[2 * i + 1], f.y, acc);
            }
            for (int o = lp >> 1; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
            if (s < S && sub == 0) logits[s] = acc * inv_sqrt_d;
        }
    }
    __syncthreads();
    float m = -INFINITY;
    for (int s = t; s < S; s += 256) m = fmaxf(m, logits[s]);
    m = block_reduce_256(m, true, red);
    float z = 0.f;
    for (int s = t; s < S; s += 256) z += expf(logits[s] - m);
    z = block_reduce_256(z, false, red);
    // The weights go out as agent-scope stores (written through this XCD's L2, since the workgroup that
    // adds the heads may sit behind another one); they are complete once the vector-memory counter
    // drains, and only then does the workgroup count itself as done.  A full release fence here would
    // write back the whole L2 once per workgroup.
    for (int j = t; j < n_vis; j += 256)
        __hip_atomic_store(&head_weights[(size_t)h * n_vis + j], expf(logits[vis_begin + j] - m) / z, __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (t == 0) {
        const unsigned done = __hip_atomic_fetch_add(&heads_done[b * kCounterStride], 1u, __ATOMIC_RELAXED,
                                                     __HIP_MEMORY_SCOPE_AGENT);
        is_last = done + 1 == (unsigned)H;
        if (is_last)                              // ready for the next call
            __hip_atomic_store(&heads_done[b * kCounterStride], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    if (is_last) {
        // agent-scope loads: they do not hit stale lines of an earlier call in this XCD's caches
        for (int j = t; j < n_vis; j += 256) {
            float a = 0.f;
#pragma unroll 16
            for (int hh = 0; hh < H; ++hh)
                a += __hip_atomic_load(&head_weights[(size_t)hh * n_vis + j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            scores[j] = a / (float)H;
        }
    }
}

// The fast path needs a power-of-two head size of 8 .. 256, 16-byte aligned operands and a sequence
// whose logits fit LDS; everything else takes the one-workgroup kernel, which needs no workspace.
static bool score_fast_path(const void *q, const void *k, int S, int d)
{
    const bool pow2 = (d & (d - 1)) == 0;
    const bool aligned = ((reinterpret_cast<uintptr_t>(q) | reinterpret_cast<uintptr_t>(k)) & 15u) == 0;
    return pow2 && d >= 8 && d <= 256 && aligned && S <= kScoreMaxSeq;
}

size_t attn_scores_workspace_bytes(int batch, int H, int n_vis)
{
    if (batch <= 0 || H <= 0 || n_vis <= 0) return 0;
    return score_counter_bytes(batch) + (size_t)batch * H * n_vis * sizeof(float);
}

sqap_status launch_attn_scores(const __half *q, const __half *k, int batch, int S, int H, int d,
                               int vis_begin, int n_vis, float *scores, void *workspace, size_t workspace_bytes,
                               hipStream_t st)
{
    if (score_fast_path(q, k, S, d) && workspace && workspace_bytes >= attn_scores_workspace_bytes(batch, H, n_vis)) {
        unsigned int *counters = reinterpret_cast<unsigned int *>(workspace);
        float *weights = reinterpret_cast<float *>(reinterpret_cast<uint8_t *>(workspace) + score_counter_bytes(batch));
        hipLaunchKernelGGL(attn_head_kernel, dim3(H, batch), dim3(256), 0, st, q, k, S, H, d, vis_begin, n_vis, scores,
                           counters, weights);
    } else {
        for (int b = 0; b < batch; ++b)
            hipLaunchKernelGGL(attn_scores_kernel, dim3(1), dim3(64 * kScoreWaves), n_vis * sizeof(float), st,
                               q + (size_t)b * H * d, k + (size_t)b * S * H * d, S, H, d, vis_begin, n_vis,
                               scores + (size_t)b * n_vis);
    }
    SQAP_HIP_CHECK(hipGetLastError());
    return SQAP_OK;
}

// ---------------------------------------------------------------------------------------------
// The retention score for callers that cannot allocate (a stream under graph capture, a serving loop
// that forbids hipMalloc): the workspace of the fast kernel is this file-scope device array instead of
// a caller's buffer.  Layout as above: kNoAllocMaxBatch counter lines, then the per-head weights.
// The array's name is only a host-side handle: the device address is looked up once per device with
// hipGetSymbolAddress (each device holds its own copy of the array at its own address) and host code
// uses that address from then on.  The array is zero when the code object is loaded; what must be zero
// at the start of a call (the counters) is put back to zero by the workgroup that finishes last, so
// every call that runs to its end leaves the array ready for the next one.
constexpr int kNoAllocMaxBatch = 64;
constexpr size_t kNoAllocMaxWeights = 512 * 1024;                  // batch * H * n_vis floats: 2 MiB
constexpr size_t kNoAllocCounterBytes = (size_t)kNoAllocMaxBatch * kCounterStride * sizeof(unsigned int);
constexpr size_t kNoAllocScratchBytes = kNoAllocCounterBytes + kNoAllocMaxWeights * sizeof(float);
static __device__ __align__(256) unsigned char scratch[kNoAllocScratchBytes];

static std::atomic<void *> g_scratch_of_device[kMaxDeviceSlots];

// Device address of `scratch` on the current device (looked up on the first call per device).
sqap_status noalloc_scratch(void **out)
{
    int dev = 0;
    SQAP_HIP_CHECK(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDeviceSlots)
        return fail(SQAP_EUNSUPPORTED, "device ordinal %d above %d", dev, kMaxDeviceSlots - 1);
    void *ptr = g_scratch_of_device[dev].load(std::memory_order_acquire);
    if (!ptr) {
        SQAP_HIP_CHECK(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) return fail(SQAP_EDEVICE, "hipGetSymbolAddress gave a null address for the scratch array");
        g_scratch_of_device[dev].store(ptr, std::memory_order_release);      // racing host threads store the same value
    }
    *out = ptr;
    return SQAP_OK;
}

size_t noalloc_max_weights() { return kNoAllocMaxWeights; }
int noalloc_max_batch() { return kNoAllocMaxBatch; }

sqap_status launch_attn_scores_noalloc(const __half *q, const __half *k, int batch, int S, int H, int d,
                                       int vis_begin, int n_vis, float *scores, hipStream_t st)
{
    if (!score_fast_path(q, k, S, d))       // the one-workgroup kernel uses no scratch memory at all
        return launch_attn_scores(q, k, batch, S, H, d, vis_begin, n_vis, scores, nullptr, 0, st);
    void *ptr = nullptr;
    sqap_status s = noalloc_scratch(&ptr);
    if (s != SQAP_OK) return s;
    // The kernel sees the array split as [batch counter lines][weights]; the weights start behind the
    // counter lines of THIS call's batch, which all lie inside the kNoAllocMaxBatch lines that are kept zero.
    unsigned int *counters = reinterpret_cast<unsigned int *>(ptr);
    float *weights = reinterpret_cast<float *>(reinterpret_cast<uint8_t *>(ptr) + kNoAllocCounterBytes);
    hipLaunchKernelGGL(attn_head_kernel, dim3(H, batch), dim3(256), 0, st, q, k, S, H, d, vis_begin, n_vis, scores,
                       counters, weights);
    SQAP_HIP_CHECK(hipGetLastError());
    return SQAP_OK;
}

}  // namespace sqap
