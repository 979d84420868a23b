// Decoder glue between the W4A4 linears of a Llama-shaped layer: rotary position embedding,
// causal softmax attention over a short prefix, residual add.  (RMSNorm and the SwiGLU gate are
// fused into the activation quantizer, quantize.hip.)  The paper does not restate the decoder;
// these follow the published architecture (Su et al. 2021 in the half-split pairing used by
// Llama; Vaswani et al. 2017).  Sequences here are a few hundred tokens (276 before pruning, 148
// after), so attention is a small fraction of a layer and is written for low latency, not for
// matrix-core throughput: binary32 FMAs over LDS tiles with an online softmax.
#include "common.h"
#include "quant_math.h"
#include "decode_attn.h"

namespace sqap {

// v'_i = v_i cos a - v_{i+d/2} sin a,  v'_{i+d/2} = v_{i+d/2} cos a + v_i sin a,
// a = pos * base^(-2i/d); angle, sine and cosine in binary64, products in binary64, one rounding
// to half.  One thread per (token, head, i); consecutive threads take consecutive i.
__global__ __launch_bounds__(256) void rope_kernel(__half *__restrict__ X, int64_t ld, const int32_t *__restrict__ pos,
                                                   int S, int H, int d, double base, const RopeFreq freq)
{
    const int half_d = d >> 1;
    const int64_t total = (int64_t)S * H * half_d;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int i = (int)(idx % half_d);
    const int64_t sh = idx / half_d;
    const int h = (int)(sh % H);
    const int s = (int)(sh / H);
    __half *v = X + (int64_t)s * ld + (int64_t)h * d;
    const double a = rope_angle(freq, pos[s], i, d, base);
    double sn, cs;
    sincos(a, &sn, &cs);
    const double lo = (double)__half2float(v[i]), hi = (double)__half2float(v[i + half_d]);
    v[i] = __float2half_rn((float)(lo * cs - hi * sn));
    v[i + half_d] = __float2half_rn((float)(hi * cs + lo * sn));
}

// Rotary embedding of a fused q|k|v row block with the key/value cache append folded in: queries are rotated
// in place, keys are rotated on their way into the cache row (the copy in the q|k|v buffer stays as it was),
// values are copied.  Same arithmetic as rope_kernel; one launch instead of a rotation and a row copy.
// One thread per (token, head-or-value slot, i): slots 0 .. H-1 queries, H .. 2H-1 keys, 2H .. 3H-1 values.
__global__ __launch_bounds__(256) void rope_append_kernel(__half *__restrict__ QKV, int64_t ld,
                                                          const int32_t *__restrict__ pos, int S, int H, int d,
                                                          double base, __half *__restrict__ KV, int64_t ldkv, const RopeFreq freq)
{
    const int half_d = d >> 1;
    const int64_t total = (int64_t)S * 3 * H * half_d;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int i = (int)(idx % half_d);
    const int64_t sh = idx / half_d;
    const int slot = (int)(sh % (3 * H));
    const int s = (int)(sh / (3 * H));
    const __half *src = QKV + (int64_t)s * ld + (int64_t)slot * d;
    if (slot >= 2 * H) {                                      // value: plain copy of the pair
        __half *dst = KV + (int64_t)s * ldkv + (int64_t)(slot - H) * d;
        dst[i] = src[i];
        dst[i + half_d] = src[i + half_d];
        return;
    }
    const double a = rope_angle(freq, pos[s], i, d, base);
    double sn, cs;
    sincos(a, &sn, &cs);
    const double lo = (double)__half2float(src[i]), hi = (double)__half2float(src[i + half_d]);
    const __half r0 = __float2half_rn((float)(lo * cs - hi * sn));
    const __half r1 = __float2half_rn((float)(hi * cs + lo * sn));
    __half *dst = slot < H ? QKV + (int64_t)s * ld + (int64_t)slot * d : KV + (int64_t)s * ldkv + (int64_t)(slot - H) * d;
    dst[i] = r0;
    dst[i + half_d] = r1;
}

sqap_status launch_rope_append(__half *QKV, int64_t ld, const int32_t *pos, int S, int H, int d, double base,
                               __half *KV, int64_t ldkv, hipStream_t st)
{
    const int64_t total = (int64_t)S * 3 * H * (d / 2);
    if (total == 0) return SQAP_OK;
    hipLaunchKernelGGL(rope_append_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, QKV, ld, pos, S, H, d,
                       base, KV, ldkv, rope_frequencies(d, base));
    SQAP_HIP_CHECK(hipGetLastError());
    return SQAP_OK;
}

// The same for many tokens: one workgroup per token evaluates the d/2 angles of its position once (the
// binary64 power, sine and cosine are a few hundred instructions per pair) and shares them between the
// heads through LDS.  With few tokens the per-pair kernel is faster (more threads in flight: 6.7 against
// 8.8 us at 84 tokens); at 2368 tokens this one takes a tenth of its time.
constexpr int kRopeMaxHalfD = 256;
constexpr int kRopeTokenKernelFrom = 512;        // tokens

__global__ __launch_bounds__(256) void rope_token_kernel(__half *__restrict__ X, int64_t ld,
                                                         const int32_t *__restrict__ pos, int H, int d, double base,
                                                         const RopeFreq freq)
{
    __shared__ double cs[kRopeMaxHalfD], sn[kRopeMaxHalfD];
    const int half_d = d >> 1, s = blockIdx.x;
    for (int i = threadIdx.x; i < half_d; i += 256) {
        const double a = rope_angle(freq, pos[s], i, d, base);
        double sv, cv;
        sincos(a, &sv, &cv);
        sn[i] = sv;
        cs[i] = cv;
    }
    __syncthreads();
    __half *row = X + (int64_t)s * ld;
    for (int idx = threadIdx.x; idx < H * half_d; idx += 256) {
        const int h = idx / half_d, i = idx - h * half_d;
        __half *v = row + (int64_t)h * d;
        const double lo = (double)__half2float(v[i]), hi = (double)__half2float(v[i + half_d]);
        v[i] = __float2half_rn((float)(lo * cs[i] - hi * sn[i]));
        v[i + half_d] = __float2half_rn((float)(hi * cs[i] + lo * sn[i]));
    }
}

sqap_status launch_rope(__half *X, int64_t ld, const int32_t *pos, int S, int H, int d, double base, hipStream_t st)
{
    const int64_t total = (int64_t)S * H * (d / 2);
    if (total == 0) return SQAP_OK;
    if (S >= kRopeTokenKernelFrom && d / 2 <= kRopeMaxHalfD) {
        hipLaunchKernelGGL(rope_token_kernel, dim3(S), dim3(256), 0, st, X, ld, pos, H, d, base, rope_frequencies(d, base));
        SQAP_HIP_CHECK(hipGetLastError());
        return SQAP_OK;
    }
    hipLaunchKernelGGL(rope_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, X, ld, pos, S, H, d, base,
                       rope_frequencies(d, base));
    SQAP_HIP_CHECK(hipGetLastError());
    return SQAP_OK;
}

// Causal attention.  Query i (of Sq) sits at sequence position Sk - Sq + i and sees keys 0 ..
// Sk - Sq + i.  A batch of sequences is a stack of row blocks (Sq rows of Q and O, Sk rows of K
// and V per sequence).  This scalar form serves the small head sizes (16 and 32): one workgroup per
// (head, block of 32 queries, sequence); keys and values pass through LDS in tiles of 64.  Thread t
// works for query t/8: in the score phase on keys 8(t%8) .. +7 of the tile, in the output phase on
// the D/8 consecutive head-dimension columns from (t%8) D/8 on.  Running maximum m, running sum l
// and the output row are rescaled when a tile raises the maximum (the usual online softmax); all in
// binary32.
constexpr int kAttQ = 32, kAttK = 64;

template <int D>
__global__ __launch_bounds__(256) void attention_kernel(const __half *__restrict__ Q, int64_t ldq,
                                                        const __half *__restrict__ Kc, int64_t ldk,
                                                        const __half *__restrict__ V, int64_t ldv, int Sq, int Sk,
                                                        int H, __half *__restrict__ O, int64_t ldo)
{
    constexpr int PITCH = D + 8;                 // halves per LDS row: keeps 16-byte alignment, staggers the banks
    constexpr int CPT = D / 8;                   // output columns per thread
    __shared__ __attribute__((aligned(16))) __half qs[kAttQ * PITCH];
    __shared__ __attribute__((aligned(16))) __half ks[kAttK * PITCH];
    __shared__ __attribute__((aligned(16))) __half vs[kAttK * PITCH];
    __shared__ float ps[kAttQ * (kAttK + 1)];
    const int t = threadIdx.x, h = blockIdx.x, q0 = blockIdx.y * kAttQ;
    const int qi = t >> 3, sub = t & 7;
    Q += (int64_t)blockIdx.z * Sq * ldq;
    O += (int64_t)blockIdx.z * Sq * ldo;
    Kc += (int64_t)blockIdx.z * Sk * ldk;
    V += (int64_t)blockIdx.z * Sk * ldv;
    const int shift = Sk - Sq;                   // query i sees keys <= i + shift
    const float inv_sqrt_d = 1.0f / sqrtf((float)D);

    for (int u = t; u < kAttQ * (D / 8); u += 256) {
        const int r = u / (D / 8), c = u % (D / 8);
        uint4 raw = make_uint4(0u, 0u, 0u, 0u);
        if (q0 + r < Sq) raw = *reinterpret_cast<const uint4 *>(Q + (int64_t)(q0 + r) * ldq + (int64_t)h * D + c * 8);
        *reinterpret_cast<uint4 *>(qs + r * PITCH + c * 8) = raw;
    }
    float o[CPT];
#pragma unroll
    for (int c = 0; c < CPT; ++c) o[c] = 0.f;
    float m = -INFINITY, l = 0.f;
    const int my_q = q0 + qi;
    const int last_key = min(Sk - 1, min(q0 + kAttQ - 1, Sq - 1) + shift);      // of the whole block
    for (int k0 = 0; k0 <= last_key; k0 += kAttK) {
        __syncthreads();                                                        // previous tile consumed (and qs written)
        for (int u = t; u < kAttK * (D / 8); u += 256) {
            const int r = u / (D / 8), c = u % (D / 8);
            uint4 kr = make_uint4(0u, 0u, 0u, 0u), vr = kr;
            if (k0 + r < Sk) {
                kr = *reinterpret_cast<const uint4 *>(Kc + (int64_t)(k0 + r) * ldk + (int64_t)h * D + c * 8);
                vr = *reinterpret_cast<const uint4 *>(V + (int64_t)(k0 + r) * ldv + (int64_t)h * D + c * 8);
            }
            *reinterpret_cast<uint4 *>(ks + r * PITCH + c * 8) = kr;
            *reinterpret_cast<uint4 *>(vs + r * PITCH + c * 8) = vr;
        }
        __syncthreads();
        // scores of this thread's 8 keys
        float sc[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) sc[j] = 0.f;
        for (int c = 0; c < D; c += 8) {
            const uint4 qraw = *reinterpret_cast<const uint4 *>(qs + qi * PITCH + c);
            const __half2 *q2 = reinterpret_cast<const __half2 *>(&qraw);
            float qf[8];
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const float2 f = __half22float2(q2[p]);
                qf[2 * p] = f.x;
                qf[2 * p + 1] = f.y;
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const uint4 kraw = *reinterpret_cast<const uint4 *>(ks + (sub * 8 + j) * PITCH + c);
                const __half2 *k2 = reinterpret_cast<const __half2 *>(&kraw);
#pragma unroll
                for (int p = 0; p < 4; ++p) {
                    const float2 f = __half22float2(k2[p]);
                    sc[j] = fmaf(qf[2 * p], f.x, sc[j]);
                    sc[j] = fmaf(qf[2 * p + 1], f.y, sc[j]);
                }
            }
        }
        float tile_max = -INFINITY;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int key = k0 + sub * 8 + j;
            const bool seen = key < Sk && key <= my_q + shift && my_q < Sq;
            sc[j] = seen ? sc[j] * inv_sqrt_d : -INFINITY;
            tile_max = fmaxf(tile_max, sc[j]);
        }
        for (int x = 1; x < 8; x <<= 1) tile_max = fmaxf(tile_max, __shfl_xor(tile_max, x));
        const float m_new = fmaxf(m, tile_max);
        // a query that has seen no key yet keeps m = -inf; exp(-inf - -inf) is avoided
        const float rescale = m_new == -INFINITY ? 1.f : expf(m - m_new);
        float tile_sum = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float pj = sc[j] == -INFINITY ? 0.f : expf(sc[j] - m_new);
            ps[qi * (kAttK + 1) + sub * 8 + j] = pj;
            tile_sum += pj;
        }
        for (int x = 1; x < 8; x <<= 1) tile_sum += __shfl_xor(tile_sum, x);
        l = l * rescale + tile_sum;
        m = m_new;
        __syncthreads();                                                        // ps complete
#pragma unroll
        for (int c = 0; c < CPT; ++c) o[c] *= rescale;
        const int kmax = min(kAttK, Sk - k0);
        for (int j = 0; j < kmax; ++j) {
            const float pj = ps[qi * (kAttK + 1) + j];
            const __half *vrow = vs + j * PITCH + sub * CPT;
#pragma unroll
            for (int c = 0; c < CPT; c += 2) {
                const float2 f = __half22float2(*reinterpret_cast<const __half2 *>(vrow + c));
                o[c] = fmaf(pj, f.x, o[c]);
                o[c + 1] = fmaf(pj, f.y, o[c + 1]);
            }
        }
    }
    if (my_q < Sq) {
        __half *dst = O + (int64_t)my_q * ldo + (int64_t)h * D + sub * CPT;
        const float inv_l = 1.0f / l;
#pragma unroll
        for (int c = 0; c < CPT; c += 2)
            *reinterpret_cast<__half2 *>(dst + c) = __floats2half2_rn(o[c] * inv_l, o[c + 1] * inv_l);
    }
}

// The same attention on the matrix cores, for head sizes 64 and 128: one workgroup of four wavefronts per
// (head, block of 32 queries, sequence), key tiles of 32.  Everything is kept transposed so that no
// accumulator ever has to change lanes:
//   S^T = K Q^T      v_mfma_f32_32x32x8_f16 with A = key rows, B = query rows: lane l holds query l%32,
//                    register i key 8(i/4) + 4(l/32) + i%4 of the tile;
//   softmax          over registers and the two lane halves (one cross-lane exchange);
//   O^T += V^T P^T   registers 4b .. 4b+3 of exp(S^T - m), converted to half, ARE the B operand of key
//                    block b (keys 8b + 4(l/32) + 0..3); A = V^T is read column-wise (2 bytes at a time)
//                    from the value tile in LDS.
// The running maximum, the running sum and the rescaling of O^T are per query, i.e. per lane.  The four
// wavefronts take the key tiles in turn (tile t belongs to wavefront t % 4), so a sequence of up to 128
// keys costs one round of loads, and merge their partial (m, l, O^T) through LDS at the end: wavefront w
// collects column tile w of the output from the other three.  The reduction over the head dimension may
// visit it in any order as long as A and B agree: MFMA j takes elements 16(j/2) + 8(l/32) + 4(j%2) + 0..3,
// so that each lane fetches 16 contiguous bytes per pair of MFMAs.
typedef _Float16 v4h __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int kAttWaves = 4;

template <int D>
__global__ __launch_bounds__(64 * kAttWaves) void attention_mfma_kernel(const __half *__restrict__ Q, int64_t ldq,
                                                            const __half *__restrict__ Kc, int64_t ldk,
                                                            const __half *__restrict__ V, int64_t ldv, int Sq, int Sk,
                                                            int H, __half *__restrict__ O, int64_t ldo)
{
    constexpr int NP = D / 16;                   // 16-byte pieces of a head row per lane half
    constexpr int CT = D / 32;                   // 32-column tiles of the head dimension
    constexpr int VP = D + 8;                    // halves per key row of the value tile in LDS (16-byte aligned, banks staggered)
    constexpr int NW = kAttWaves;
    constexpr int VT_BYTES = NW * 32 * VP * 2;
    constexpr int MERGE_BYTES = CT * NW * 4096 + NW * 64 * 8;      // O^T pieces [ct][wave][16 regs][64 lanes] + (m, l)
    __shared__ __attribute__((aligned(16))) uint8_t lds[VT_BYTES > MERGE_BYTES ? VT_BYTES : MERGE_BYTES];
    const int l = threadIdx.x & 63, c = l & 31, h = l >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    __half *vt = reinterpret_cast<__half *>(lds) + wave * (32 * VP);
    const int head = blockIdx.x, q0 = blockIdx.y * 32;
    Q += (int64_t)blockIdx.z * Sq * ldq + (int64_t)head * D;
    O += (int64_t)blockIdx.z * Sq * ldo + (int64_t)head * D;
    Kc += (int64_t)blockIdx.z * Sk * ldk + (int64_t)head * D;
    V += (int64_t)blockIdx.z * Sk * ldv + (int64_t)head * D;
    const int shift = Sk - Sq;
    const int my_q = q0 + c;
    const bool q_ok = my_q < Sq;
    // scores are kept in units of ln 2, so that the exponentials are single v_exp_f32 instructions
    const float inv_sqrt_d = 1.4426950408889634f / sqrtf((float)D);
    union Piece { uint4 u; v4h v[2]; };

    Piece qf[NP];
#pragma unroll
    for (int m = 0; m < NP; ++m) {
        qf[m].u = make_uint4(0u, 0u, 0u, 0u);
        if (q_ok) qf[m].u = *reinterpret_cast<const uint4 *>(Q + (int64_t)my_q * ldq + 16 * m + 8 * h);
    }
    v16f ot[CT];
#pragma unroll
    for (int ct = 0; ct < CT; ++ct)
#pragma unroll
        for (int i = 0; i < 16; ++i) ot[ct][i] = 0.f;
    float mrun = -INFINITY, lrun = 0.f;
    const int last_key = min(Sk - 1, min(q0 + 31, Sq - 1) + shift);
    const int n_tiles = last_key / 32 + 1;

    Piece kf[NP];
    auto load_keys = [&](int k0) {
        const int key = k0 + c;
#pragma unroll
        for (int m = 0; m < NP; ++m) {
            kf[m].u = make_uint4(0u, 0u, 0u, 0u);
            if (key < Sk) kf[m].u = *reinterpret_cast<const uint4 *>(Kc + (int64_t)key * ldk + 16 * m + 8 * h);
        }
    };
    // keys and values of the next tile are asked for while the current one is worked on: these rows were
    // just written by another kernel and come from memory, two microseconds away
    uint4 vraw[D / 16];
    auto load_values = [&](int k0) {
#pragma unroll
        for (int n = 0; n < D / 16; ++n) {
            const int u = l + 64 * n, key = u / (D / 8), dp = u % (D / 8);
            vraw[n] = make_uint4(0u, 0u, 0u, 0u);
            if (k0 + key < Sk) vraw[n] = *reinterpret_cast<const uint4 *>(V + (int64_t)(k0 + key) * ldv + dp * 8);
        }
    };
    if (wave < n_tiles) {
        load_keys(wave * 32);
        load_values(wave * 32);
    }
    for (int kt = wave; kt < n_tiles; kt += NW) {
        const int k0 = kt * 32;
        v16f st;
#pragma unroll
        for (int i = 0; i < 16; ++i) st[i] = 0.f;
#pragma unroll
        for (int m = 0; m < NP; ++m) {
            st = __builtin_amdgcn_mfma_f32_32x32x8f16(kf[m].v[0], qf[m].v[0], st, 0, 0, 0);
            st = __builtin_amdgcn_mfma_f32_32x32x8f16(kf[m].v[1], qf[m].v[1], st, 0, 0, 0);
        }
        if (kt + NW < n_tiles) load_keys(k0 + 32 * NW);      // in flight during the softmax and the second product
        __builtin_amdgcn_wave_barrier();
        // value tile into LDS as it lies in memory, 16 bytes per lane (the previous tile's readers are this same
        // wavefront: LDS operations of one wavefront complete in order); the transposition happens on the way
        // out, below
#pragma unroll
        for (int n = 0; n < D / 16; ++n) {
            const int u = l + 64 * n, key = u / (D / 8), dp = u % (D / 8);
            *reinterpret_cast<uint4 *>(vt + key * VP + dp * 8) = vraw[n];
        }
        if (kt + NW < n_tiles) load_values(k0 + 32 * NW);
        float tmax = -INFINITY;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int key = k0 + 8 * (i >> 2) + 4 * h + (i & 3);
            const bool seen = q_ok && key < Sk && key <= my_q + shift;
            st[i] = seen ? st[i] * inv_sqrt_d : -INFINITY;
            tmax = fmaxf(tmax, st[i]);
        }
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
        const float m_new = fmaxf(mrun, tmax);
        const float rescale = m_new == -INFINITY ? 1.f : __builtin_amdgcn_exp2f(mrun - m_new);
        float tsum = 0.f;
        v4h pb[4];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const float pi = st[i] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(st[i] - m_new);
            tsum += pi;
            pb[i >> 2][i & 3] = (_Float16)pi;
        }
        tsum += __shfl_xor(tsum, 32);
        lrun = lrun * rescale + tsum;
        mrun = m_new;
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
#pragma unroll
            for (int i = 0; i < 16; ++i) ot[ct][i] *= rescale;
        __builtin_amdgcn_wave_barrier();                     // the value tile is written (same wavefront, in order)
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                // A = V^T: this lane's column 32 ct + c of keys 8b + 4h + 0..3: four 2-byte reads, consecutive
                // lanes on consecutive halves of one key row
                const _Float16 *col = reinterpret_cast<const _Float16 *>(vt) + (8 * b + 4 * h) * VP + 32 * ct + c;
                const v4h va = {col[0], col[VP], col[2 * VP], col[3 * VP]};
                ot[ct] = __builtin_amdgcn_mfma_f32_32x32x8f16(va, pb[b], ot[ct], 0, 0, 0);
            }
        __builtin_amdgcn_wave_barrier();
    }
    // merge: every wavefront publishes its (m, l) and, for each column tile it does not own, its piece of O^T
    __syncthreads();                                         // the value tiles are no longer needed
    float *ml = reinterpret_cast<float *>(lds + CT * NW * 4096);
    ml[(wave * 64 + l) * 2] = mrun;
    ml[(wave * 64 + l) * 2 + 1] = lrun;
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) {
        if (ct != wave) {
            float *dst = reinterpret_cast<float *>(lds + (ct * NW + wave) * 4096);
#pragma unroll
            for (int i = 0; i < 16; ++i) dst[i * 64 + l] = ot[ct][i];
        }
    }
    __syncthreads();
    if (wave < CT) {
        float mall = -INFINITY;
#pragma unroll
        for (int w = 0; w < NW; ++w) mall = fmaxf(mall, ml[(w * 64 + l) * 2]);
        float lall = 0.f, f[NW];
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const float mw = ml[(w * 64 + l) * 2];
            f[w] = mw == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(mw - mall);
            lall += ml[(w * 64 + l) * 2 + 1] * f[w];
        }
        v16f acc;
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
            if (ct == wave) {
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[i] = ot[ct][i] * f[ct];         // static indices after unrolling
            }
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            if (w != wave) {
                const float *src = reinterpret_cast<const float *>(lds + (wave * NW + w) * 4096);
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[i] = fmaf(src[i * 64 + l], f[w], acc[i]);
            }
        }
        if (q_ok) {
            const float inv_l = 1.0f / lall;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                union { uint2 u; __half2 p[2]; } out;
                out.p[0] = __floats2half2_rn(acc[4 * g] * inv_l, acc[4 * g + 1] * inv_l);
                out.p[1] = __floats2half2_rn(acc[4 * g + 2] * inv_l, acc[4 * g + 3] * inv_l);
                *reinterpret_cast<uint2 *>(O + (int64_t)my_q * ldo + 32 * wave + 8 * g + 4 * h) = out.u;
            }
        }
    }
}

sqap_status launch_attention(const __half *Q, int64_t ldq, const __half *Kc, int64_t ldk, const __half *V,
                             int64_t ldv, int batch, int Sq, int Sk, int H, int d, __half *O, int64_t ldo, hipStream_t st)
{
    if (Sq == 0 || batch == 0) return SQAP_OK;
    if (d == 64 || d == 128) {
        const dim3 wgrid(H, (Sq + 31) / 32, batch);
        if (d == 64)
            hipLaunchKernelGGL(attention_mfma_kernel<64>, wgrid, dim3(64 * kAttWaves), 0, st, Q, ldq, Kc, ldk, V, ldv, Sq, Sk, H, O, ldo);
        else
            hipLaunchKernelGGL(attention_mfma_kernel<128>, wgrid, dim3(64 * kAttWaves), 0, st, Q, ldq, Kc, ldk, V, ldv, Sq, Sk, H, O, ldo);
        SQAP_HIP_CHECK(hipGetLastError());
        return SQAP_OK;
    }
    const dim3 grid(H, (Sq + kAttQ - 1) / kAttQ, batch);
#define SQAP_ATT_CASE(DD)                                                                                          \
    case DD:                                                                                                       \
        hipLaunchKernelGGL(attention_kernel<DD>, grid, dim3(256), 0, st, Q, ldq, Kc, ldk, V, ldv, Sq, Sk, H, O, ldo); \
        break;
    switch (d) {
        SQAP_ATT_CASE(16)
        SQAP_ATT_CASE(32)
    default:
        return fail(SQAP_EUNSUPPORTED, "attention: head size %d (16, 32, 64 or 128)", d);
    }
#undef SQAP_ATT_CASE
    SQAP_HIP_CHECK(hipGetLastError());
    return SQAP_OK;
}

// One decode step's attention in a single launch: the new token's query and key are rotated (same
// arithmetic as rope_kernel), the rotated key and the value go into row `past` of the cache, and the
// query attends to cache rows 0 .. past.  One workgroup per head.  At one token each of the three
// launches this replaces (rotation + append, attention, activation quantizer) is a few microseconds
// of latency and no work, so the quantizer of the following linear is folded in as well: the
// workgroup that finishes last (a device-wide arrival counter) quantizes the whole output row.
//
// Scores: 16 lanes per key, lane c holding columns 8c .. 8c+7 (one 16-byte load per key row); softmax over
// chunks of 192 keys with the usual running maximum and sum; output: the same lane layout over the value
// rows, the 16 key groups added through LDS.  All binary32.  A chunk's key AND value rows (12 of each per
// lane) are asked for at once, the first chunk's before the rotation, whose binary64 sine and cosine are a
// longer dependent chain than the rest of the kernel: a prefix of up to 191 positions costs one round of loads.
__global__ __launch_bounds__(256) void decode_attention_kernel(const __half *__restrict__ QKV,
                                                               const int32_t *__restrict__ pos, int H, int d,
                                                               double base, __half *KV, int64_t ldkv, int past,
                                                               __half *O, uint8_t *__restrict__ Xq,
                                                               __half *__restrict__ sx, unsigned int *counter,
                                                               const RopeFreq freq)
{
    __shared__ DecodeAttnLds lds;
    __shared__ int last_flag;
    float *ored = lds.ored, *wred = lds.wred;
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int width = H * d;
    decode_attention_head<false>(lds, blockIdx.x, QKV, pos[0], H, d, base, KV, ldkv, past, O, nullptr, freq);
    if (!Xq) return;

    // the workgroup that arrives last quantizes the whole row (as quantize_rows_kernel does)
    __threadfence();                                   // this head's outputs before the arrival
    __syncthreads();
    if (t == 0) {
        const unsigned int before = atomicAdd(counter, 1u);
        last_flag = before == (unsigned int)(H - 1);
    }
    __syncthreads();
    if (!last_flag) return;
    __threadfence();                                   // the other heads' outputs after the arrival
    __half *row = reinterpret_cast<__half *>(ored);
    const int groups = width >> 3;
    float amax = 0.f;
    for (int g = t; g < groups; g += 256) {
        const uint4 raw = reinterpret_cast<const uint4 *>(O)[g];
        reinterpret_cast<uint4 *>(row)[g] = raw;
        float f[8];
        unpack_halves(raw, f);
#pragma unroll
        for (int e = 0; e < 8; ++e) amax = fmaxf(amax, fabsf(f[e]));
    }
    amax = wavefront_max(amax);
    if (lane == 0) wred[wave] = amax;
    __syncthreads();
    amax = fmaxf(fmaxf(wred[0], wred[1]), fmaxf(wred[2], wred[3]));
    const __half sh = row_scale(amax);
    const float sf = __half2float(sh);
    const float rcp = 1.0f / sf;
    if (t == 0) {
        sx[0] = sh;
        atomicExch(counter, 0u);                       // the next call starts from zero again
    }
    for (int g = t; g < groups; g += 256) {
        float f[8];
        unpack_halves(reinterpret_cast<const uint4 *>(row)[g], f);
        uint32_t packed = 0;
#pragma unroll
        for (int e = 0; e < 8; ++e) packed |= code4(quotient(f[e], sf, rcp)) << (4 * e);
        reinterpret_cast<uint32_t *>(Xq)[g] = packed;
    }
}

sqap_status launch_decode_attention(const __half *QKV, const int32_t *pos, int H, int d, double base, __half *KV,
                                    int64_t ldkv, int past, __half *O, uint8_t *Xq, __half *sx,
                                    unsigned int *counter, hipStream_t st)
{
    hipLaunchKernelGGL(decode_attention_kernel, dim3(H), dim3(256), 0, st, QKV, pos, H, d, base, KV, ldkv, past, O, Xq,
                       sx, counter, rope_frequencies(d, base));
    SQAP_HIP_CHECK(hipGetLastError());
    return SQAP_OK;
}

// x <- half(float(x) + float(delta)), rows of K halves with pitches; 8 elements per thread
__global__ __launch_bounds__(256) void residual_add_kernel(__half *__restrict__ X, int64_t ldx,
                                                           const __half *__restrict__ Dl, int64_t ldd, int M, int K)
{
    const int groups = K >> 3;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)M * groups) return;
    const int g = (int)(idx % groups);
    const int64_t r = idx / groups;
    uint4 *xp = reinterpret_cast<uint4 *>(X + r * ldx) + g;
    uint4 a = *xp;
    const uint4 b = reinterpret_cast<const uint4 *>(Dl + r * ldd)[g];
    __half2 *a2 = reinterpret_cast<__half2 *>(&a);
    const __half2 *b2 = reinterpret_cast<const __half2 *>(&b);
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const float2 x = __half22float2(a2[p]), y = __half22float2(b2[p]);
        float s0 = x.x + y.x, s1 = x.y + y.y;
        asm volatile("" : "+v"(s0), "+v"(s1));       // binary32 sums first, then one conversion each
        a2[p] = __floats2half2_rn(s0, s1);
    }
    *xp = a;
}

sqap_status launch_residual_add(__half *X, int64_t ldx, const __half *Dl, int64_t ldd, int M, int K, hipStream_t st)
{
    const int64_t total = (int64_t)M * (K >> 3);
    if (total == 0) return SQAP_OK;
    hipLaunchKernelGGL(residual_add_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, X, ldx, Dl, ldd, M, K);
    SQAP_HIP_CHECK(hipGetLastError());
    return SQAP_OK;
}

}  // namespace sqap
