// One decode step's attention for ONE head, as a device function shared by the single-launch kernel
// (glue.hip) and the whole-step kernel (decoder_step.hip), plus the rotation-frequency table both use.
// Device code only.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>
#include <cmath>

#include "common.h"

namespace sqap {

// A pointer that was loaded from memory (a table of per-layer pointers, say) is a generic pointer to the
// compiler: loads through it become flat loads, each fenced by a full wait because it might address LDS.
// Saying that it addresses global memory turns them back into global loads that overlap.
// (Address-space pointers only take built-in types: halves travel as 16-bit integers, 16-byte pieces as vectors.)
#define SQAP_GLOBAL __attribute__((address_space(1)))
typedef unsigned int sqap_v4u __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 global_load16(const void *p)
{
    const sqap_v4u v = *(const SQAP_GLOBAL sqap_v4u *)p;
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void global_store_half(__half *p, __half v)
{
    *(SQAP_GLOBAL unsigned short *)p = __half_as_ushort(v);
}

// The rotation frequencies base^(-2i/d), i < d/2, depend on the model alone: the host evaluates them (binary64
// pow) and hands them over as a kernel argument, which takes the power out of the dependent chain
// power -> angle -> sine and cosine that every pair used to walk (a third of a rotary launch's time at a few
// hundred tokens).  Head sizes above 2 * kRopeTableMax evaluate the power on the device as before.
constexpr int kRopeTableMax = 128;
struct RopeFreq {
    double f[kRopeTableMax];
};
static RopeFreq rope_frequencies(int d, double base)
{
    RopeFreq r = {};
    for (int i = 0; i < d / 2 && i < kRopeTableMax; ++i) r.f[i] = std::pow(base, -2.0 * (double)i / (double)d);
    return r;
}
__device__ __forceinline__ double rope_angle(const RopeFreq &freq, int pos, int i, int d, double base)
{
    const double f = (d >> 1) <= kRopeTableMax ? freq.f[i] : pow(base, -2.0 * (double)i / (double)d);
    return (double)pos * f;
}

// Scores: 16 lanes per key, lane c holding columns 8c .. 8c+7 (one 16-byte load per key row); softmax over
// chunks of 192 keys with the usual running maximum and sum, the probabilities kept in registers; output: the
// same lane layout over the value rows, the 16 key groups added through LDS.  All binary32.  A chunk's key AND
// value rows (12 of each per lane) are asked for at once, the first chunk's before the rotation, whose
// binary64 sine and cosine are a longer dependent chain than the rest of the function.
constexpr int kDecKeys = 12;              // keys per lane group and chunk: their key and value rows are in flight together
constexpr int kDecChunk = 16 * kDecKeys;   // keys per softmax chunk
constexpr int kDecMaxD = 128;              // head size limit: 16 lanes x 8 columns
constexpr int kDecMaxRow = 8192;           // H * d limit of the fused quantizer (row staged in LDS)

__device__ __forceinline__ void unpack_halves(const uint4 raw, float (&f)[8])
{
    const __half2 *h2 = reinterpret_cast<const __half2 *>(&raw);
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const float2 x = __half22float2(h2[p]);
        f[2 * p] = x.x;
        f[2 * p + 1] = x.y;
    }
}


// LDS of one head's attention (the reduction buffer doubles as the staged output row of the fused quantizer).
constexpr int kDecRedFloats = 16 * kDecMaxD > kDecMaxRow / 2 ? 16 * kDecMaxD : kDecMaxRow / 2;
struct DecodeAttnLds {
    __attribute__((aligned(16))) float qf[kDecMaxD];
    __attribute__((aligned(16))) __half knew[kDecMaxD], vnew[kDecMaxD];
    __attribute__((aligned(16))) float ored[kDecRedFloats];
    float wred[12];            // chunk maxima of the four wavefronts (two sets, by chunk parity); their sums
};
static_assert(sizeof(float) * kDecRedFloats >= kDecMaxRow * sizeof(__half), "the staged row must fit the reduction buffer");

// 16 bytes of LDS as a plain vector.  (Accesses typed as the uint4 class make the compiler wait for every load
// in flight that lands in LDS, the weight stream included: it takes them as possibly the same memory.  The
// kernels wait for what they read themselves.)
typedef int sqap_v4i __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 lds_load16(const void *p)
{
    const sqap_v4i v = *reinterpret_cast<const sqap_v4i *>(p);
    return make_uint4((unsigned)v.x, (unsigned)v.y, (unsigned)v.z, (unsigned)v.w);
}
__device__ __forceinline__ void lds_store16(void *p, const uint4 v)
{
    *reinterpret_cast<sqap_v4i *>(p) = sqap_v4i{(int)v.x, (int)v.y, (int)v.z, (int)v.w};
}

// The half in the low 16 bits of a tagged word (the whole-step kernel's rows: the high 16 bits say which
// step and layer wrote the word).
__device__ __forceinline__ __half untag(unsigned w) { return __ushort_as_half((unsigned short)(w & 0xffffu)); }

// Rotation of head h's query and key of the new token (same arithmetic as rope_kernel), cache append (rotated
// key | value into row `past` of KV), attention of the query over cache rows 0 .. past, output into
// O[h * d .. h * d + d) (and into trace, when given).  Called by EVERY thread of the workgroup (it contains
// workgroup barriers); the first 256 threads do the work, any others only keep step.  LDS in `lds`.
// TAGGED (the whole-step kernel): the new token's q, k, v of this head were fetched by the caller as tagged
// words into LDS (`staged`: q at word 0, k at 256, v at 512, complete when every thread has reached the
// function's first barrier; QKV is not used); O is a row of tagged words
// that other workgroups of the launch wait for (64-bit agent-scope stores, tag `tag`); `sincos_tab` (d / 2 pairs
// of binary64 sine, cosine of the token's angles, evaluated once per step by the same sincos call) replaces the
// evaluation per layer: same bits.  d even, d <= 128.
// (V_LATE asks for the value rows after the scores instead of together with the key rows: half the
// registers for one more memory round trip; not used at present.)
template <bool TAGGED>
__device__ __forceinline__ void decode_attention_head(DecodeAttnLds &lds, int h, const __half *QKV, int pos0, int H,
                                                      int d, double base, __half *KV, int64_t ldkv, int past,
                                                      void *O, __half *trace, const RopeFreq &freq,
                                                      const double2 *sincos_tab = nullptr, const unsigned *staged = nullptr,
                                                      unsigned tag = 0)
{
    constexpr bool AGENT = TAGGED;
    // (tagged form: the wavefronts have weight loads in flight; what the barriers below hand over is in LDS)
    auto sync = [] {
        if constexpr (TAGGED) lds_barrier();
        else __syncthreads();
    };
    float *qf = lds.qf, *ored = lds.ored, *wred = lds.wred;
    __half *knew = lds.knew, *vnew = lds.vnew;
    int t = threadIdx.x;
    // Inside a loop over layers everything below that depends only on the lane is loop invariant; hoisted out, it
    // would sit in registers (in practice: in scratch memory) for the whole step.  The empty asm makes the
    // compiler take t as a new value here, so the addresses are formed where they are used.
    if (AGENT) asm volatile("" : "+v"(t));
    const int lane = t & 63, wave = t >> 6;
    const int half_d = d >> 1, width = H * d;
    const int Sk = past + 1;

    const int grp = t >> 4, c = t & 15;              // key group, column chunk
    // (in a workgroup of more than 256 threads the others only walk through the barriers)
    const bool on = t < 256;
    const bool col_ok = on && c * 8 < d;
    const __half *kbase = KV + (int64_t)h * d + c * 8, *vbase = kbase + width;
    // a cached row's 8 columns of this lane (zeros past the prefix; the new token's row comes from LDS later)
    auto cached = [&](const __half *gbase, int key) {
        uint4 raw = make_uint4(0u, 0u, 0u, 0u);
        if (col_ok && key < past) raw = global_load16(gbase + (int64_t)key * ldkv);
        return raw;
    };
    // the new token's query, key and value elements of this lane (rotation pairs i and i + d / 2): asked for
    // before the cache rows, because loads return in order and the rotation is the longer chain.  (Tagged form:
    // they come from LDS, where the caller's fetching wavefront puts them; the cache rows do not depend on
    // them and are asked for before the barrier that waits for that wavefront.)
    const __half *q = QKV + (int64_t)h * d, *k = QKV + width + (int64_t)h * d, *v = QKV + 2 * width + (int64_t)h * d;
    __half qkv_new[6] = {};
    if constexpr (!TAGGED) {
        if (t < half_d) {
            qkv_new[0] = q[t];
            qkv_new[1] = q[t + half_d];
            qkv_new[2] = k[t];
            qkv_new[3] = k[t + half_d];
            qkv_new[4] = v[t];
            qkv_new[5] = v[t + half_d];
        }
    }
    constexpr bool V_LATE = false;
    uint4 kraw[kDecKeys], vraw[V_LATE ? 1 : kDecKeys];
    // (all key rows first: loads return in order, and the scores need the keys only)
#pragma unroll
    for (int j = 0; j < kDecKeys; ++j) kraw[j] = cached(kbase, 16 * j + grp);
    if (!V_LATE) {
#pragma unroll
        for (int j = 0; j < kDecKeys; ++j) vraw[j] = cached(vbase, 16 * j + grp);
    }
    if constexpr (TAGGED) {
        sync();                                        // the new token's q, k, v are in `staged`
        if (t < half_d) {
            qkv_new[0] = untag(staged[t]);
            qkv_new[1] = untag(staged[t + half_d]);
            qkv_new[2] = untag(staged[256 + t]);
            qkv_new[3] = untag(staged[256 + t + half_d]);
            qkv_new[4] = untag(staged[512 + t]);
            qkv_new[5] = untag(staged[512 + t + half_d]);
        }
    }

    // rotation of this head's query and key; the value is copied
    if (t < half_d) {
        const int i = t;
        double sn, cs;
        if constexpr (AGENT) {                         // (the table is not optional in this form)
            sn = sincos_tab[i].x;
            cs = sincos_tab[i].y;
        } else {
            const double a = rope_angle(freq, pos0, i, d, base);
            sincos(a, &sn, &cs);
        }
        __half *krow = KV + (int64_t)past * ldkv + (int64_t)h * d, *vrow = krow + width;
        double lo = (double)__half2float(qkv_new[0]), hi = (double)__half2float(qkv_new[1]);
        qf[i] = __half2float(__float2half_rn((float)(lo * cs - hi * sn)));
        qf[i + half_d] = __half2float(__float2half_rn((float)(hi * cs + lo * sn)));
        lo = (double)__half2float(qkv_new[2]);
        hi = (double)__half2float(qkv_new[3]);
        const __half k0 = __float2half_rn((float)(lo * cs - hi * sn));
        const __half k1 = __float2half_rn((float)(hi * cs + lo * sn));
        knew[i] = k0;
        knew[i + half_d] = k1;
        global_store_half(krow + i, k0);
        global_store_half(krow + i + half_d, k1);
        const __half v0 = qkv_new[4], v1 = qkv_new[5];
        vnew[i] = v0;
        vnew[i + half_d] = v1;
        global_store_half(vrow + i, v0);
        global_store_half(vrow + i + half_d, v1);
    }
    sync();
    float q8[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) q8[e] = col_ok ? qf[c * 8 + e] : 0.f;
    const float inv_sqrt_d = 1.0f / sqrtf((float)d);

    // Softmax over chunks with a running maximum; the probabilities never leave the registers.  After the
    // 16-lane sums a group's twelve scores are in all of its lanes; the chunk's maximum crosses the wavefronts
    // through LDS (the only barrier of a chunk); lane c of a group exponentiates score c, the group's lanes
    // exchange the results; every wavefront keeps the sum of ITS keys' probabilities, rescaled like the output
    // (the four are added at the end, (w0 + w1) + (w2 + w3)).
    float o[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = 0.f;
    float m = -INFINITY, l_wave = 0.f;
    int parity = 0;
    for (int c0 = 0; c0 < Sk; c0 += kDecChunk, parity ^= 1) {
        const int n = min(kDecChunk, Sk - c0);
#pragma unroll
        for (int j = 0; j < kDecKeys; ++j) {
            const int key = c0 + 16 * j + grp;
            if (c0 > 0) {
                kraw[j] = cached(kbase, key);
                if (!V_LATE) vraw[j] = cached(vbase, key);
            }
            if (key == past && col_ok) {
                kraw[j] = lds_load16(knew + c * 8);
                if (!V_LATE) vraw[j] = lds_load16(vnew + c * 8);
            }
        }
        float sj[kDecKeys];
        float mx = -INFINITY;
#pragma unroll
        for (int j = 0; j < kDecKeys; ++j) {
            float kf[8];
            unpack_halves(kraw[j], kf);
            float s = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) s = fmaf(q8[e], kf[e], s);
            // the 16 lanes' sum in all of them (quad permutes, then the mirrors: operand modifiers, no LDS permute)
            s += dpp_move_f<kDppXor1>(s);
            s += dpp_move_f<kDppXor2>(s);
            s += dpp_move_f<kDppHalfMirror>(s);
            s += dpp_move_f<kDppMirror>(s);
            sj[j] = 16 * j + grp < n ? s * inv_sqrt_d : -INFINITY;
            mx = fmaxf(mx, sj[j]);
        }
        // (late form: the key registers are free now; the value rows arrive during the softmax)
        uint4 vlate[V_LATE ? kDecKeys : 1];
        if (V_LATE) {
#pragma unroll
            for (int j = 0; j < kDecKeys; ++j) {
                const int key = c0 + 16 * j + grp;
                vlate[j] = cached(vbase, key);
                if (key == past && col_ok) vlate[j] = lds_load16(vnew + c * 8);
            }
        }
        mx = fmaxf(fmaxf(row_value(mx, 0), row_value(mx, 1)), fmaxf(row_value(mx, 2), row_value(mx, 3)));      // (the same in a group's lanes)
        if (lane == 0 && wave < 4) wred[parity * 4 + wave] = mx;
        sync();                                        // (the other parity's maxima were read before the barrier of the chunk before)
        const float m_new = fmaxf(m, fmaxf(fmaxf(wred[parity * 4], wred[parity * 4 + 1]), fmaxf(wred[parity * 4 + 2], wred[parity * 4 + 3])));
        // lane c's score (a chain of selects: the array stays in registers)
        float mine = -INFINITY;
#pragma unroll
        for (int j = 0; j < kDecKeys; ++j) mine = c == j ? sj[j] : mine;
        const float pm = mine == -INFINITY ? 0.f : expf(mine - m_new);      // (a key past the end, or lanes 12 .. 15)
        const float rescale = expf(m - m_new);         // m = -inf only before the first chunk: exp(-inf) = 0
        m = m_new;
        float psum = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] *= rescale;
#pragma unroll
        for (int j = 0; j < kDecKeys; ++j) {
            const float pj = __shfl(pm, (lane & 48) | j);
            psum += pj;
            float vf[8];
            if (!V_LATE) unpack_halves(vraw[j], vf);
            else unpack_halves(vlate[j], vf);
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = fmaf(pj, vf[e], o[e]);
        }
        psum = (row_value(psum, 0) + row_value(psum, 1)) + (row_value(psum, 2) + row_value(psum, 3));       // the four groups of the wavefront
        l_wave = l_wave * rescale + psum;
    }
    if (lane == 0 && wave < 4) wred[8 + wave] = l_wave;
    if (col_ok) {
#pragma unroll
        for (int e = 0; e < 8; ++e) ored[grp * kDecMaxD + c * 8 + e] = o[e];
    }
    sync();
    {
        float acc = 0.f;
        if (t < d) {
#pragma unroll
            for (int g = 0; g < 16; ++g) acc += ored[g * kDecMaxD + t];
        }
        const float l = (wred[8] + wred[9]) + (wred[10] + wred[11]);
        const __half r = __float2half_rn(acc * (1.0f / l));
        if constexpr (!TAGGED) {
            if (t < d) reinterpret_cast<__half *>(O)[(int64_t)h * d + t] = r;
        } else {
            // two tagged words per 64-bit agent-scope store (d is even, so a pair never leaves the head)
            const unsigned mine = __half_as_ushort(r), next = __shfl_down(mine, 1);
            if (t < d && (t & 1) == 0) {
                const unsigned long long lo = (tag << 16) | mine, hi = (tag << 16) | next;
                __hip_atomic_store(reinterpret_cast<unsigned long long *>(reinterpret_cast<unsigned *>(O) + (int64_t)h * d + t),
                                   lo | (hi << 32), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (trace) *reinterpret_cast<unsigned *>(trace + (int64_t)h * d + t) = mine | (next << 16);
            }
        }
    }
}

}  // namespace sqap
