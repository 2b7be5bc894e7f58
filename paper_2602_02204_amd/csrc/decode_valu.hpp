// Vector-ALU split-context decode kernel: covers fp32 and bf16 KV, head_dim 64 and 128, page sizes 16 and 32, any
// group size up to GP.  A workgroup walks the segments of its ranges (see plan.hpp) for one KV head; within a segment
// each wave streams whole token rows with 16-byte loads (a row of D elements is spread over D*es/16 adjacent lanes),
// keeps one online-softmax state per lane group, and the states are merged by cross-lane shuffles, then through LDS.
#pragma once
#include "common.hpp"

namespace omni {

template <typename T> struct ElemTraits;
template <> struct ElemTraits<float> {
    static constexpr int kVec = 4;
    __device__ static __forceinline__ void unpack(const uint4 &r, float *f) {
        f[0] = __uint_as_float(r.x); f[1] = __uint_as_float(r.y); f[2] = __uint_as_float(r.z); f[3] = __uint_as_float(r.w);
    }
};
template <> struct ElemTraits<uint16_t> {          // bf16 bit patterns
    static constexpr int kVec = 8;
    __device__ static __forceinline__ void unpack(const uint4 &r, float *f) {
        f[0] = __uint_as_float(r.x << 16); f[1] = __uint_as_float(r.x & 0xffff0000u);
        f[2] = __uint_as_float(r.y << 16); f[3] = __uint_as_float(r.y & 0xffff0000u);
        f[4] = __uint_as_float(r.z << 16); f[5] = __uint_as_float(r.z & 0xffff0000u);
        f[6] = __uint_as_float(r.w << 16); f[7] = __uint_as_float(r.w & 0xffff0000u);
    }
};

template <typename T, int D, int GP>
__global__ __launch_bounds__(kThreads) void decode_valu_kernel(AttnParams p) {
    constexpr int VEC = ElemTraits<T>::kVec;
    constexpr int LPR = D / VEC;               // lanes per token row
    constexpr int TPW = 64 / LPR;              // token rows per wave-wide load
    static_assert(LPR <= 64 && (LPR & (LPR - 1)) == 0, "row must fit a wave");

    __shared__ CombineSmem<D> sm;
    __shared__ PlanSmem ps;
    extern __shared__ int E[];                 // B + 1 tile offsets

    int w, kvh;
    wg_coords(p, &w, &kvh);
    const Plan pl = attn_prologue<D>(p, &ps, E, w, kvh);
    const int G = p.G;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane % LPR, sub = lane / LPR;
    const int ps_mask = (1 << p.log2_ps) - 1;
    const T *kc = reinterpret_cast<const T *>(p.k_cache);
    const T *vc = reinterpret_cast<const T *>(p.v_cache);

    for_each_segment<D>(p, pl, &ps, E, sm, w, kvh, [&](const Segment &seg) {
    const int t0 = seg.lo * kTile;
    const int t1 = min(seg.L, seg.hi * kTile);

    // query rows of the group, this lane's VEC elements of each
    float qf[GP][VEC];
#pragma unroll
    for (int g = 0; g < GP; ++g) {
        if (g < G) {
            const uint4 raw = *reinterpret_cast<const uint4 *>(
                reinterpret_cast<const T *>(p.q) + ((size_t)seg.b * p.Hq + kvh * G + g) * D + c * VEC);
            ElemTraits<T>::unpack(raw, qf[g]);
        } else {
#pragma unroll
            for (int e = 0; e < VEC; ++e) qf[g][e] = 0.f;
        }
    }

    float m[GP], l[GP], o[GP][VEC];
#pragma unroll
    for (int g = 0; g < GP; ++g) {
        m[g] = -INFINITY; l[g] = 0.f;
#pragma unroll
        for (int e = 0; e < VEC; ++e) o[g][e] = 0.f;
    }

    const int32_t *bt = p.block_table + (size_t)seg.b * p.MB;

    for (int tt = t0 + wave * TPW; tt < t1; tt += kWaves * TPW) {
        const int t = tt + sub;
        const bool valid = t < t1;
        uint4 kraw = make_uint4(0, 0, 0, 0), vraw = make_uint4(0, 0, 0, 0);
        if (valid) {
            const int page = bt[t >> p.log2_ps];
            const size_t off = ((((size_t)page * p.Hkv + kvh) << p.log2_ps) + (t & ps_mask)) * D + c * VEC;
            kraw = nt_load16(kc + off);
            vraw = nt_load16(vc + off);
        }
        float kf[VEC], vf[VEC];
        ElemTraits<T>::unpack(kraw, kf);
        ElemTraits<T>::unpack(vraw, vf);
#pragma unroll
        for (int g = 0; g < GP; ++g) {
            if (g < G) {                                  // uniform
                float dot = 0.f;
#pragma unroll
                for (int e = 0; e < VEC; ++e) dot = fmaf(qf[g][e], kf[e], dot);
#pragma unroll
                for (int off = 1; off < LPR; off <<= 1) dot += __shfl_xor(dot, off);
                if (valid) {
                    // the product must be rounded before the max is subtracted (no fused multiply-subtract), so that
                    // s - max is exactly 0 for the maximal score
#pragma clang fp contract(off)
                    const float s = dot * p.scale_log2;
                    const float mn = fmaxf(m[g], s);
                    const float a = fast_exp2(m[g] - mn);       // exp2(-inf) = 0 on the first token
                    const float pw = fast_exp2(s - mn);
                    l[g] = l[g] * a + pw;
#pragma unroll
                    for (int e = 0; e < VEC; ++e) o[g][e] = fmaf(pw, vf[e], o[g][e] * a);
                    m[g] = mn;
                }
            }
        }
    }

    // merge the TPW lane groups of the wave
#pragma unroll
    for (int g = 0; g < GP; ++g) {
        if (g < G) {
#pragma unroll
            for (int off = LPR; off < 64; off <<= 1) {
                const float mo = __shfl_xor(m[g], off);
                const float lo = __shfl_xor(l[g], off);
                const float M = fmaxf(m[g], mo);
                const float a = m[g] > -INFINITY ? fast_exp2(m[g] - M) : 0.f;
                const float bsc = mo > -INFINITY ? fast_exp2(mo - M) : 0.f;
                l[g] = l[g] * a + lo * bsc;
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    const float oo = __shfl_xor(o[g][e], off);
                    o[g][e] = o[g][e] * a + oo * bsc;
                }
                m[g] = M;
            }
            if (sub == 0) {
#pragma unroll
                for (int e = 0; e < VEC; ++e) sm.o[wave][g][c * VEC + e] = o[g][e];
                if (c == 0) { sm.m[wave][g] = m[g]; sm.l[wave][g] = l[g]; }
            }
        }
    }
    });
}

}  // namespace omni
