// Shared pieces of the attention kernels: launch parameters, dtype helpers, the in-workgroup combine of the four
// waves' online-softmax states, and the workspace layout.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "plan.hpp"

namespace omni {

constexpr int kMaxGroup = 16;          // query heads per KV head the kernels cover
constexpr float kLog2e = 1.4426950408889634f;

// Workspace layout (bytes from the workspace base, all 256-byte aligned):
//   [0, 256)                 plan words written by item 0: PL, R, T(lo), T(hi)
//   [256, 256 + 8*B)         per request: first item index, number of partitions (int2)
//   ml_off                   per (item, query head): running max (log2 domain) and sum, float2
//   o_off                    per (item, query head): unnormalised output row, D floats
struct Workspace {
    int32_t *plan_words;
    int2 *req_info;
    float2 *part_ml;
    float *part_o;
};

struct AttnParams {
    const void *q;
    const void *k_cache;
    const void *v_cache;
    const int32_t *block_table;
    const int32_t *context_lens;
    void *out;
    Workspace ws;
    PlanParams plan;
    float scale_log2;                   // scale * log2(e): scores are kept in the log2 domain and exp2 is used
    int Hq, Hkv, G, MB;
    int log2_ps;
    int out_bf16;
};

__device__ __forceinline__ float bf16_bits_to_float(uint32_t bits16) { return __uint_as_float(bits16 << 16); }

__device__ __forceinline__ uint16_t float_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);   // NaN stays NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// LDS exchange area for the four waves of a workgroup: per wave an unnormalised output tile [kMaxGroup][D + 4]
// (the +4 floats of padding spread the rows of different heads over different banks) and (m, l) per head.
template <int D>
struct CombineSmem {
    float o[kWaves][kMaxGroup][D + 4];
    float m[kWaves][kMaxGroup];
    float l[kWaves][kMaxGroup];
};

// Combine the four waves' (m, l, o) of this item and store: the normalised output when the request has a single
// partition, else the unnormalised row plus (m, l) for the merge kernel.  Must be called by all 256 threads after the
// waves have filled `sm` (this function synchronises first).
template <int D>
__device__ __forceinline__ void wg_combine_and_store(const CombineSmem<D> &sm, const AttnParams &p, const Item &it,
                                                     int r, int kvh) {
    __syncthreads();
    const int G = p.G;
    const int head0 = kvh * G;
    for (int idx = threadIdx.x; idx < G * D; idx += kThreads) {
        const int g = idx / D, d = idx - g * D;
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) M = fmaxf(M, sm.m[w][g]);
        float num = 0.f, den = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            const float mw = sm.m[w][g];
            if (mw > -INFINITY) {
                const float a = fast_exp2(mw - M);
                num += a * sm.o[w][g][d];
                den += a * sm.l[w][g];
            }
        }
        if (it.nparts == 1) {
            const float res = den > 0.f ? num / den : 0.f;
            const size_t oi = ((size_t)it.b * p.Hq + head0) * D + idx;
            if (p.out_bf16) reinterpret_cast<uint16_t *>(p.out)[oi] = float_to_bf16_rne(res);
            else reinterpret_cast<float *>(p.out)[oi] = res;
        } else {
            const size_t pi = (size_t)r * p.Hq + head0;
            p.ws.part_o[pi * D + idx] = num;
            if (d == 0) p.ws.part_ml[pi + g] = make_float2(M, den);
        }
    }
    if (threadIdx.x == 0 && kvh == 0 && it.part == 0) p.ws.req_info[it.b] = make_int2(it.start, it.nparts);
}

}  // namespace omni
