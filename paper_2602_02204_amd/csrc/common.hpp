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
//   [256, 256 + 4*B*Hkv)     per (request, KV head): arrival counter of its partitions; zero between calls
//   ml_off                   per (slot, query head): running max (log2 domain) and sum, float2
//   o_off                    per (slot, query head): unnormalised output row, D floats
struct Workspace {
    int32_t *plan_words;
    int32_t *arrivals;
    float2 *part_ml;
    float *part_o;
};

struct AttnParams {
    const void *q;
    const void *k_cache;
    const void *v_cache;
    const void *k_new;                  // fused decode step only (else null): rows to append at context_lens[b] - 1
    const void *v_new;
    const int32_t *block_table;
    const int32_t *context_lens;
    void *out;
    Workspace ws;
    PlanParams plan;
    float scale_log2;                   // scale * log2(e): scores are kept in the log2 domain and exp2 is used
    int Hq, Hkv, G, MB;
    int log2_ps;
    int out_bf16;
#ifdef OMNI_TRACE
    long long *trace;                   // development builds only: per-wave phase timestamps
#endif
};

// Phase timestamps for development builds (compiled out otherwise): slot `id` of this wave's record.
#ifdef OMNI_TRACE
#define OMNI_STAMP(p, id)                                                                              \
    do {                                                                                               \
        if ((p).trace && (threadIdx.x & 63) == 0)                                                      \
            (p).trace[((size_t)blockIdx.x * kWaves + (threadIdx.x >> 6)) * 16 + (id)] = wall_clock64(); \
    } while (0)
#else
#define OMNI_STAMP(p, id) do { } while (0)
#endif

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
    int flag;                          // set when this workgroup is the last partition of its (request, KV head) to arrive
};

// Relaxed device-scope accesses: coherent across the compute dies without a cache-wide fence.
__device__ __forceinline__ void dev_store(float *ptr, float v) {
    __hip_atomic_store(ptr, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float dev_load(const float *ptr) {
    return __hip_atomic_load(ptr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ void store_out(const AttnParams &p, size_t index, float v) {
    if (p.out_bf16) reinterpret_cast<uint16_t *>(p.out)[index] = float_to_bf16_rne(v);
    else reinterpret_cast<float *>(p.out)[index] = v;
}

// One thread: count this workgroup's arrival for the request of `seg`; true if it is the last piece to arrive.
__device__ __forceinline__ bool count_arrival(const AttnParams &p, const Segment &seg, int kvh) {
    const int old = __hip_atomic_fetch_add(&p.ws.arrivals[seg.b * p.Hkv + kvh], 1, __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_AGENT);
    return old == seg.nparts - 1;
}

// All 256 threads: log-sum-exp merge of the request's pieces, in slot order.  Every thread owns up to kMergeIdx
// output elements; the loads of kRound pieces for all of them are issued before any is used, so a round costs one
// trip to memory, and no load depends on a loaded value.  Puts the arrival counter back to zero for the next
// call.
template <int D, int kMergeIdx, int kRound>
__device__ __forceinline__ void merge_request_impl(const AttnParams &p, const Segment &seg, int kvh) {
    const int G = p.G, head0 = kvh * G, n = seg.nparts;
    const size_t out0 = ((size_t)seg.b * p.Hq + head0) * D;
    float M[kMergeIdx], num[kMergeIdx], den[kMergeIdx];
#pragma unroll
    for (int i = 0; i < kMergeIdx; ++i) { M[i] = -INFINITY; num[i] = 0.f; den[i] = 0.f; }
    for (int j0 = 0; j0 < n; j0 += kRound) {
        float mj[kMergeIdx][kRound], lj[kMergeIdx][kRound], oj[kMergeIdx][kRound];
#pragma unroll
        for (int i = 0; i < kMergeIdx; ++i) {
            const int idx = threadIdx.x + i * kThreads;
            const int g = idx / D;
#pragma unroll
            for (int u = 0; u < kRound; ++u) {
                lj[i][u] = 0.f; mj[i][u] = 0.f; oj[i][u] = 0.f;
                if (idx < G * D && j0 + u < n) {
                    const size_t pi = (size_t)(seg.slot_first + j0 + u) * p.Hq + head0;
                    mj[i][u] = dev_load(&p.ws.part_ml[pi + g].x);
                    lj[i][u] = dev_load(&p.ws.part_ml[pi + g].y);
                    oj[i][u] = dev_load(&p.ws.part_o[pi * D + idx]);
                }
            }
        }
#pragma unroll
        for (int i = 0; i < kMergeIdx; ++i) {
#pragma unroll
            for (int u = 0; u < kRound; ++u) {
                if (lj[i][u] > 0.f) {
                    const float Mn = fmaxf(M[i], mj[i][u]);
                    const float a = fast_exp2(M[i] - Mn);            // 0 while M is still -inf
                    const float w = fast_exp2(mj[i][u] - Mn);
                    num[i] = num[i] * a + w * oj[i][u];
                    den[i] = den[i] * a + w * lj[i][u];
                    M[i] = Mn;
                }
            }
        }
    }
#pragma unroll
    for (int i = 0; i < kMergeIdx; ++i) {
        const int idx = threadIdx.x + i * kThreads;
        if (idx < G * D) store_out(p, out0 + idx, den[i] > 0.f ? num[i] / den[i] : 0.f);
    }
    if (threadIdx.x == 0)
        __hip_atomic_store(&p.ws.arrivals[seg.b * p.Hkv + kvh], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <int D>
__device__ __forceinline__ void merge_request(const AttnParams &p, const Segment &seg, int kvh) {
    // up to 8 heads: 4 (or 2) output elements per thread, four pieces per round; up to 16 heads: twice the elements, two pieces
    if (p.G * D <= 4 * kThreads) merge_request_impl<D, 4, 4>(p, seg, kvh);
    else merge_request_impl<D, kMaxGroup * D / kThreads, 2>(p, seg, kvh);
}

// Combine the four waves' (m, l, o) of one segment and finish it.  Must be called by all 256 threads after the waves
// have filled `sm` (this function synchronises first, and again before it returns so that `sm` may be refilled).
//   - A request that lies inside one range gets its normalised output row at once.
//   - Otherwise the unnormalised row and (m, l) go to the segment's workspace slot, and the workgroup that arrives
//     last for its (request, KV head) performs the log-sum-exp merge over the request's slots, in slot order:
//         out = sum_j 2^(m_j - M) o_j / sum_j 2^(m_j - M) l_j,  M = max_j m_j,  empty pieces (l_j = 0) skipped.
//     "Last" is decided by an arrival counter: a workgroup writes its partial rows, waits for the writes to be
//     acknowledged, then adds one; the workgroup that reads nparts-1 merges and puts the counter back to zero.
//     Nobody waits for anybody, so the scheme cannot hang; the result does not depend on which workgroup merges.
//     The partial rows cross between compute dies whose L2 caches are not coherent with each other.  A device-scope
//     fence would write back and invalidate a whole L2 per workgroup (measured: 4x the kernel time); instead every
//     access to the partial rows and to the counter is a relaxed device-scope atomic (sc1 loads and stores), which
//     goes to the coherence point without touching the rest of the cache.
template <int D>
__device__ __forceinline__ void wg_combine_and_store(CombineSmem<D> &sm, const AttnParams &p, const Segment &seg,
                                                     int kvh) {
    __syncthreads();
    const int G = p.G;
    const int head0 = kvh * G;
    const size_t out0 = ((size_t)seg.b * p.Hq + head0) * D;
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
        if (seg.nparts == 1) {
            store_out(p, out0 + idx, den > 0.f ? num / den : 0.f);
        } else {
            const size_t pi = (size_t)seg.slot * p.Hq + head0;
            dev_store(&p.ws.part_o[pi * D + idx], num);
            if (d == 0) {
                dev_store(&p.ws.part_ml[pi + g].x, M);
                dev_store(&p.ws.part_ml[pi + g].y, den);
            }
        }
    }
    // The barrier's workgroup-scope release makes every wave wait until its device-scope stores above are
    // acknowledged, so they are globally visible before the arrival is counted.
    __syncthreads();
    if (seg.nparts == 1) return;                                     // uniform

    if (threadIdx.x == 0) sm.flag = count_arrival(p, seg, kvh);
    __syncthreads();
    const bool last = sm.flag;
    __syncthreads();                                                 // flag may be rewritten by the next segment
    if (last) merge_request<D>(p, seg, kvh);                         // uniform
}

// blockIdx -> (workgroup index w within its KV head, KV head).  Workgroups are dealt to the eight compute dies
// round-robin by blockIdx; this mapping gives every die a share of every KV head (a KV head is a fixed 4 KB or 8 KB
// slice of each page, i.e. a fixed set of address bits) instead of binding each die to one head.
__device__ __forceinline__ void wg_coords(const AttnParams &p, int *w, int *kvh) {
    constexpr int kDies = 8;
    const int bid = blockIdx.x;
    if (gridDim.x % (kDies * p.Hkv) == 0) {
        const int x = bid % kDies, y = bid / kDies;
        *kvh = y % p.Hkv;
        *w = x + kDies * (y / p.Hkv);
    } else {
        *w = bid / p.Hkv;
        *kvh = bid - *w * p.Hkv;
    }
}

// Prologue shared by the partition kernels: build the plan in shared memory, write the all-zero rows of empty
// requests (first workgroup of each KV head) and the plan words (first workgroup of the grid).
template <int D>
__device__ __forceinline__ Plan attn_prologue(const AttnParams &p, PlanSmem *ps, int *E, int w, int kvh,
                                              int first_len = 0, bool have_first = false) {
    const Plan pl = plan_build(p.context_lens, p.plan, ps, E, E + p.plan.B + 1, [&](int b) {
        if (w == 0) {
            const size_t o0 = ((size_t)b * p.Hq + kvh * p.G) * D;
            for (int i = 0; i < p.G * D; ++i) store_out(p, o0 + i, 0.f);
        }
    }, first_len, have_first);
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        const unsigned long long T = ps->total_tokens;
        p.ws.plan_words[0] = pl.S * kTile; p.ws.plan_words[1] = pl.nranges;
        p.ws.plan_words[2] = (int)(T & 0xffffffffULL); p.ws.plan_words[3] = (int)(T >> 32);
    }
    return pl;
}

// Drive `process(seg)` over every segment of every range of workgroup w, finishing each with the combine above.
template <int D, typename Process>
__device__ __forceinline__ void for_each_segment(const AttnParams &p, const Plan &pl, PlanSmem *ps, const int *E,
                                                 CombineSmem<D> &sm, int w, int kvh, Process process) {
    for (int range = w; range < pl.nranges; range += p.plan.nw) {
        const int start = range * pl.S, end = min(pl.C, start + pl.S);
        int b = plan_first_request(p.plan, ps, E, start);
        while (true) {
            const Segment seg = plan_segment(E, E + p.plan.B + 1, pl, b, range, start, end);
            process(seg);
            wg_combine_and_store<D>(sm, p, seg, kvh);
            if (__builtin_amdgcn_readfirstlane(E[b]) + seg.hi >= end) break;
            do { ++b; } while (b < p.plan.B - 1 && E[b + 1] == E[b]);       // skip requests that own no tile
        }
    }
}

}  // namespace omni
