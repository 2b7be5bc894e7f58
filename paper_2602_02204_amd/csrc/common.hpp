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
//   [0, 256)                 plan words written by the first workgroup: range length in tokens, number of ranges,
//                            total context tokens (low, high word)
//   256                      per (slot, query head): running max (log2 domain) and sum, float2
//   o_off                    per (slot, query head): unnormalised output row, D floats
// A slot is one piece of one request (range index + request index); nothing in the workspace needs initialising.
struct Workspace {
    int32_t *plan_words;
    float2 *part_ml;
    float *part_o;
    int2 *merge_rec;                    // [B]: (first partial-result slot, pieces) of every request, left by the
                                        // attention kernel for the merge kernel
};

// Shared memory of the matrix-core kernel behind the plan's arrays: room for `ring_states` online-softmax states, each
// one wave's share of one request as o[G][D + 4] floats followed by m[16] and l[16].
struct MfmaLds {
    int ring_off;                       // bytes from the start of dynamic shared memory
    int state_floats;
    int ring_states;                    // 4 .. kMaxStates
    int total;                          // bytes of dynamic shared memory
    int static_bytes;                   // bytes of the kernel variant's static K staging area (0 if K is not staged)
    bool two_per_cu;                    // total + static_bytes leave room for a second workgroup on the compute unit
};

struct AttnParams {
    const void *q;
    const void *k_cache;
    const void *v_cache;
    const float *k_scale;               // 8-bit KV cache only (else null): [P, Hkv] scales of the K and V pools
    const float *v_scale;
    const void *k_new;                  // fused decode step only (else null): rows to append at context_lens[b] - 1
    const void *v_new;
    const int32_t *block_table;
    const int32_t *context_lens;
    const int32_t *q_lens;              // several query tokens per request only, may be null: how many of the Tq request b
                                        // brings (its last q_lens[b] tokens, rows 0 .. q_lens[b] - 1 of its Tq); null = Tq
    void *out;
    Workspace ws;
    PlanParams plan;
    float scale_log2;                   // scale * log2(e): scores are kept in the log2 domain and exp2 is used
    int Hq, Hkv, G, MB;
    int Tq;                             // query tokens per request (1 = plain decode); q and out are [B, Tq, Hq, D]
    int T, t_off;                       // this launch covers query tokens t_off .. t_off + T - 1 of every request
    int Gq;                             // T * G: the (query token, head) columns of one KV head in this launch
    int log2_ps;
    int out_bf16;
    MfmaLds lds;                        // matrix-core kernel only
};

// Column c of KV head kvh stands for query token t_off + c / G of its request and head kvh * G + c % G.  Its row of
// `out` [B][Tq][Hq] for request b, and its row of the partial results [slot][T][Hq] (this launch's tokens only):
__device__ __forceinline__ size_t out_row(const AttnParams &p, size_t b, int kvh, int c) {
    if (p.Tq == 1) return b * p.Hq + kvh * p.G + c;              // plain decode: no division
    const int qi = c / p.G, g = c - qi * p.G;
    return (b * p.Tq + p.t_off + qi) * p.Hq + kvh * p.G + g;
}
__device__ __forceinline__ size_t partial_row(const AttnParams &p, size_t slot, int kvh, int c) {
    if (p.T == 1) return slot * p.Hq + kvh * p.G + c;
    const int qi = c / p.G, g = c - qi * p.G;
    return (slot * p.T + qi) * p.Hq + kvh * p.G + g;
}

__device__ __forceinline__ float bf16_bits_to_float(uint32_t bits16) { return __uint_as_float(bits16 << 16); }

__device__ __forceinline__ uint16_t float_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);   // NaN stays NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Loads of data that is read once (the KV cache in a decode step): marked non-temporal, so that the stream does not
// displace what the caches hold for others.  Measured on the thinker batch: 54 instead of 59 us for the attention kernel.
__device__ __forceinline__ uint4 nt_load16(const void *p) {
    typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
    const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void nt_store16(void *p, const uint4 &v) {
    typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
    const u32x4_t w = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(w, reinterpret_cast<u32x4_t *>(p));
}
__device__ __forceinline__ uint2 nt_load8(const void *p) {
    typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
    const u32x2_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x2_t *>(p));
    return make_uint2(v.x, v.y);
}

// LDS exchange area for the four waves of a workgroup: per wave an unnormalised output tile [kMaxGroup][D + 4]
// (the +4 floats of padding spread the rows of different heads over different banks) and (m, l) per head.
template <int D>
struct CombineSmem {
    float o[kWaves][kMaxGroup][D + 4];
    float m[kWaves][kMaxGroup];
    float l[kWaves][kMaxGroup];
};

__device__ __forceinline__ void store_out(const AttnParams &p, size_t index, float v) {
    if (p.out_bf16) reinterpret_cast<uint16_t *>(p.out)[index] = float_to_bf16_rne(v);
    else reinterpret_cast<float *>(p.out)[index] = v;
}
// Four consecutive output elements in one store (index a multiple of four).
__device__ __forceinline__ void store_out4(const AttnParams &p, size_t index, const float4 &r) {
    if (p.out_bf16) {
        uint2 pk;
        pk.x = (uint32_t)float_to_bf16_rne(r.x) | ((uint32_t)float_to_bf16_rne(r.y) << 16);
        pk.y = (uint32_t)float_to_bf16_rne(r.z) | ((uint32_t)float_to_bf16_rne(r.w) << 16);
        *reinterpret_cast<uint2 *>(reinterpret_cast<uint16_t *>(p.out) + index) = pk;
    } else {
        *reinterpret_cast<float4 *>(reinterpret_cast<float *>(p.out) + index) = r;
    }
}

// One element of a finished segment: the normalised output if the request lies inside one range, else the
// unnormalised value (plus, once per head, the running max and sum) into the segment's partial-result slot.  The
// merge kernel that follows in the stream puts the slots of a request together; the kernel boundary between the two
// is what makes rows written on one compute die visible to a workgroup running on another (their L2 caches are not
// coherent with each other, and doing the exchange inside one kernel needs device-scope release/acquire fences that
// write back and invalidate a whole L2: measured at +40 % kernel time, and without them stale rows were observed).
template <int D>
__device__ __forceinline__ void store_segment_element(const AttnParams &p, const Segment &seg, int head0, int idx,
                                                      float M, float num, float den) {
    if (seg.nparts == 1) {
        store_out(p, ((size_t)seg.b * p.Hq + head0) * D + idx, den > 0.f ? num / den : 0.f);
    } else {
        const size_t pi = (size_t)seg.slot * p.Hq + head0;
        p.ws.part_o[pi * D + idx] = num;
        if (idx % D == 0) p.ws.part_ml[pi + idx / D] = make_float2(M, den);
    }
}

// Combine the four waves' (m, l, o) of one segment and store it: the part between the barriers.  All 256 threads
// call it once the waves' states in `sm` are visible.
template <int D>
__device__ __forceinline__ void wg_combine_segment(const CombineSmem<D> &sm, const AttnParams &p, const Segment &seg,
                                                   int kvh) {
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
        store_segment_element<D>(p, seg, head0, idx, M, num, den);
    }
}

// The same with the synchronisation around it: waits until the waves have filled `sm`, and returns when `sm` may be
// refilled.
template <int D>
__device__ __forceinline__ void wg_combine_and_store(CombineSmem<D> &sm, const AttnParams &p, const Segment &seg,
                                                     int kvh) {
    lds_barrier();
    wg_combine_segment<D>(sm, p, seg, kvh);
    lds_barrier();
}

// The all-zero output rows of an empty request for the columns of one KV head, written by the 64 lanes of a wave
// together, four elements per lane and store.
template <int D>
__device__ __forceinline__ void wave_zero_rows(const AttnParams &p, int b, int kvh) {
    for (int idx = 4 * (int)(threadIdx.x & 63); idx < p.Gq * D; idx += 4 * 64) {
        const int c = idx / D, d = idx - c * D;
        const size_t at = out_row(p, b, kvh, c) * D + d;
        if (p.out_bf16) *reinterpret_cast<uint2 *>(reinterpret_cast<uint16_t *>(p.out) + at) = make_uint2(0u, 0u);
        else *reinterpret_cast<float4 *>(reinterpret_cast<float *>(p.out) + at) = make_float4(0.f, 0.f, 0.f, 0.f);
    }
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
        if (w == 0) wave_zero_rows<D>(p, b, kvh);
    }, first_len, have_first);
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        const unsigned long long T = ps->total_tokens;
        p.ws.plan_words[0] = pl.S * kTile; p.ws.plan_words[1] = pl.nranges;
        p.ws.plan_words[2] = (int)(T & 0xffffffffULL); p.ws.plan_words[3] = (int)(T >> 32);
    }
    return pl;
}

// What the merge kernel needs to know of every request: its first partial-result slot and the number of ranges that
// touch it (0: no tile, 1: finished by the attention kernel).  Written by the grid's first workgroup when its own
// work is done (all 256 threads call this; E[] is the plan's array in shared memory), so that the merge kernel's
// workgroups, one per request and KV head, neither scan the lengths nor divide: one 8-byte read each.
__device__ __forceinline__ void write_merge_records(const AttnParams &p, const Plan &pl, const int *E) {
    for (int b = threadIdx.x; b < p.plan.B; b += kThreads) {
        const int e0 = E[b], e1 = E[b + 1];
        const int first_range = e0 / pl.S;
        p.ws.merge_rec[b] = make_int2(first_range + b, e1 > e0 ? (e1 - 1) / pl.S - first_range + 1 : 0);
    }
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
    if (blockIdx.x == 0) write_merge_records(p, pl, E);
}

}  // namespace omni
