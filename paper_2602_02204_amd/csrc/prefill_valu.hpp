// Vector-ALU kernel for multi-token queries over the paged cache: every dtype and head size the library knows
// (fp32 / bf16, head_dim 64 / 128).  It is the fp32-exact path of the multi-token call (tolerance 1e-5 on fp32
// caches) and the fallback where the matrix-core kernel does not apply; it is not tuned.
//
// A wave owns one query token of one (request, KV head) and walks the token's whole context, four tokens at a time:
// lane group tg = lane / 16 takes token t + tg, and the 16 lanes of a group each hold D / 16 consecutive dims of the
// K / V row.  The G query heads of the group are done in passes of up to four heads (the rows are read again per
// pass), each lane group keeping one online-softmax state (m, l, o) per head; the four groups are merged at the end.
#pragma once
#include "prefill_mfma.hpp"

namespace omni {

constexpr int kPrefillValuHeads = 4;                  // query heads per pass over the context

template <typename T, int E>
__device__ __forceinline__ void load_row_slice(const char *row, int c, float (&x)[E]) {
    if constexpr (sizeof(T) == 4) {
#pragma unroll
        for (int v = 0; v < E / 4; ++v) {
            const float4 f = *reinterpret_cast<const float4 *>(row + (size_t)(c * E + 4 * v) * 4);
            x[4 * v] = f.x; x[4 * v + 1] = f.y; x[4 * v + 2] = f.z; x[4 * v + 3] = f.w;
        }
    } else if constexpr (E == 8) {
        const uint4 u = *reinterpret_cast<const uint4 *>(row + (size_t)c * 16);
        const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
        for (int v = 0; v < 4; ++v) { x[2 * v] = bf16_bits_to_float(w[v] & 0xffffu); x[2 * v + 1] = __uint_as_float(w[v] & 0xffff0000u); }
    } else {
        const uint2 u = *reinterpret_cast<const uint2 *>(row + (size_t)c * 8);
        x[0] = bf16_bits_to_float(u.x & 0xffffu); x[1] = __uint_as_float(u.x & 0xffff0000u);
        x[2] = bf16_bits_to_float(u.y & 0xffffu); x[3] = __uint_as_float(u.y & 0xffff0000u);
    }
}

template <typename T, int D>
__global__ __launch_bounds__(kThreads) void prefill_valu_kernel(PrefillParams p, int log2_ps) {
    constexpr int E = D / 16;                                    // dims per lane
    constexpr int HC = kPrefillValuHeads;
    const int b = blockIdx.z, kvh = blockIdx.y;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 15, tg = lane >> 4;
    const int L = p.context_lens[b];
    const int n_q = min(p.q_lens[b], L);
    const int qi = blockIdx.x * kWaves + wave;                   // query token inside the chunk
    if (qi >= min(n_q, p.max_q_len)) return;                     // a chunk longer than the grid's bound is cut off there
    const int pos = L - n_q + qi;                                // attends to tokens 0 .. pos
    const size_t q_row = (size_t)(p.q_offsets[b] + qi);
    const int ps = 1 << log2_ps;
    const size_t row_bytes = (size_t)D * sizeof(T);
    const size_t page_stride = (size_t)p.Hkv * ps * row_bytes;
    const char *kbase = reinterpret_cast<const char *>(p.k_cache) + (size_t)kvh * ps * row_bytes;
    const char *vbase = reinterpret_cast<const char *>(p.v_cache) + (size_t)kvh * ps * row_bytes;
    const int32_t *bt = p.block_table + (size_t)b * p.MB;

    for (int g0 = 0; g0 < p.G; g0 += HC) {
        const int nh = min(HC, p.G - g0);
        float q[HC][E], o[HC][E], m[HC], l[HC];
#pragma unroll
        for (int h = 0; h < HC; ++h) {
            m[h] = -INFINITY; l[h] = 0.f;
#pragma unroll
            for (int e = 0; e < E; ++e) { q[h][e] = 0.f; o[h][e] = 0.f; }
            if (h < nh)
                load_row_slice<T, E>(reinterpret_cast<const char *>(p.q) + (q_row * p.Hq + kvh * p.G + g0 + h) * row_bytes, c, q[h]);
        }
        for (int t0 = 0; t0 <= pos; t0 += 4) {
            const int t = t0 + tg;
            if (t > pos) continue;                               // lanes of a group stay together
            const size_t off = (size_t)bt[t >> log2_ps] * page_stride + (size_t)(t & (ps - 1)) * row_bytes;
            float k[E], v[E];
            load_row_slice<T, E>(kbase + off, c, k);
            load_row_slice<T, E>(vbase + off, c, v);
#pragma unroll
            for (int h = 0; h < HC; ++h) {
                float s = 0.f;
#pragma unroll
                for (int e = 0; e < E; ++e) s = fmaf(q[h][e], k[e], s);
                s += __shfl_xor(s, 1); s += __shfl_xor(s, 2); s += __shfl_xor(s, 4); s += __shfl_xor(s, 8);
                s *= p.scale_log2;
                const float mn = fmaxf(m[h], s);
                const float a = fast_exp2(m[h] - mn);            // exp2(-inf) = 0 on the first token
                const float w = fast_exp2(s - mn);
                l[h] = l[h] * a + w;
#pragma unroll
                for (int e = 0; e < E; ++e) o[h][e] = fmaf(w, v[e], o[h][e] * a);
                m[h] = mn;
            }
        }
        // merge the four lane groups (a group that saw no token has m = -inf, l = 0)
#pragma unroll
        for (int h = 0; h < HC; ++h) {
#pragma unroll
            for (int d = 16; d <= 32; d <<= 1) {
                const float mo = __shfl_xor(m[h], d), lo = __shfl_xor(l[h], d);
                const float M = fmaxf(m[h], mo);
                const float a = m[h] > -INFINITY ? fast_exp2(m[h] - M) : 0.f;
                const float bsc = mo > -INFINITY ? fast_exp2(mo - M) : 0.f;
                l[h] = l[h] * a + lo * bsc;
#pragma unroll
                for (int e = 0; e < E; ++e) o[h][e] = o[h][e] * a + __shfl_xor(o[h][e], d) * bsc;
                m[h] = M;
            }
            if (h < nh && tg == 0) {                             // pos >= 0: at least one token, l > 0
                const float inv = 1.f / l[h];
                const size_t at = (q_row * p.Hq + kvh * p.G + g0 + h) * D + (size_t)c * E;
#pragma unroll
                for (int e = 0; e < E; ++e) {
                    const float r = o[h][e] * inv;
                    if (p.out_bf16) reinterpret_cast<uint16_t *>(p.out)[at + e] = float_to_bf16_rne(r);
                    else reinterpret_cast<float *>(p.out)[at + e] = r;
                }
            }
        }
    }
}

}  // namespace omni
