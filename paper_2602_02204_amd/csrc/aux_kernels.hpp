// KV append and the debug gather.
#pragma once
#include "common.hpp"

namespace omni {

struct AppendParams {
    const void *k_new, *v_new;
    void *k_cache, *v_cache;
    const int32_t *block_table, *positions;
    int B, Hkv, MB, log2_ps;
    int row_vecs;                    // 16-byte vectors per row (D * elem_size / 16)
    int positions_are_lengths;       // positions[] holds context lengths: append at length - 1
};

// One thread per 16 bytes of one (request, KV head) row; K and V rows are copied bit for bit.
__global__ __launch_bounds__(kThreads) void kv_append_kernel(AppendParams p) {
    const long long idx = (long long)blockIdx.x * kThreads + threadIdx.x;
    const long long total = (long long)p.B * p.Hkv * p.row_vecs;
    if (idx >= total) return;
    const int c = (int)(idx % p.row_vecs);
    const long long row = idx / p.row_vecs;
    const int g = (int)(row % p.Hkv), b = (int)(row / p.Hkv);
    const int pos = p.positions[b] - (p.positions_are_lengths ? 1 : 0);
    if (pos < 0) return;
    const int page = p.block_table[(size_t)b * p.MB + (pos >> p.log2_ps)];
    const int slot = pos & ((1 << p.log2_ps) - 1);
    const size_t dst = ((((size_t)page * p.Hkv + g) << p.log2_ps) + slot) * p.row_vecs + c;
    const size_t src = (size_t)row * p.row_vecs + c;
    reinterpret_cast<uint4 *>(p.k_cache)[dst] = reinterpret_cast<const uint4 *>(p.k_new)[src];
    reinterpret_cast<uint4 *>(p.v_cache)[dst] = reinterpret_cast<const uint4 *>(p.v_new)[src];
}

struct GatherParams {
    const void *cache;
    const int32_t *block_table, *context_lens;
    void *dense_out;
    int request, Hkv, MB, log2_ps, row_vecs;
};

// dense_out[t, g, :] = cache row of token t of the request, KV head g.
__global__ __launch_bounds__(kThreads) void gather_kernel(GatherParams p) {
    const long long idx = (long long)blockIdx.x * kThreads + threadIdx.x;
    const int L = p.context_lens[p.request];
    const long long total = (long long)L * p.Hkv * p.row_vecs;
    if (idx >= total) return;
    const int c = (int)(idx % p.row_vecs);
    const long long row = idx / p.row_vecs;
    const int g = (int)(row % p.Hkv), t = (int)(row / p.Hkv);
    const int page = p.block_table[(size_t)p.request * p.MB + (t >> p.log2_ps)];
    const int slot = t & ((1 << p.log2_ps) - 1);
    const size_t src = ((((size_t)page * p.Hkv + g) << p.log2_ps) + slot) * p.row_vecs + c;
    reinterpret_cast<uint4 *>(p.dense_out)[idx] = reinterpret_cast<const uint4 *>(p.cache)[src];
}

}  // namespace omni
