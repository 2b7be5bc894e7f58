// Log-sum-exp merge of split requests, KV append, and the debug gather.
#pragma once
#include "common.hpp"

namespace omni {

// Merge kernel: one workgroup per (request, KV head), launched right after the attention kernel.  It takes the
// request's first slot and number of pieces from the records the attention kernel's first workgroup left in the
// workspace (one 8-byte read; scanning the lengths again in every workgroup and dividing by the range length cost
// 0.5 us more at 256 requests and 10 - 28 us at 1024 - 2048); for a request that was cut
// by range boundaries combines its partial-result slots, in slot order:
//     out = sum_j 2^(m_j - M) o_j / sum_j 2^(m_j - M) l_j,   M = max_j m_j,   pieces with l_j = 0 skipped.
// Requests inside one range (finished by the attention kernel) and empty requests return at once.
// Every thread owns four consecutive output elements (one 16-byte load per piece); the loads of kRound pieces are
// issued before any is used, so a round costs one trip to memory and no load depends on a loaded value.
template <int D, int kRound>
__device__ __forceinline__ void merge_request(const AttnParams &p, int b, int kvh, int slot_first, int n) {
    for (int idx = 4 * threadIdx.x; idx < p.Gq * D; idx += 4 * kThreads) {    // one pass up to 1024 elements
        const int g = idx / D;                                                // column: (query token, head)
        const size_t out0 = out_row(p, b, kvh, g) * D + (idx - g * D);
        float M = -INFINITY, den = 0.f;
        float4 num = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int j0 = 0; j0 < n; j0 += kRound) {
            float2 ml[kRound];
            float4 oj[kRound];
#pragma unroll
            for (int u = 0; u < kRound; ++u) {
                ml[u] = make_float2(0.f, 0.f); oj[u] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (j0 + u < n) {
                    const size_t pi = partial_row(p, slot_first + j0 + u, kvh, g);
                    ml[u] = p.ws.part_ml[pi];
                    oj[u] = *reinterpret_cast<const float4 *>(p.ws.part_o + pi * D + (idx - g * D));
                }
            }
#pragma unroll
            for (int u = 0; u < kRound; ++u) {
                if (ml[u].y > 0.f) {
                    const float Mn = fmaxf(M, ml[u].x);
                    const float a = fast_exp2(M - Mn);               // 0 while M is still -inf
                    const float w = fast_exp2(ml[u].x - Mn);
                    num.x = num.x * a + w * oj[u].x; num.y = num.y * a + w * oj[u].y;
                    num.z = num.z * a + w * oj[u].z; num.w = num.w * a + w * oj[u].w;
                    den = den * a + w * ml[u].y;
                    M = Mn;
                }
            }
        }
        const bool live = den > 0.f;
        store_out4(p, out0, make_float4(live ? num.x / den : 0.f, live ? num.y / den : 0.f, live ? num.z / den : 0.f,
                                        live ? num.w / den : 0.f));
    }
}

template <int D>
__global__ __launch_bounds__(kThreads) void merge_kernel(AttnParams p) {
    const int b = blockIdx.x / p.Hkv, kvh = blockIdx.x - b * p.Hkv;
    const int2 rec = p.ws.merge_rec[b];                      // first slot and number of pieces, from the attention kernel
    const int n = __builtin_amdgcn_readfirstlane(rec.y);
    if (n < 2) return;                                       // no tile (its zero row is written) or finished already
    const int slot_first = __builtin_amdgcn_readfirstlane(rec.x);
    // 4, 8 or 16 pieces per round, so that a request cut into many pieces still costs few dependent trips to memory
    if (n <= 4) merge_request<D, 4>(p, b, kvh, slot_first, n);
    else if (n <= 8) merge_request<D, 8>(p, b, kvh, slot_first, n);
    else merge_request<D, 16>(p, b, kvh, slot_first, n);
}

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

struct AppendQuantParams {
    const void *k_new, *v_new;       // bf16 [B, Hkv, 128]
    void *k_cache, *v_cache;         // E4M3 bytes [P, Hkv, ps, 128]
    float *k_scale, *v_scale;        // [P, Hkv]
    const int32_t *block_table, *positions;
    float headroom;
    int B, Hkv, MB, log2_ps;
};

// Quantising append into an 8-bit cache: 16 lanes per row of 128 bf16 values (8 each), the K rows first, then the V
// rows.  A row at slot 0 opens its page and fixes the page's scale for its KV head, max(amax * headroom, 2^-100) / 448
// (amax over the row by cross-lane maxima); any other row takes the scale its page has.  Bytes: x / scale (one
// correctly rounded fp32 division), clamped to +-448, converted by the hardware's round-to-nearest-even E4M3 conversion;
// NaN becomes the byte 0x7f.
__global__ __launch_bounds__(kThreads) void kv_append_quant_kernel(AppendQuantParams p) {
    constexpr int D = 128;
    const long long t = (long long)blockIdx.x * kThreads + threadIdx.x;
    const long long rows = (long long)p.B * p.Hkv;
    const long long row2 = t >> 4;
    const int c = (int)(t & 15);
    const bool in_grid = row2 < 2 * rows;
    const bool is_v = row2 >= rows;
    const long long row = in_grid ? row2 - (is_v ? rows : 0) : 0;
    const int g = (int)(row % p.Hkv), b = (int)(row / p.Hkv);
    const int pos = in_grid ? p.positions[b] : -1;
    const bool live = pos >= 0;
    float x[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) x[i] = 0.f;
    if (live) {
        const uint4 raw = *(reinterpret_cast<const uint4 *>(is_v ? p.v_new : p.k_new) + row * (D / 8) + c);
        const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) { x[2 * i] = bf16_bits_to_float(w[i] & 0xffffu); x[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u); }
    }
    float amax = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) amax = fmaxf(amax, fabsf(x[i]));             // a NaN element never raises the maximum
#pragma unroll
    for (int off = 1; off < 16; off <<= 1) amax = fmaxf(amax, __shfl_xor(amax, off));
    if (!live) return;
    const int page = p.block_table[(size_t)b * p.MB + (pos >> p.log2_ps)];
    const int slot = pos & ((1 << p.log2_ps) - 1);
    float *scales = is_v ? p.v_scale : p.k_scale;
    const size_t si = (size_t)page * p.Hkv + g;
    float sc;
    if (slot == 0) {
        float top = amax * p.headroom;
        if (!(top > 0x1p-100f)) top = 0x1p-100f;
        sc = top / 448.0f;
        if (c == 0) scales[si] = sc;
    } else {
        sc = scales[si];
    }
    uint32_t out[2];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float a = fminf(fmaxf(x[2 * i] / sc, -448.0f), 448.0f), bq = fminf(fmaxf(x[2 * i + 1] / sc, -448.0f), 448.0f);
        uint32_t pk = (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(a, bq, 0, false) & 0xffffu;
        if (x[2 * i] != x[2 * i]) pk = (pk & 0xff00u) | 0x7fu;
        if (x[2 * i + 1] != x[2 * i + 1]) pk = (pk & 0x00ffu) | 0x7f00u;
        if (i & 1) out[i >> 1] |= pk << 16; else out[i >> 1] = pk;
    }
    char *dst = reinterpret_cast<char *>(is_v ? p.v_cache : p.k_cache) + ((((size_t)page * p.Hkv + g) << p.log2_ps) + slot) * D + c * 8;
    *reinterpret_cast<uint2 *>(dst) = make_uint2(out[0], out[1]);
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

struct PackParams {
    const void *k_src, *v_src;       // pack: the pools; unpack: the dense buffers
    void *k_dst, *v_dst;             // pack: the dense buffers; unpack: the pools
    const int32_t *block_table, *context_lens;
    const long long *token_offsets;  // first dense row of each request; < 0: skip the request
    const int32_t *q_lens;           // null: whole requests; else only the last q_lens[b] tokens of each request move,
                                     // and dense row token_offsets[b] holds the first of them
    int max_tokens;                  // with q_lens: at most this many tokens of a request move (the grid's bound)
    int Hkv, MB, log2_ps, row_vecs;
};

constexpr int kPackTokens = 32;      // tokens per workgroup

// Dense <-> paged copy of whole requests, bit for bit.  Workgroup (x, b) moves tokens [32x, 32x + 32) of request b:
// dense row (token_offsets[b] + t) holds the Hkv rows of token t back to back, the pool keeps them in page
// block_table[b][t / ps], slot t % ps.  A thread moves 16-byte pieces, two of K and two of V in flight at a time
// (more per thread, or more tokens per workgroup, measured slower: 4.6 TB/s read + written at 32 tokens and two
// pieces against 3.2 at eight pieces).
// Consecutive threads take consecutive pieces of the dense side, so dense traffic is fully coalesced and pool traffic
// comes in whole 256- or 512-byte rows.
template <bool kUnpack>
__global__ __launch_bounds__(kThreads) void kv_pack_kernel(PackParams p) {
    constexpr int kU = 2;                                    // pieces of K and of V a thread keeps in flight
    const int b = blockIdx.y;
    const int L = p.context_lens[b];
    const int n_move = p.q_lens ? max(0, min(p.q_lens[b], L)) : L;
    const int first = L - n_move;                                          // first token that moves
    const int end = p.q_lens ? first + min(n_move, p.max_tokens) : L;      // one past the last (a longer chunk is cut off)
    const int t0 = first + blockIdx.x * kPackTokens;
    const long long off = p.token_offsets[b] - first;                      // dense row of token 0 (may be virtual)
    if (p.token_offsets[b] < 0 || t0 >= end) return;
    const int log2_rv = 31 - __clz(p.row_vecs);              // row_vecs is 8, 16 or 32
    const int vecs_per_token = p.Hkv << log2_rv;
    const int total = min(kPackTokens, end - t0) * vecs_per_token;
    const int32_t *bt = p.block_table + (size_t)b * p.MB;
    const uint4 *ks = reinterpret_cast<const uint4 *>(p.k_src), *vs = reinterpret_cast<const uint4 *>(p.v_src);
    uint4 *kd = reinterpret_cast<uint4 *>(p.k_dst), *vd = reinterpret_cast<uint4 *>(p.v_dst);
    for (int i0 = threadIdx.x; i0 < total; i0 += kU * kThreads) {
        size_t src[kU], dst[kU];
        uint4 kv[kU], vv[kU];
#pragma unroll
        for (int u = 0; u < kU; ++u) {
            const int i = i0 + u * kThreads;
            src[u] = dst[u] = 0;
            if (i < total) {
                const int tok = i / vecs_per_token, r = i - tok * vecs_per_token;
                const int g = r >> log2_rv, c = r & (p.row_vecs - 1);
                const int t = t0 + tok;
                const int page = bt[t >> p.log2_ps], slot = t & ((1 << p.log2_ps) - 1);
                const size_t paged = (((((size_t)page * p.Hkv + g) << p.log2_ps) + slot) << log2_rv) + c;
                const size_t dense = (size_t)(off + t) * vecs_per_token + r;
                src[u] = kUnpack ? dense : paged;
                dst[u] = kUnpack ? paged : dense;
            }
        }
#pragma unroll
        for (int u = 0; u < kU; ++u)
            if (i0 + u * kThreads < total) { kv[u] = nt_load16(ks + src[u]); vv[u] = nt_load16(vs + src[u]); }
#pragma unroll
        for (int u = 0; u < kU; ++u)
            if (i0 + u * kThreads < total) {
                // measured: scattered 4 KB pieces into the pools go faster as non-temporal stores, a dense buffer does not
                if (kUnpack) { nt_store16(kd + dst[u], kv[u]); nt_store16(vd + dst[u], vv[u]); }
                else { kd[dst[u]] = kv[u]; vd[dst[u]] = vv[u]; }
            }
    }
}

// Measurement aid: read two buffers front to back with 16-byte loads (each wave takes 4 KB pieces, two at a time,
// strided over the grid) and fold the words into a checksum nobody needs.  What this kernel reaches on a buffer of the
// KV pool's size is the memory system's ceiling for a kernel of that duration.
__global__ __launch_bounds__(kThreads) void stream_read_kernel(const uint4 *__restrict__ a, size_t a_vecs,
                                                               const uint4 *__restrict__ b, size_t b_vecs,
                                                               unsigned *sink) {
    const size_t lane = threadIdx.x & 63;
    const size_t gw = ((size_t)blockIdx.x * kThreads + threadIdx.x) >> 6, nw = ((size_t)gridDim.x * kThreads) >> 6;
    unsigned acc = 0;
    for (int which = 0; which < 2; ++which) {
        const uint4 *src = which ? b : a;
        const size_t vecs = which ? b_vecs : a_vecs;
        const size_t pieces = (vecs + 255) / 256;                 // 256 vectors = 4 KB
        for (size_t pc = gw * 2; pc < pieces; pc += nw * 2) {
            uint4 v[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const size_t idx = (pc + (i >> 2)) * 256 + (size_t)(i & 3) * 64 + lane;
                v[i] = idx < vecs ? nt_load16(src + idx) : make_uint4(0, 0, 0, 0);
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) acc += v[i].x ^ v[i].y ^ v[i].z ^ v[i].w;
        }
    }
    if (acc == 0x9e3779b9u) *sink = acc;                          // practically never: keeps the loads alive
}

}  // namespace omni
