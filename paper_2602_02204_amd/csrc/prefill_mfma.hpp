// Matrix-core attention kernel for multi-token queries over the paged cache (chunked prefill): bf16 q/K/V,
// head_dim 128, group size <= 16.  Query i of request b's chunk sits at position p = L_b - n_b + i and attends to
// tokens 0 .. p (causal inside the chunk).
//
// A workgroup (8 waves, two per SIMD) owns one (request, KV head, block of query tokens).  Its 256 "columns" are the
// (query token, query head of the group) pairs of that block in token-major order; a wave owns 32 consecutive ones =
// two 16-column MFMA blocks.  The same transposed products as in the decode kernel are used, per 32-token tile and
// per column block:
//   S^T = K Q^T     (A = K rows from shared memory, B = the block's queries, held in registers for the whole kernel)
//   O^T += V^T P^T  (A = V transposed, B = the softmax weights; both as fp16: V is converted once per workgroup on
//                    its way into shared memory, exactly for 2^-14 <= |V| <= 65504, and fp16 weights carry 11
//                    significant bits, so one product does what bf16 weights need a hi + lo pair for)
// so every lane owns one column: running reference, sum and rescale never cross lanes on the common path.
// What differs from decode is reuse: K/V tiles are fetched once per workgroup into shared memory (double buffered,
// one barrier per 64 tokens) and feed 16 column blocks, and V^T comes out of shared memory through transposing reads.
// That makes the path a dense contraction, not a stream.  The three pieces of a tile's work are software-pipelined
// across tiles, so that a wave has matrix-core and vector-ALU instructions to issue side by side; on this chip both
// kinds go through one issue port per SIMD, and the sum of the two instruction streams is what bounds the kernel.
#pragma once
#include <type_traits>

#include "decode_mfma.hpp"

namespace omni {

constexpr int kPrefillThreads = 512;                  // 8 waves = 2 per SIMD share one K/V tile in shared memory
constexpr int kPrefillWaves = kPrefillThreads / 64;
constexpr int kPrefillBlocks = 2;                     // 16-column MFMA blocks per wave
constexpr int kPrefillCols = 16 * kPrefillBlocks;     // (token, head) pairs per wave
constexpr int kPrefillRowBytes = 256 + 16;            // a 256-byte K row plus padding: conflict-free 16-byte LDS reads
constexpr int kPrefillVRowBytes = 256 + 32;           // V rows: conflict-free 8-byte transposing reads (4 rows x 32 B)
constexpr float kPrefillBias = 6.f;                   // a moved reference sits this many log2 units below the maximum
constexpr float kPrefillSumLimit = 32768.f;           // sum of a lane's 8 weights of a tile beyond which the reference moves

// Transposing 64-bit read from shared memory (see its use below for the lane arrangement).
__device__ __forceinline__ uint2 lds_read_tr16_b64(const char *p) {
    typedef short short4_t __attribute__((ext_vector_type(4)));
    const short4_t v = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (short4_t __attribute__((address_space(3))) *)(const __attribute__((address_space(3))) char *)p);
    return __builtin_bit_cast(uint2, v);
}

typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ f32x4_t mfma_f16(const uint4 &a, const uint4 &b, f32x4_t c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
}

typedef float f32x2_t __attribute__((ext_vector_type(2)));

// c + the two fp16 values packed in w, in fp32.
__device__ __forceinline__ float sum_f16x2(uint32_t w, float c) {
    const f16x2_t ones = {(_Float16)1.f, (_Float16)1.f};
    return __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2_t, w), ones, c, false);
}

// Two floats -> packed fp16, round to nearest even.
__device__ __forceinline__ uint32_t pack_f16x2(float lo, float hi) {
    const f32x2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2_t));
}

// Eight bf16 values -> eight fp16 values.  Exact wherever the value is a normal fp16 number (2^-14 <= |V| <= 65504);
// below that the spacing is 2^-24, i.e. an absolute error of at most 2^-25; above it the value becomes infinite and
// shows in the result.
__device__ __forceinline__ uint4 bf16x8_to_f16x8(const uint4 &v) {
    uint4 r;
    r.x = pack_f16x2(bf16_bits_to_float(v.x & 0xffffu), __uint_as_float(v.x & 0xffff0000u));
    r.y = pack_f16x2(bf16_bits_to_float(v.y & 0xffffu), __uint_as_float(v.y & 0xffff0000u));
    r.z = pack_f16x2(bf16_bits_to_float(v.z & 0xffffu), __uint_as_float(v.z & 0xffff0000u));
    r.w = pack_f16x2(bf16_bits_to_float(v.w & 0xffffu), __uint_as_float(v.w & 0xffff0000u));
    return r;
}

// Eight E4M3 bytes times a scale -> eight fp16 values: widened exactly (bf16, then fp32), scaled in fp32, rounded once.
__device__ __forceinline__ uint4 fp8x8_scaled_to_f16x8(uint32_t lo, uint32_t hi, float sc) {
    const uint4 v = fp8x8_to_bf16x8(lo, hi);
    uint4 r;
    r.x = pack_f16x2(bf16_bits_to_float(v.x & 0xffffu) * sc, __uint_as_float(v.x & 0xffff0000u) * sc);
    r.y = pack_f16x2(bf16_bits_to_float(v.y & 0xffffu) * sc, __uint_as_float(v.y & 0xffff0000u) * sc);
    r.z = pack_f16x2(bf16_bits_to_float(v.z & 0xffffu) * sc, __uint_as_float(v.z & 0xffff0000u) * sc);
    r.w = pack_f16x2(bf16_bits_to_float(v.w & 0xffffu) * sc, __uint_as_float(v.w & 0xffff0000u) * sc);
    return r;
}

struct PrefillParams {
    const void *q;                    // [Tq, Hq, D] bf16
    const void *k_cache, *v_cache;
    const float *k_scale, *v_scale;   // 8-bit cache only (else null): [P, Hkv] scales of the K and V pools
    const int32_t *block_table, *context_lens, *q_lens;
    const long long *q_offsets;
    void *out;                        // [Tq, Hq, D]
    float scale_log2;
    int Hq, Hkv, G, MB;
    int out_bf16;
    // Context split (matrix-core kernel): each workgroup's 64-token steps are dealt to num_splits workgroups, which
    // leave unnormalised rows and (reference, sum) per (request, query token < max_q_len, head, split) for the merge.
    int num_splits;                   // 1: no split, results go straight to out
    int min_split_steps;              // fewest 64-token steps a split's share may have
    int max_q_len;
    float *part_o;                    // [B, max_q_len, Hq, num_splits, D]
    float2 *part_ml;                  // [B, max_q_len, Hq, num_splits]
    const int32_t *order;             // null, or [B]: the requests by descending context length (blockIdx.z -> request)
    int B;
};

// A split's share of the context is at least this many 64-token steps: below that the pieces' trip through memory
// costs more than the extra workgroups bring.  Decided per query block on the device, where the lengths are known.
constexpr int kPrefillMinSplitTokens = 256;          // default; a tuning value
__device__ __forceinline__ int prefill_effective_splits(int num_splits, int n_steps, int min_split_steps) {
    return max(1, min(num_splits, n_steps / min_split_steps));
}

// Query tokens per workgroup for a group of G heads: its 256 columns are the (token, head) pairs in token-major order,
// cut into runs of 32 for the waves wherever that falls.
__host__ __device__ inline int prefill_tokens_per_block(int G) { return kPrefillWaves * kPrefillCols / G; }

// KV8: the pools hold 8-bit E4M3 bytes with one scale per (page, KV head).  The staging threads widen K to bf16
// (exact) and V times its page's scale to fp16 (one rounding, 2^-12 relative: the size of the weights' own rounding) on
// the way into shared memory, so the products are the 16-bit ones; the K scale of each 16-token half of a tile joins
// the softmax scale in the exponent's multiply-add.
template <int PS, bool KV8 = false>
__global__ __launch_bounds__(kPrefillThreads, 1) void prefill_mfma_kernel(PrefillParams p) {
    constexpr int D = 128;
    constexpr int ES = KV8 ? 1 : 2;                              // bytes per cache element
    constexpr int kLog2Ps = (PS == 16) ? 4 : 5;
    constexpr int kTileBytes = kTile * kPrefillVRowBytes;        // room for one K or V tile in shared memory
    __shared__ __align__(16) char smem[2][2][2][kTileBytes];     // [buffer][tile of the step][K, V]
    __shared__ float kscale_lds[2][2][2];                        // 8-bit cache: [buffer][tile][16-token half] K scales

    // Workgroups are dispatched in blockIdx order, z slowest: with the requests taken longest first the long-running
    // workgroups start first and the short ones fill the end of the launch.
    const int b = p.order ? p.order[blockIdx.z] : (int)blockIdx.z, kvh = blockIdx.y;
    const int G = p.G, head0 = kvh * G;
    const int L = p.context_lens[b];
    const int n_q = min(p.q_lens[b], L);
    const int n_live = min(n_q, p.max_q_len);                    // a chunk longer than the grid's bound is cut off there
    const int QB = prefill_tokens_per_block(G);
    const int NS = p.num_splits;
    const int split = NS > 1 ? (int)blockIdx.x % NS : 0;
    const int q0 = (NS > 1 ? (int)blockIdx.x / NS : (int)blockIdx.x) * QB;      // first query token of this workgroup
    if (n_live <= 0 || q0 >= n_live) return;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int col = lane & 15, j = lane >> 4;
    const long long q_row0 = p.q_offsets[b];
    const int pos0 = L - n_q;                                    // position of the chunk's first token
    const int wg_last = min(n_live, q0 + QB) - 1;                // last query token of the workgroup
    const int n_tiles = (pos0 + wg_last) / kTile + 1;            // tiles that hold tokens 0 .. position of wg_last

    // ---- this lane's columns (one per column block): query token, head, position; and the queries as MFMA B operands
    int pos[kPrefillBlocks];                                     // -1: padding column (never stored)
    uint4 Q[kPrefillBlocks][4];
    int wave_max_pos = -1;
#pragma unroll
    for (int cb = 0; cb < kPrefillBlocks; ++cb) {
        const int c = wave * kPrefillCols + cb * 16 + col;       // column of the workgroup
        const int tl = c / G, g = c - tl * G;
        const int qi = q0 + tl;                                  // query token inside the chunk
        const bool live = tl < QB && qi < n_live;
        pos[cb] = live ? pos0 + qi : -1;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) Q[cb][kk] = make_uint4(0, 0, 0, 0);
        if (live) {
            const char *qrow = reinterpret_cast<const char *>(p.q) + ((size_t)(q_row0 + qi) * p.Hq + head0 + g) * (D * 2);
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) Q[cb][kk] = *reinterpret_cast<const uint4 *>(qrow + (4 * kk + j) * 16);
        }
        wave_max_pos = max(wave_max_pos, pos[cb]);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) wave_max_pos = max(wave_max_pos, __shfl_xor(wave_max_pos, off));
    // the smallest live position of the wave: tiles that end at or before it need no mask
    int wave_min_pos = 0x7fffffff;
#pragma unroll
    for (int cb = 0; cb < kPrefillBlocks; ++cb) wave_min_pos = min(wave_min_pos, pos[cb] >= 0 ? pos[cb] : 0x7fffffff);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) wave_min_pos = min(wave_min_pos, __shfl_xor(wave_min_pos, off));

    // ---- staging: a step is 64 tokens = two 32-token tiles; thread t moves piece t of the 512 16-byte pieces of
    // each tile's K rows and V rows (piece = 16 * token + chunk).  The products below run as a pipeline in which V of a
    // tile is needed two tiles after its K, so V is fetched and staged one step behind K.
    const size_t page_stride = (size_t)p.Hkv * PS * D * ES;
    const char *kbase = reinterpret_cast<const char *>(p.k_cache) + (size_t)kvh * PS * D * ES;
    const char *vbase = reinterpret_cast<const char *>(p.v_cache) + (size_t)kvh * PS * D * ES;
    const int32_t *bt = p.block_table + (size_t)b * p.MB;
    const int st_tok = threadIdx.x >> 4, st_chunk = threadIdx.x & 15;       // token 0..31 of a tile
    const int lds_off = st_tok * kPrefillRowBytes + st_chunk * 16;
    const int lds_off_v = st_tok * kPrefillVRowBytes + st_chunk * 16;
    const int n_steps = (n_tiles + 1) >> 1;
    // this workgroup's share of the steps: [s_begin, s_end), all of them without a split.  The launch provides NS
    // workgroups per query block; how many of them share the work depends on the block's context.
    const int ns_eff = prefill_effective_splits(NS, n_steps, p.min_split_steps);
    if (split >= ns_eff) return;
    const int s_begin = (int)((long long)n_steps * split / ns_eff);
    const int s_end = (int)((long long)n_steps * (split + 1) / ns_eff);
    uint4 sk[2], sv_[2];                                         // 8-bit cache: 8 bytes each, in .x and .y
    float sks[2] = {1.f, 1.f}, svs[2] = {1.f, 1.f};             // 8-bit cache: the scales of the rows' pages
    // Page numbers are looked up one step before the rows they address are fetched, so that no fetch waits for its
    // own table entry: pg_k holds the pages of the step whose K rows are fetched next, pg_v (the same entries one
    // step later) those of the step whose V rows are fetched next.
    int pg_k[2], pg_v[2] = {0, 0};
    auto lookup = [&](int step) __attribute__((always_inline)) {
#pragma unroll
        for (int sub = 0; sub < 2; ++sub)                                   // an entry of the table for every lane
            pg_k[sub] = bt[min((2 * step + sub) * kTile + st_tok, L - 1) >> kLog2Ps];
    };
    auto fetch_rows = [&](auto fast, const char *base, const float *scale, int step, const int (&pg)[2], uint4 (&r)[2],
                          float (&sc)[2]) __attribute__((always_inline)) {
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
            const int t = (2 * step + sub) * kTile + st_tok;
            const char *src = base + (size_t)pg[sub] * page_stride + (size_t)(t & (PS - 1)) * (D * ES) + st_chunk * (8 * ES);
            const bool in = decltype(fast)::value || (step < s_end && t < L);
            r[sub] = make_uint4(0, 0, 0, 0);                                // rows beyond the context are zero
            if constexpr (KV8) {
                if (in) {
                    const uint2 v = *reinterpret_cast<const uint2 *>(src);
                    r[sub].x = v.x; r[sub].y = v.y;
                }
                sc[sub] = scale[(size_t)pg[sub] * p.Hkv];                   // the page is a valid one also beyond the context
            } else {
                if (in) r[sub] = *reinterpret_cast<const uint4 *>(src);
            }
        }
    };
    auto stage_k = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
            if constexpr (KV8) {
                *reinterpret_cast<uint4 *>(&smem[buf][sub][0][lds_off]) = fp8x8_to_bf16x8(sk[sub].x, sk[sub].y);
                if (st_chunk == 0 && (st_tok & 15) == 0) kscale_lds[buf][sub][st_tok >> 4] = sks[sub];
            } else {
                *reinterpret_cast<uint4 *>(&smem[buf][sub][0][lds_off]) = sk[sub];
            }
        }
    };
    auto stage_v = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
            if constexpr (KV8)
                *reinterpret_cast<uint4 *>(&smem[buf][sub][1][lds_off_v]) = fp8x8_scaled_to_f16x8(sv_[sub].x, sv_[sub].y, svs[sub]);
            else
                *reinterpret_cast<uint4 *>(&smem[buf][sub][1][lds_off_v]) = bf16x8_to_f16x8(sv_[sub]);
        }
    };

    // ---- per-column online-softmax state
    float m[kPrefillBlocks], l[kPrefillBlocks];
    f32x4_t acc[kPrefillBlocks][8];
#pragma unroll
    for (int cb = 0; cb < kPrefillBlocks; ++cb) {
        m[cb] = -INFINITY; l[cb] = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[cb][e] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    }
    // A tile of this workgroup's steps that holds tokens some column of this wave sees.
    auto tile_active = [&](int t) { return t >= 2 * s_begin && t < 2 * s_end && t * kTile <= wave_max_pos; };

    // ---- the three pieces of a tile's work
    // Raw scores q.k of the column blocks: S[cb][h] holds tokens 16 h + 4 j .. + 3 of the tile for column `col`.  The
    // softmax scale is applied inside the exponent (one fused multiply-add per score): scale > 0, so the order of
    // scores is that of the raw dot products.
    auto scores = [&](const char *ks, f32x4_t (&S)[kPrefillBlocks][2], const float *ksc, float (&a)[2]) __attribute__((always_inline)) {
        if constexpr (KV8) {                                     // read with the rows: both are replaced together
            a[0] = ksc[0] * p.scale_log2; a[1] = ksc[1] * p.scale_log2;
        }
        uint4 K[8];
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            K[kk] = *reinterpret_cast<const uint4 *>(ks + col * kPrefillRowBytes + (4 * kk + j) * 16);
            K[4 + kk] = *reinterpret_cast<const uint4 *>(ks + (16 + col) * kPrefillRowBytes + (4 * kk + j) * 16);
        }
#pragma unroll
        for (int cb = 0; cb < kPrefillBlocks; ++cb) {
            S[cb][0] = f32x4_t{0.f, 0.f, 0.f, 0.f}; S[cb][1] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
#pragma unroll
            for (int cb = 0; cb < kPrefillBlocks; ++cb) {
                S[cb][0] = mfma_bf16(K[kk], Q[cb][kk], S[cb][0]);
                S[cb][1] = mfma_bf16(K[4 + kk], Q[cb][kk], S[cb][1]);
            }
        }
    };
    // Weights of tile t from its raw scores: P[cb] as one fp16 MFMA operand.  A column's reference m (log2 domain) is
    // moved only when a weight would leave the fp16 range, which shows in the sum of the tile's weights: any common
    // reference gives the same softmax.  A move puts m at the running maximum less the bias, so the largest weight of a
    // column then lies between 2^bias and the limit, and a weight loses precision as an fp16 subnormal only when it is
    // 2^-20 of the largest or less.  After a column's first tiles moves are rare, so the maximum over the tile, its
    // exchange between the four lane groups of a column and the rescale of what was summed under the old reference
    // leave the common path.  The sums are taken over the rounded weights, the ones the matrix cores multiply.
    auto weights = [&](auto fast, int t, f32x4_t (&S)[kPrefillBlocks][2], uint4 (&P)[kPrefillBlocks], const float (&a)[2]) __attribute__((always_inline)) {
        const int tb = t * kTile;
        if constexpr (!decltype(fast)::value) {
            if (tb + kTile - 1 > wave_min_pos) {                 // tokens after the column's position
#pragma unroll
                for (int cb = 0; cb < kPrefillBlocks; ++cb)
#pragma unroll
                    for (int r = 0; r < 8; ++r)
                        if (tb + slot_token(j, r) > pos[cb]) S[cb][r >> 2][r & 3] = -INFINITY;
            }
        }
        float psum[kPrefillBlocks];
        auto form = [&](int cb) __attribute__((always_inline)) {
            float pw[8];
#pragma unroll
            for (int r = 0; r < 8; ++r) pw[r] = fast_exp2(fmaf(S[cb][r >> 2][r & 3], KV8 ? a[r >> 2] : p.scale_log2, -m[cb]));
            P[cb] = make_uint4(pack_f16x2(pw[0], pw[1]), pack_f16x2(pw[2], pw[3]), pack_f16x2(pw[4], pw[5]),
                               pack_f16x2(pw[6], pw[7]));
            psum[cb] = sum_f16x2(P[cb].w, sum_f16x2(P[cb].z, sum_f16x2(P[cb].y, sum_f16x2(P[cb].x, 0.f))));
        };
        bool over = false;
#pragma unroll
        for (int cb = 0; cb < kPrefillBlocks; ++cb) {
            form(cb);
            over |= !(psum[cb] < kPrefillSumLimit);              // also true for an infinite or undefined sum
        }
        if (__any(over)) {
#pragma unroll
            for (int cb = 0; cb < kPrefillBlocks; ++cb) {
                const float t0 = fmaxf(fmaxf(S[cb][0][0], S[cb][0][1]), fmaxf(S[cb][0][2], S[cb][0][3]));
                const float t1 = fmaxf(fmaxf(S[cb][1][0], S[cb][1][1]), fmaxf(S[cb][1][2], S[cb][1][3]));
                // the largest scaled score of the tile, in log2 units (scales are positive)
                float tmax = KV8 ? fmaxf(t0 * a[0], t1 * a[1]) : fmaxf(t0, t1) * p.scale_log2;
                tmax = fmaxf(tmax, __shfl_xor(tmax, 16));
                tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
                // a column whose tokens are all masked so far keeps a finite stand-in: exp2 then sees -inf - finite
                const float mn = fmaxf(fmaxf(m[cb], tmax - kPrefillBias), -1e30f);
                const float alpha = fast_exp2(m[cb] - mn);       // 0 while m is still -inf
                l[cb] *= alpha;
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[cb][e] *= alpha;
                m[cb] = mn;
                form(cb);
            }
        }
#pragma unroll
        for (int cb = 0; cb < kPrefillBlocks; ++cb) l[cb] += psum[cb];
    };
    // O^T += V^T P^T.  The V^T operands, shared by the column blocks, come transposed out of shared memory: in a
    // transposing 8-byte read the 16 lanes of a group each name four consecutive 16-bit values (lane 4k + q: dims
    // 4q .. 4q+3 of token k of the group's four tokens) and lane i receives value i of each token, i.e. one output dim
    // for four tokens.  Two reads (tokens 4j .. 4j+3 and 16+4j .. 16+4j+3, exactly the tokens whose weights this lane
    // group holds) make the operand of one 16-dim block of output rows.
    auto pv = [&](const char *vs, const uint4 (&P)[kPrefillBlocks]) __attribute__((always_inline)) {
        const char *v_lo = vs + (4 * j + (col >> 2)) * kPrefillVRowBytes + (col & 3) * 8;
        const char *v_hi = v_lo + 16 * kPrefillVRowBytes;
#pragma unroll
        for (int eb = 0; eb < 8; ++eb) {
            const uint2 a0 = lds_read_tr16_b64(v_lo + eb * 32);
            const uint2 a1 = lds_read_tr16_b64(v_hi + eb * 32);
            const uint4 A = make_uint4(a0.x, a0.y, a1.x, a1.y);
#pragma unroll
            for (int cb = 0; cb < kPrefillBlocks; ++cb) acc[cb][eb] = mfma_f16(A, P[cb], acc[cb][eb]);
        }
    };
    // ---- the pipeline.  Phase t multiplies the weights of tile t-1 into the accumulators and forms the scores of
    // tile t+1 on the matrix cores while the vector ALUs turn the scores of tile t into weights; the three are
    // independent, so one wave keeps both units busy.  A step is the two phases of an (even, odd) pair of tiles and
    // ends with one barrier: during step s the workgroup reads K of step s (tiles 2s, 2s+1) and V of step s-1 from
    // shared memory and stages K of step s+1 and V of step s.  Steps in which every tile touched lies wholly before
    // all of the wave's positions run without the per-tile conditions (`fast`).
    f32x4_t Se[kPrefillBlocks][2], So[kPrefillBlocks][2];        // scores of the even / odd tile in flight
    uint4 Pe[kPrefillBlocks], Po[kPrefillBlocks];                // weights of the even / odd tile in flight
    float ae[2] = {0.f, 0.f}, ao[2] = {0.f, 0.f};                // 8-bit cache: their scores' multipliers per 16-token half
    const float *k_scale = KV8 ? p.k_scale + kvh : nullptr, *v_scale = KV8 ? p.v_scale + kvh : nullptr;
#pragma unroll
    for (int cb = 0; cb < kPrefillBlocks; ++cb) Pe[cb] = Po[cb] = make_uint4(0, 0, 0, 0);
    auto step_body = [&](auto fast, int s) __attribute__((always_inline)) {
        constexpr bool kFast = decltype(fast)::value;
        const int buf = s & 1;
        fetch_rows(fast, vbase, v_scale, s, pg_v, sv_, svs);     // in flight while this step is computed
        fetch_rows(fast, kbase, k_scale, s + 1, pg_k, sk, sks);
        pg_v[0] = pg_k[0]; pg_v[1] = pg_k[1];
        lookup(s + 2);
        // phase 2s-1: P.V of tile 2s-2, weights of tile 2s-1, scores of tile 2s
        if (kFast || tile_active(2 * s - 2)) pv(smem[buf ^ 1][0][1], Pe);
        if (kFast || tile_active(2 * s)) scores(smem[buf][0][0], Se, kscale_lds[buf][0], ae);
        if (kFast || tile_active(2 * s - 1)) weights(fast, 2 * s - 1, So, Po, ao);
        // phase 2s: P.V of tile 2s-1, weights of tile 2s, scores of tile 2s+1
        if (kFast || tile_active(2 * s - 1)) pv(smem[buf ^ 1][1][1], Po);
        if (kFast || tile_active(2 * s + 1)) scores(smem[buf][1][0], So, kscale_lds[buf][1], ao);
        if (kFast || s < s_end) {                                // ahead of the weights: one block with the MFMAs above
            stage_k(buf ^ 1);
            stage_v(buf);
        }
        if (kFast || tile_active(2 * s)) weights(fast, 2 * s, Se, Pe, ae);
        if (kFast || s < s_end) lds_barrier();
    };
    // last step whose tiles 2s-2 .. 2s+1 are all wholly visible to every live column of the wave and all this
    // workgroup's, and whose fetches (V of step s, K of step s+1) lie wholly inside the context
    const int fast_last = wave_max_pos < 0 ? -1 : min(min(((wave_min_pos - (kTile - 1)) / kTile - 1) / 2, L / (2 * kTile) - 2),
                                                      s_end - 1);

    {
        lookup(s_begin);
        fetch_rows(std::false_type{}, kbase, k_scale, s_begin, pg_k, sk, sks);
        pg_v[0] = pg_k[0]; pg_v[1] = pg_k[1];
        lookup(s_begin + 1);
        stage_k(s_begin & 1);
        lds_barrier();
        for (int s = s_begin; s <= s_end; ++s) {
            if (s > s_begin && s <= fast_last) step_body(std::true_type{}, s);
            else step_body(std::false_type{}, s);
        }
    }

    // ---- normalise and store: a lane holds, for each of its columns, dims 16 eb + 4j .. + 3 of every 16-dim block eb
#pragma unroll
    for (int cb = 0; cb < kPrefillBlocks; ++cb) {
        float lsum = l[cb];
        lsum += __shfl_xor(lsum, 16);                            // the four lane groups hold disjoint tokens
        lsum += __shfl_xor(lsum, 32);
        if (pos[cb] < 0) continue;
        const int c = wave * kPrefillCols + cb * 16 + col;
        const int tl = c / G, g = c - tl * G;
        if (ns_eff > 1) {                                        // a piece for the merge: unnormalised, with (m, l)
            const size_t pi = ((((size_t)b * p.max_q_len + q0 + tl) * p.Hq + head0 + g) * NS + split);
            float *po = p.part_o + pi * D;
#pragma unroll
            for (int eb = 0; eb < 8; ++eb)
                *reinterpret_cast<float4 *>(po + 16 * eb + 4 * j) = make_float4(acc[cb][eb][0], acc[cb][eb][1], acc[cb][eb][2], acc[cb][eb][3]);
            if (j == 0) p.part_ml[pi] = make_float2(m[cb], lsum);
            continue;
        }
        const size_t row = ((size_t)(q_row0 + q0 + tl) * p.Hq + head0 + g) * D;
        const float inv = 1.f / lsum;                            // every live column saw its own position: lsum > 0
#pragma unroll
        for (int eb = 0; eb < 8; ++eb) {                         // acc[cb][eb][i] = O^T[dim 16 eb + 4 j + i][column]
            const float o0 = acc[cb][eb][0] * inv, o1 = acc[cb][eb][1] * inv, o2 = acc[cb][eb][2] * inv, o3 = acc[cb][eb][3] * inv;
            const size_t at = row + 16 * eb + 4 * j;
            if (p.out_bf16) {
                uint2 pk;
                pk.x = (uint32_t)float_to_bf16_rne(o0) | ((uint32_t)float_to_bf16_rne(o1) << 16);
                pk.y = (uint32_t)float_to_bf16_rne(o2) | ((uint32_t)float_to_bf16_rne(o3) << 16);
                *reinterpret_cast<uint2 *>(reinterpret_cast<uint16_t *>(p.out) + at) = pk;
            } else {
                *reinterpret_cast<float4 *>(reinterpret_cast<float *>(p.out) + at) = make_float4(o0, o1, o2, o3);
            }
        }
    }
}

// order[r] = the request with the r-th longest context (ties by index): one workgroup, thread t ranks request t.
constexpr int kPrefillOrderMax = 1024;
__global__ __launch_bounds__(kPrefillOrderMax) void prefill_order_kernel(const int32_t *__restrict__ context_lens, int B,
                                                                         int32_t *__restrict__ order) {
    __shared__ int lens[kPrefillOrderMax];
    const int t = threadIdx.x;
    if (t < B) lens[t] = context_lens[t];
    __syncthreads();
    if (t >= B) return;
    const int mine = lens[t];
    int rank = 0;
    for (int j = 0; j < B; ++j) rank += (lens[j] > mine) || (lens[j] == mine && j < t);
    order[rank] = t;
}

// Merge of a context split: out row = sum_s 2^(m_s - M) o_s / sum_s 2^(m_s - M) l_s over the pieces with l_s > 0, in
// split order (M = the largest reference among them; any common reference gives the same quotient).  One thread per
// four output elements of one (query token, head); grid (ceil(max_q_len * Hq * 32 / 256), B).
__global__ __launch_bounds__(kThreads) void prefill_merge_kernel(PrefillParams p) {
    constexpr int D = 128;
    const int b = blockIdx.y;
    const long long lin = (long long)blockIdx.x * kThreads + threadIdx.x;
    const int d4 = (int)(lin & 31);
    const long long rh = lin >> 5;
    const int head = (int)(rh % p.Hq);
    const long long qi = rh / p.Hq;
    const int L = p.context_lens[b];
    const int n_q = min(p.q_lens[b], L);
    const int n_live = min(n_q, p.max_q_len);
    if (qi >= n_live) return;
    // the split count of the row's query block, as the attention kernel derived it
    const int QB = prefill_tokens_per_block(p.G);
    const int wg_last = min(n_live, ((int)qi / QB + 1) * QB) - 1;
    const int n_tiles = (L - n_q + wg_last) / kTile + 1;
    const int ns_eff = prefill_effective_splits(p.num_splits, (n_tiles + 1) >> 1, p.min_split_steps);
    if (ns_eff == 1) return;                                     // written by the attention kernel itself
    const int NS = p.num_splits;
    const size_t pi = (((size_t)b * p.max_q_len + qi) * p.Hq + head) * NS;
    float M = -INFINITY, den = 0.f;
    float4 num = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int s = 0; s < ns_eff; ++s) {
        const float2 ml = p.part_ml[pi + s];
        if (ml.y > 0.f) {
            const float4 o = *reinterpret_cast<const float4 *>(p.part_o + (pi + s) * D + 4 * d4);
            const float Mn = fmaxf(M, ml.x);
            const float a = fast_exp2(M - Mn);                   // 0 while M is still -inf
            const float w = fast_exp2(ml.x - Mn);
            num.x = num.x * a + w * o.x; num.y = num.y * a + w * o.y;
            num.z = num.z * a + w * o.z; num.w = num.w * a + w * o.w;
            den = den * a + w * ml.y;
            M = Mn;
        }
    }
    const float inv = 1.f / den;                                 // the split that holds the token's own position has l > 0
    const size_t at = ((size_t)(p.q_offsets[b] + qi) * p.Hq + head) * D + 4 * d4;
    if (p.out_bf16) {
        uint2 pk;
        pk.x = (uint32_t)float_to_bf16_rne(num.x * inv) | ((uint32_t)float_to_bf16_rne(num.y * inv) << 16);
        pk.y = (uint32_t)float_to_bf16_rne(num.z * inv) | ((uint32_t)float_to_bf16_rne(num.w * inv) << 16);
        *reinterpret_cast<uint2 *>(reinterpret_cast<uint16_t *>(p.out) + at) = pk;
    } else {
        *reinterpret_cast<float4 *>(reinterpret_cast<float *>(p.out) + at) = make_float4(num.x * inv, num.y * inv, num.z * inv, num.w * inv);
    }
}

}  // namespace omni
