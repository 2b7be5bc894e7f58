// Matrix-core attention kernel for multi-token queries over the paged cache (chunked prefill): bf16 q/K/V,
// head_dim 128, group size <= 16.  Query i of request b's chunk sits at position p = L_b - n_b + i and attends to
// tokens 0 .. p (causal inside the chunk).
//
// A workgroup (8 waves, two per SIMD) owns one (request, KV head, block of query tokens).  Its "columns" are the
// (query token, query head of the group) pairs of that block; a wave owns 32 of them = two 16-column MFMA blocks.
// The same transposed products as in the decode kernel are used, per 32-token tile and per column block:
//   S^T = K Q^T     (A = K rows from shared memory, B = the block's queries, held in registers for the whole kernel)
//   O^T += V^T P^T  (A = V transposed, B = the softmax weights; both as fp16: V * 2^-4 is converted once per
//                    workgroup on its way into shared memory, exactly for 2^-10 <= |V| < 2^20, and fp16 weights carry
//                    11 significant bits, so one product does what bf16 weights need a hi + lo pair for)
// so every lane owns one column: running max, sum and rescale never cross lanes except two max exchanges per tile.
// What differs from decode is reuse: K/V tiles are fetched once per workgroup into shared memory (double buffered,
// one barrier per 64 tokens) and feed 16 column blocks, and the 8x8 in-lane transpose of V is done once per wave and
// tile for its two blocks.  That makes the path a dense contraction, not a stream; with the softmax arithmetic on
// the vector ALUs (no packed fp32 here) about as long as the matrix-core work, both units bound it.
#pragma once
#include "decode_mfma.hpp"

namespace omni {

constexpr int kPrefillThreads = 512;                  // 8 waves = 2 per SIMD share one K/V tile in shared memory
constexpr int kPrefillWaves = kPrefillThreads / 64;
constexpr int kPrefillBlocks = 2;                     // 16-column MFMA blocks per wave
constexpr int kPrefillCols = 16 * kPrefillBlocks;     // (token, head) pairs per wave
constexpr int kPrefillRowBytes = 256 + 16;            // a 256-byte K row plus padding: conflict-free 16-byte LDS reads
constexpr int kPrefillVRowBytes = 256 + 32;           // V rows: conflict-free 8-byte transposing reads (4 rows x 32 B)
constexpr float kPrefillSlack = 8.f;                  // log2 units a score may exceed a column's reference maximum

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

// Two floats -> packed fp16, round to nearest even.
__device__ __forceinline__ uint32_t pack_f16x2(float lo, float hi) {
    const f32x2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2_t));
}

constexpr float kPrefillVScale = 0x1p-4f;             // V is held in shared memory as fp16 of V * 2^-4 (see the kernel)
constexpr float kPrefillBias = 6.f;                   // the softmax weights are held as 2^6 times exp2(score - reference)

// Eight bf16 values -> eight fp16 values of V * 2^-4.  Exact wherever the scaled value is a normal fp16 number
// (2^-10 <= |V| < 2^20); below that the spacing is 2^-24, i.e. an absolute error of at most 2^-21 on V; above it the
// value becomes infinite and shows in the result.
__device__ __forceinline__ uint4 bf16x8_to_scaled_f16x8(const uint4 &v) {
    uint4 r;
    r.x = pack_f16x2(bf16_bits_to_float(v.x & 0xffffu) * kPrefillVScale, __uint_as_float(v.x & 0xffff0000u) * kPrefillVScale);
    r.y = pack_f16x2(bf16_bits_to_float(v.y & 0xffffu) * kPrefillVScale, __uint_as_float(v.y & 0xffff0000u) * kPrefillVScale);
    r.z = pack_f16x2(bf16_bits_to_float(v.z & 0xffffu) * kPrefillVScale, __uint_as_float(v.z & 0xffff0000u) * kPrefillVScale);
    r.w = pack_f16x2(bf16_bits_to_float(v.w & 0xffffu) * kPrefillVScale, __uint_as_float(v.w & 0xffff0000u) * kPrefillVScale);
    return r;
}

struct PrefillParams {
    const void *q;                    // [Tq, Hq, D] bf16
    const void *k_cache, *v_cache;
    const int32_t *block_table, *context_lens, *q_lens;
    const long long *q_offsets;
    void *out;                        // [Tq, Hq, D]
    float scale_log2;
    int Hq, Hkv, G, MB;
    int out_bf16;
};

// Query tokens per wave and per workgroup for a group of G heads.
__host__ __device__ inline int prefill_tokens_per_wave(int G) { return kPrefillCols / G; }
__host__ __device__ inline int prefill_tokens_per_block(int G) { return kPrefillWaves * prefill_tokens_per_wave(G); }

template <int PS>
__global__ __launch_bounds__(kPrefillThreads, 1) void prefill_mfma_kernel(PrefillParams p) {
    constexpr int D = 128;
    constexpr int kLog2Ps = (PS == 16) ? 4 : 5;
    constexpr int kTileBytes = kTile * kPrefillVRowBytes;        // room for one K or V tile in shared memory
    __shared__ __align__(16) char smem[2][2][2][kTileBytes];     // [buffer][tile of the step][K, V]

    const int b = blockIdx.z, kvh = blockIdx.y;
    const int G = p.G, head0 = kvh * G;
    const int L = p.context_lens[b];
    const int n_q = min(p.q_lens[b], L);
    const int TW = prefill_tokens_per_wave(G), QB = kPrefillWaves * TW;
    const int q0 = blockIdx.x * QB;                              // first query token of this workgroup
    if (n_q <= 0 || q0 >= n_q) return;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int col = lane & 15, j = lane >> 4;
    const long long q_row0 = p.q_offsets[b];
    const int pos0 = L - n_q;                                    // position of the chunk's first token
    const int wg_last = min(n_q, q0 + QB) - 1;                   // last query token of the workgroup
    const int n_tiles = (pos0 + wg_last) / kTile + 1;            // tiles that hold tokens 0 .. position of wg_last

    // ---- this lane's four columns: query token, head, position; and the queries as MFMA B operands
    int pos[kPrefillBlocks];                                     // -1: padding column (never stored)
    uint4 Q[kPrefillBlocks][4];
    int wave_max_pos = -1;
#pragma unroll
    for (int cb = 0; cb < kPrefillBlocks; ++cb) {
        const int c = cb * 16 + col;
        const int tl = c / G, g = c - tl * G;
        const int qi = q0 + wave * TW + tl;                      // query token inside the chunk
        const bool live = tl < TW && qi < n_q;
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
    // each tile's K rows and V rows (piece = 16 * token + chunk)
    const size_t page_stride = (size_t)p.Hkv * PS * D * 2;
    const char *kbase = reinterpret_cast<const char *>(p.k_cache) + (size_t)kvh * PS * D * 2;
    const char *vbase = reinterpret_cast<const char *>(p.v_cache) + (size_t)kvh * PS * D * 2;
    const int32_t *bt = p.block_table + (size_t)b * p.MB;
    const int st_tok = threadIdx.x >> 4, st_chunk = threadIdx.x & 15;       // token 0..31 of a tile
    const int lds_off = st_tok * kPrefillRowBytes + st_chunk * 16;
    const int lds_off_v = st_tok * kPrefillVRowBytes + st_chunk * 16;
    uint4 sk[2], sv_[2];
    auto fetch_step = [&](int step) __attribute__((always_inline)) {
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
            const int t = (2 * step + sub) * kTile + st_tok;
            sk[sub] = sv_[sub] = make_uint4(0, 0, 0, 0);                    // rows beyond the context are zero
            if (t < L) {
                const int pg = bt[t >> kLog2Ps];
                const size_t o = (size_t)pg * page_stride + (size_t)(t & (PS - 1)) * 256 + st_chunk * 16;
                sk[sub] = *reinterpret_cast<const uint4 *>(kbase + o);
                sv_[sub] = *reinterpret_cast<const uint4 *>(vbase + o);
            }
        }
    };
    auto stage_step = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
            *reinterpret_cast<uint4 *>(&smem[buf][sub][0][lds_off]) = sk[sub];
            *reinterpret_cast<uint4 *>(&smem[buf][sub][1][lds_off_v]) = bf16x8_to_scaled_f16x8(sv_[sub]);
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

    float raw_limit[kPrefillBlocks];                                 // raw score above which a column's m must move
#pragma unroll
    for (int cb = 0; cb < kPrefillBlocks; ++cb) raw_limit[cb] = -INFINITY;
    const float inv_scale_log2 = 1.f / p.scale_log2;
    // ---- one 32-token tile, in three pieces, so that the loop below can run the two tiles of a step interleaved:
    // the score MFMAs of the second tile and the P.V MFMAs of the first are in the matrix-core queue while the vector
    // ALUs do the softmax of the first and of the second tile.
    auto read_k = [&](const char *ks, uint4 (&K)[8]) __attribute__((always_inline)) {
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            K[kk] = *reinterpret_cast<const uint4 *>(ks + col * kPrefillRowBytes + (4 * kk + j) * 16);
            K[4 + kk] = *reinterpret_cast<const uint4 *>(ks + (16 + col) * kPrefillRowBytes + (4 * kk + j) * 16);
        }
    };
    // Raw scores q.k of the column blocks.  The softmax scale is applied inside the exponent (one fused multiply-add
    // per score): scale > 0, so the order of scores is that of the raw dot products.
    auto scores = [&](const uint4 (&K)[8], f32x4_t (&s0)[kPrefillBlocks], f32x4_t (&s1)[kPrefillBlocks]) __attribute__((always_inline)) {
#pragma unroll
        for (int cb = 0; cb < kPrefillBlocks; ++cb) {
            s0[cb] = f32x4_t{0.f, 0.f, 0.f, 0.f}; s1[cb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                s0[cb] = mfma_bf16(K[kk], Q[cb][kk], s0[cb]);
                s1[cb] = mfma_bf16(K[4 + kk], Q[cb][kk], s1[cb]);
            }
        }
    };
    auto softmax = [&](int tb, const f32x4_t (&s0)[kPrefillBlocks], const f32x4_t (&s1)[kPrefillBlocks],
                       uint4 (&P)[kPrefillBlocks]) __attribute__((always_inline)) {
        const bool need_mask = tb + kTile - 1 > wave_min_pos;
#pragma unroll
        for (int cb = 0; cb < kPrefillBlocks; ++cb) {
            float sv[8];
#pragma unroll
            for (int i = 0; i < 4; ++i) { sv[i] = s0[cb][i]; sv[4 + i] = s1[cb][i]; }
            if (need_mask) {                                     // tokens after the column's position
#pragma unroll
                for (int r = 0; r < 8; ++r)
                    if (tb + slot_token(j, r) > pos[cb]) sv[r] = -INFINITY;
            }
            float lmax = sv[0];
#pragma unroll
            for (int r = 1; r < 8; ++r) lmax = fmaxf(lmax, sv[r]);
            // The reference m of a column (log2 domain) is moved, and its sums rescaled, only when a score exceeds it
            // by more than bias + slack: any common reference gives the same softmax.  A move puts m at the running
            // maximum less the bias, so the largest weight of a column lies in [2^bias, 2^(bias + slack)]: below the
            // largest fp16 number, and a weight loses precision as an fp16 subnormal only when it is 2^-20 of the
            // largest or less.  After a column's first tiles moves are rare, so the exchange between the four lane
            // groups of a column and the rescale of 32 accumulators leave the common path.
            if (__any(lmax > raw_limit[cb])) {
                float tmax = lmax;
                tmax = fmaxf(tmax, __shfl_xor(tmax, 16));
                tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
                // a column whose tokens are all masked so far keeps a finite stand-in: exp2 then sees -inf - finite
                const float mn = fmaxf(fmaxf(m[cb], fmaf(tmax, p.scale_log2, -kPrefillBias)), -1e30f);
                const float alpha = fast_exp2(m[cb] - mn);
                l[cb] *= alpha;
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[cb][e] *= alpha;
                m[cb] = mn;
                raw_limit[cb] = (mn + kPrefillBias + kPrefillSlack) * inv_scale_log2;
            }
            float pw[8], psum = 0.f;
#pragma unroll
            for (int r = 0; r < 8; ++r) { pw[r] = fast_exp2(fmaf(sv[r], p.scale_log2, -m[cb])); psum += pw[r]; }
            l[cb] += psum;
            // the weights go to the matrix core as fp16 (11 significant bits; the sum above keeps the fp32 values)
            P[cb] = make_uint4(pack_f16x2(pw[0], pw[1]), pack_f16x2(pw[2], pw[3]), pack_f16x2(pw[4], pw[5]),
                               pack_f16x2(pw[6], pw[7]));
        }
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

    const int n_steps = (n_tiles + 1) >> 1;
    fetch_step(0);
    stage_step(0);
    lds_barrier();
    for (int step = 0; step < n_steps; ++step) {
        const int buf = step & 1;
        const bool more = step + 1 < n_steps;
        if (more) fetch_step(step + 1);                          // in flight while this step is computed
        const int tb0 = 2 * step * kTile, tb1 = tb0 + kTile;
        const bool live1 = tb1 <= wave_max_pos;                  // the tiles hold tokens some column of this wave sees
        if (tb0 <= wave_max_pos) {
            uint4 K[8];
            f32x4_t s0a[kPrefillBlocks], s1a[kPrefillBlocks], s0b[kPrefillBlocks], s1b[kPrefillBlocks];
            uint4 P[kPrefillBlocks];
            read_k(smem[buf][0][0], K);
            scores(K, s0a, s1a);
            if (live1) read_k(smem[buf][1][0], K);               // arrives during the first softmax
            softmax(tb0, s0a, s1a, P);
            if (live1) scores(K, s0b, s1b);                      // queued ahead of the first product
            pv(smem[buf][0][1], P);
            if (live1) {
                softmax(tb1, s0b, s1b, P);                       // while the matrix cores work on the queue
                pv(smem[buf][1][1], P);
            }
        }
        if (more) stage_step(buf ^ 1);
        lds_barrier();
    }

    // ---- normalise and store: a lane holds, for each of its columns, dims 16 eb + 4j .. + 3 of every 16-dim block eb
#pragma unroll
    for (int cb = 0; cb < kPrefillBlocks; ++cb) {
        float lsum = l[cb];
        lsum += __shfl_xor(lsum, 16);                            // the four lane groups hold disjoint tokens
        lsum += __shfl_xor(lsum, 32);
        if (pos[cb] < 0) continue;
        const int c = cb * 16 + col;
        const int tl = c / G, g = c - tl * G;
        const size_t row = ((size_t)(q_row0 + q0 + wave * TW + tl) * p.Hq + head0 + g) * D;
        const float inv = (1.f / kPrefillVScale) / lsum;         // every live column saw its own position: lsum > 0
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

}  // namespace omni
