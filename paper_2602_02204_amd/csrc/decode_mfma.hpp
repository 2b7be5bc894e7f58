// Matrix-core split-context decode kernel for bf16 q/K/V with head_dim 128 and group size <= 16.
//
// One workgroup = one (request, partition, KV head); its four waves take 32-token tiles round-robin and each keeps
// its own online-softmax state; the states meet in LDS at the end.
//
// Per 32-token tile a wave computes, with v_mfma_f32_16x16x32_bf16 (A: 16 rows x 32 k, B: 32 k x 16 columns;
// a lane holds row/column lane%16 and the 8 consecutive k of group lane/16):
//   S^T = K Q^T     A = K rows (row = token), B = the group's query heads (column = head, zero beyond G)
//   O^T += V^T P^T  A = V transposed in registers (row = output dim), B = softmax weights (column = head)
// With this orientation every lane owns one head (lane%16) in S^T, in P^T and in the O^T accumulators, so the
// running max, the rescale factor and the weights never cross lanes except for two max-exchanges per tile.
// The k-slots of a lane group may be bound to any 8 tokens / any 8 dims as long as both operands agree:
//   - for K Q^T the 8 k-slots of group j in step kk are dims (4kk+j)*8 .. +8: one 16-byte load per lane;
//   - for V^T P^T the 8 k-slots of group j are tokens {4j..4j+3, 16+4j..16+4j+3}, exactly the tokens whose scores
//     the S^T accumulators of that lane group hold, so P needs no data movement; V is loaded row-wise (a 256-byte
//     row per 16 lanes) and an 8x8 in-lane transpose (v_perm_b32) turns 8 rows x 8 dims into 8 operands.
// The weights go to the matrix core as bf16 hi + bf16 lo (two MFMAs), which keeps them to ~2^-16 relative.
#pragma once
#include "common.hpp"

namespace omni {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ f32x4_t mfma_bf16(const uint4 &a, const uint4 &b, f32x4_t c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    f32x2_t x = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(x, bf16x2_t));
}

__device__ __forceinline__ uint32_t dword_of(const uint4 &v, int w) {
    return w == 0 ? v.x : (w == 1 ? v.y : (w == 2 ? v.z : v.w));
}

// token of k-slot r (0..7) of lane group j inside a 32-token tile
__device__ __forceinline__ int slot_token(int j, int r) { return (r < 4) ? 4 * j + r : 16 + 4 * j + (r - 4); }

template <int PS>
struct MfmaTileLoader {
    // lane constants
    const char *kbase, *vbase;       // pool base + KV-head offset
    size_t page_stride;              // bytes between pages
    int koff;                        // byte offset of this lane's K chunk inside a 16-token block
    int voff;                        // byte offset of this lane's V chunk inside a row
    int j;
    const int32_t *bt;               // block-table row of the request

    // Issue the 16 loads of tile `tb` (first token).  Pages whose first token is at or past t1 are replaced by the
    // tile's first page so that no table entry beyond the request's pages is dereferenced.
    __device__ __forceinline__ void issue(int tb, int t1, uint4 (&K)[8], uint4 (&V)[8]) const {
        if constexpr (PS == 16) {
            const int pi = __builtin_amdgcn_readfirstlane(tb >> 4);
            const int second = (tb + 16 < t1) ? pi + 1 : pi;
            const int pg0 = bt[pi], pg1 = bt[second];
            const char *k0 = kbase + (size_t)pg0 * page_stride + koff;
            const char *k1 = kbase + (size_t)pg1 * page_stride + koff;
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                K[kk] = *reinterpret_cast<const uint4 *>(k0 + kk * 64);
                K[4 + kk] = *reinterpret_cast<const uint4 *>(k1 + kk * 64);
            }
            const char *v0 = vbase + (size_t)pg0 * page_stride + voff + (4 * j) * 256;
            const char *v1 = vbase + (size_t)pg1 * page_stride + voff + (4 * j) * 256;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                V[r] = *reinterpret_cast<const uint4 *>(v0 + r * 256);
                V[4 + r] = *reinterpret_cast<const uint4 *>(v1 + r * 256);
            }
        } else {
            const int pi = __builtin_amdgcn_readfirstlane(tb >> 5);
            const int pg = bt[pi];
            const char *k0 = kbase + (size_t)pg * page_stride + koff;
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                K[kk] = *reinterpret_cast<const uint4 *>(k0 + kk * 64);
                K[4 + kk] = *reinterpret_cast<const uint4 *>(k0 + 16 * 256 + kk * 64);
            }
            const char *v0 = vbase + (size_t)pg * page_stride + voff + (4 * j) * 256;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                V[r] = *reinterpret_cast<const uint4 *>(v0 + r * 256);
                V[4 + r] = *reinterpret_cast<const uint4 *>(v0 + (16 + r) * 256);
            }
        }
    }
};

struct MfmaState {
    float m, l;
    f32x4_t acc[8];          // acc[e][i] = O^T[dim 32j + 8i + e][head lane%16]
};

// One 32-token tile: scores, online softmax, weighted V accumulation.
__device__ __forceinline__ void mfma_tile(const uint4 (&K)[8], uint4 (&V)[8], const uint4 (&Q)[4], MfmaState &st,
                                          int tb, int t1, int j, float scale_log2) {
    // Scores are rounded before the running max is subtracted (no fused multiply-subtract): s - max is then exactly
    // 0 for the maximal score, and a length-1 context returns its V row bit for bit.
#pragma clang fp contract(off)
    f32x4_t s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        s0 = mfma_bf16(K[kk], Q[kk], s0);
        s1 = mfma_bf16(K[4 + kk], Q[kk], s1);
    }
    float sv[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) { sv[i] = s0[i] * scale_log2; sv[4 + i] = s1[i] * scale_log2; }
    if (tb + 32 > t1) {                                  // ragged last tile (uniform branch)
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            if (tb + slot_token(j, r) >= t1) {           // unowned slot: its K/V bits are arbitrary, possibly NaN
                sv[r] = -INFINITY;
                V[r] = make_uint4(0, 0, 0, 0);
            }
        }
    }
    float tmax = sv[0];
#pragma unroll
    for (int r = 1; r < 8; ++r) tmax = fmaxf(tmax, sv[r]);
    tmax = fmaxf(tmax, __shfl_xor(tmax, 16));
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
    const float mn = fmaxf(st.m, tmax);                  // finite: every tile holds at least one live token
    const float alpha = fast_exp2(st.m - mn);
    float pw[8], psum = 0.f;
#pragma unroll
    for (int r = 0; r < 8; ++r) { pw[r] = fast_exp2(sv[r] - mn); psum += pw[r]; }
    st.l = st.l * alpha + psum;
    st.m = mn;
    uint4 Ph, Pl;
    {
        uint32_t h[4], lo[4];
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            h[w] = pack_bf16x2(pw[2 * w], pw[2 * w + 1]);
            const float r0 = pw[2 * w] - bf16_bits_to_float(h[w] & 0xffffu);
            const float r1 = pw[2 * w + 1] - __uint_as_float(h[w] & 0xffff0000u);
            lo[w] = pack_bf16x2(r0, r1);
        }
        Ph = make_uint4(h[0], h[1], h[2], h[3]);
        Pl = make_uint4(lo[0], lo[1], lo[2], lo[3]);
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) st.acc[e] *= alpha;
    // 8x8 transpose: operand e holds dim e of the lane's 8-dim chunk for the 8 tokens of its lane group
    // (dword w of V[r] holds dims 2w and 2w+1 of token slot r)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int w = e >> 1;
        const uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;
        uint4 A;
        A.x = __builtin_amdgcn_perm(dword_of(V[1], w), dword_of(V[0], w), sel);
        A.y = __builtin_amdgcn_perm(dword_of(V[3], w), dword_of(V[2], w), sel);
        A.z = __builtin_amdgcn_perm(dword_of(V[5], w), dword_of(V[4], w), sel);
        A.w = __builtin_amdgcn_perm(dword_of(V[7], w), dword_of(V[6], w), sel);
        st.acc[e] = mfma_bf16(A, Ph, st.acc[e]);
        st.acc[e] = mfma_bf16(A, Pl, st.acc[e]);
    }
}

template <int PS>
__global__ __launch_bounds__(kThreads, 2) void decode_mfma_kernel(AttnParams p) {
    constexpr int D = 128;
    __shared__ CombineSmem<D> sm;
    __shared__ int sm_plan[16];

    const int r = blockIdx.x / p.Hkv, kvh = blockIdx.x - r * p.Hkv;
    Item it;
    int R;
    long long Ttot;
    const bool have = plan_find(p.context_lens, p.plan, r, sm_plan, &it, &R, &Ttot);
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        p.ws.plan_words[0] = have ? it.PL : 0; p.ws.plan_words[1] = R;
        p.ws.plan_words[2] = (int)(Ttot & 0xffffffffLL); p.ws.plan_words[3] = (int)(Ttot >> 32);
    }
    if (!have) return;

    const int G = p.G;
    const int plen = piece_len(it.L, it.nparts);
    const int t0 = it.part * plen;
    const int t1 = min(it.L, t0 + plen);
    const int ntiles = (t1 - t0 + kTile - 1) / kTile;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int col = lane & 15, j = lane >> 4;

    // B operand of K Q^T: column = head `col` of the group, k-slots = dims (4kk + j)*8 .. +8
    uint4 Q[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) Q[kk] = make_uint4(0, 0, 0, 0);
    if (col < G) {
        const char *qrow = reinterpret_cast<const char *>(p.q) + ((size_t)it.b * p.Hq + kvh * G + col) * (D * 2);
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) Q[kk] = *reinterpret_cast<const uint4 *>(qrow + (4 * kk + j) * 16);
    }

    MfmaTileLoader<PS> ld;
    ld.page_stride = (size_t)p.Hkv * PS * D * 2;
    ld.kbase = reinterpret_cast<const char *>(p.k_cache) + (size_t)kvh * PS * D * 2;
    ld.vbase = reinterpret_cast<const char *>(p.v_cache) + (size_t)kvh * PS * D * 2;
    ld.koff = col * 256 + j * 16;
    ld.voff = col * 16;
    ld.j = j;
    ld.bt = p.block_table + (size_t)it.b * p.MB;

    MfmaState st;
    st.m = -INFINITY; st.l = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) st.acc[e] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    uint4 K0[8], V0[8], K1[8], V1[8];
    int ti = wave;
    if (ti < ntiles) {
        ld.issue(t0 + ti * kTile, t1, K0, V0);
        while (true) {
            const bool more1 = ti + kWaves < ntiles;
            if (more1) ld.issue(t0 + (ti + kWaves) * kTile, t1, K1, V1);
            mfma_tile(K0, V0, Q, st, t0 + ti * kTile, t1, j, p.scale_log2);
            if (!more1) break;
            ti += kWaves;
            const bool more0 = ti + kWaves < ntiles;
            if (more0) ld.issue(t0 + (ti + kWaves) * kTile, t1, K0, V0);
            mfma_tile(K1, V1, Q, st, t0 + ti * kTile, t1, j, p.scale_log2);
            if (!more0) break;
            ti += kWaves;
        }
    }

    // the sum is per lane (its 8 token slots per tile): add the four lane groups; m is already common to them
    st.l += __shfl_xor(st.l, 16);
    st.l += __shfl_xor(st.l, 32);
    if (col < G) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float4 lo4 = make_float4(st.acc[0][i], st.acc[1][i], st.acc[2][i], st.acc[3][i]);
            float4 hi4 = make_float4(st.acc[4][i], st.acc[5][i], st.acc[6][i], st.acc[7][i]);
            *reinterpret_cast<float4 *>(&sm.o[wave][col][32 * j + 8 * i]) = lo4;
            *reinterpret_cast<float4 *>(&sm.o[wave][col][32 * j + 8 * i + 4]) = hi4;
        }
        if (j == 0) { sm.m[wave][col] = st.m; sm.l[wave][col] = st.l; }
    }
    wg_combine_and_store<D>(sm, p, it, r, kvh);
}

}  // namespace omni
