// Matrix-core split-context decode kernel for bf16 q/K/V with head_dim 128 and group size <= 16.
//
// A workgroup takes the ranges the plan gives it (see plan.hpp) for one KV head; the 32-token tiles of a range are dealt
// to its four waves in contiguous runs, a wave keeps one online-softmax state per request its run touches, and the
// states meet in LDS when the range is done.
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
// With T query tokens per request (kernel variant MT, T * G <= 16) a column is a (query token, head) pair instead of
// a head: it has its own query row, its own causal limit (tokens 0 .. L - T + i) and its own output row; everything
// that is said of a head above holds per column.  An 8-bit cache (variant KV8) is widened to bf16 in registers.
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

constexpr int kAppendFlag = 1 << 30;   // in a slot's tile word: the tile holds the token to append (fused decode step)

// token of k-slot r (0..7) of lane group j inside a 32-token tile
__device__ __forceinline__ int slot_token(int j, int r) { return (r < 4) ? 4 * j + r : 16 + 4 * j + (r - 4); }

template <int PS>
struct MfmaTileLoader {
    const char *kbase, *vbase;       // pool base + KV-head offset
    size_t page_stride;              // bytes between pages
    int koff;                        // byte offset of this lane's K chunk inside a 16-token block
    int voff;                        // byte offset of this lane's first V row chunk inside a 16-token block

    // The 8 K loads / 8 V loads of one 32-token tile.  pg0 / pg1 are the physical pages of its first / second 16
    // tokens (wave-uniform; with 32-token pages only pg0 is used).
    __device__ __forceinline__ void issue_k(int pg0, int pg1, uint4 (&K)[8]) const {
        const size_t o0 = (size_t)pg0 * page_stride;
        const size_t o1 = (PS == 16) ? (size_t)pg1 * page_stride : o0 + 16 * 256;
        const char *k0 = kbase + o0 + koff, *k1 = kbase + o1 + koff;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            K[kk] = nt_load16(k0 + kk * 64);
            K[4 + kk] = nt_load16(k1 + kk * 64);
        }
    }
    // K through shared memory: the loads above fetch 64 bytes of each of 16 rows per instruction, i.e. every cache line
    // in two halves by two instructions, which keeps non-temporal loads from paying off for K.  Here a wave copies the
    // tile's rows into its own 8 KB of shared memory with loads that cover four whole rows per instruction (lane l of
    // instruction r: row 4r + l/16 of the 16-token block, 16-byte chunk (l % 16) ^ row, landing at 16 l behind the
    // instruction's base: the xor spreads a column of chunks over the banks), and reads its MFMA operands back from
    // there.  No register holds the tile while it is on its way.
    int kst_goff[4];                 // per lane: byte offset of the chunk it fetches in instruction r, inside a block
    int kst_roff[4];                 // per lane: byte offset of the operand of k-step kk inside a staged block
    __device__ __forceinline__ void init_staging(int lane) {
        const int sub = lane >> 4, p16 = lane & 15, i = lane & 15, j = lane >> 4;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int row = 4 * r + sub;
            kst_goff[r] = row * 256 + ((p16 ^ row) << 4);
        }
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) kst_roff[kk] = i * 256 + (((4 * kk + j) ^ i) << 4);
    }
    __device__ __forceinline__ void issue_k_staged(int pg0, int pg1, char *stage) const {
        const size_t o0 = (size_t)pg0 * page_stride;
        const size_t o1 = (PS == 16) ? (size_t)pg1 * page_stride : o0 + 16 * 256;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(kbase + o0 + kst_goff[r]),
                                             (__attribute__((address_space(3))) void *)(stage + r * 1024), 16, 0, 2);
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(kbase + o1 + kst_goff[r]),
                                             (__attribute__((address_space(3))) void *)(stage + 4096 + r * 1024), 16, 0, 2);
        }
    }
    __device__ __forceinline__ void read_k_staged(const char *stage, uint4 (&K)[8]) const {
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            K[kk] = *reinterpret_cast<const uint4 *>(stage + kst_roff[kk]);
            K[4 + kk] = *reinterpret_cast<const uint4 *>(stage + 4096 + kst_roff[kk]);
        }
    }
    __device__ __forceinline__ void issue_v(int pg0, int pg1, uint4 (&V)[8]) const {
        const size_t o0 = (size_t)pg0 * page_stride;
        const size_t o1 = (PS == 16) ? (size_t)pg1 * page_stride : o0 + 16 * 256;
        const char *v0 = vbase + o0 + voff, *v1 = vbase + o1 + voff;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            V[r] = nt_load16(v0 + r * 256);
            V[4 + r] = nt_load16(v1 + r * 256);
        }
    }
};

// 8 E4M3 bytes (two dwords, dims ascending) -> 8 bf16 (exact: 4 significant bits fit in 8).
__device__ __forceinline__ uint4 fp8x8_to_bf16x8(uint32_t lo, uint32_t hi) {
    uint4 r;
    r.x = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(lo, 1.0f, false));
    r.y = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(lo, 1.0f, true));
    r.z = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(hi, 1.0f, false));
    r.w = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(hi, 1.0f, true));
    return r;
}

// Loads of one 32-token tile of an 8-bit KV cache (128-byte rows).  K: a lane (token = lane%16, group j) takes the 32
// bytes of dims 32j .. 32j+31 as two 16-byte loads, and MFMA step kk of group j uses dims 32j + 8kk .. +8 (the query
// operand is bound the same way).  V: a lane (chunk = lane%16, group j) takes 8 bytes = dims 8*chunk .. +8 of rows
// 4j .. 4j+3 and 16+4j .. 16+4j+3.  The scales of the tile's pages ride along.
template <int PS>
struct Mfma8TileLoader {
    const char *kbase, *vbase;
    const float *k_scale, *v_scale;  // already offset by the KV head
    size_t page_stride;
    int Hkv, koff, voff;

    __device__ __forceinline__ void issue_k(int pg0, int pg1, uint4 (&Kr)[4], float (&ks)[2]) const {
        const int pgb = (PS == 16) ? pg1 : pg0;
        const char *k0 = kbase + (size_t)pg0 * page_stride + koff;
        const char *k1 = (PS == 16) ? kbase + (size_t)pg1 * page_stride + koff : k0 + 16 * 128;
        Kr[0] = *reinterpret_cast<const uint4 *>(k0);
        Kr[1] = *reinterpret_cast<const uint4 *>(k0 + 16);
        Kr[2] = *reinterpret_cast<const uint4 *>(k1);
        Kr[3] = *reinterpret_cast<const uint4 *>(k1 + 16);
        ks[0] = k_scale[(size_t)pg0 * Hkv];
        ks[1] = k_scale[(size_t)pgb * Hkv];
    }
    // K through shared memory, as in the 16-bit loader: a 16-token block is 2 KB = two instructions of eight whole rows
    // (lane l of instruction r: row 8r + l/8, 16-byte chunk (l % 8) ^ (row % 8)); a lane reads its 32 bytes of a row back
    // as two chunks.
    int kst_goff[2], kst_roff[2];
    __device__ __forceinline__ void init_staging(int lane) {
        const int i = lane & 15, j = lane >> 4;
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            const int row = 8 * r + (lane >> 3);
            kst_goff[r] = row * 128 + (((lane & 7) ^ (row & 7)) << 4);
        }
#pragma unroll
        for (int e = 0; e < 2; ++e) kst_roff[e] = i * 128 + (((2 * j + e) ^ (i & 7)) << 4);
    }
    __device__ __forceinline__ void issue_k_staged(int pg0, int pg1, char *stage, float (&ks)[2]) const {
        const int pgb = (PS == 16) ? pg1 : pg0;
        const size_t o0 = (size_t)pg0 * page_stride;
        const size_t o1 = (PS == 16) ? (size_t)pg1 * page_stride : o0 + 16 * 128;
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(kbase + o0 + kst_goff[r]),
                                             (__attribute__((address_space(3))) void *)(stage + r * 1024), 16, 0, 2);
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(kbase + o1 + kst_goff[r]),
                                             (__attribute__((address_space(3))) void *)(stage + 2048 + r * 1024), 16, 0, 2);
        }
        ks[0] = k_scale[(size_t)pg0 * Hkv];
        ks[1] = k_scale[(size_t)pgb * Hkv];
    }
    __device__ __forceinline__ void read_k_staged(const char *stage, uint4 (&Kr)[4]) const {
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            Kr[e] = *reinterpret_cast<const uint4 *>(stage + kst_roff[e]);
            Kr[2 + e] = *reinterpret_cast<const uint4 *>(stage + 2048 + kst_roff[e]);
        }
    }
    __device__ __forceinline__ void issue_v(int pg0, int pg1, uint2 (&Vr)[8], float (&vs)[2]) const {
        const int pgb = (PS == 16) ? pg1 : pg0;
        const char *v0 = vbase + (size_t)pg0 * page_stride + voff;
        const char *v1 = (PS == 16) ? vbase + (size_t)pg1 * page_stride + voff : v0 + 16 * 128;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            Vr[r] = nt_load8(v0 + r * 128);
            Vr[4 + r] = nt_load8(v1 + r * 128);
        }
        vs[0] = v_scale[(size_t)pg0 * Hkv];
        vs[1] = v_scale[(size_t)pgb * Hkv];
    }
};

// Scores of a tile of an 8-bit cache: bytes are widened to bf16 right before each MFMA step; the K scale of each
// 16-token half joins the softmax scale.
__device__ __forceinline__ void mfma_scores_fp8(const uint4 (&Kr)[4], const uint4 (&Q)[4], float (&sv)[8],
                                                float scale_log2, const float (&ks)[2]) {
#pragma clang fp contract(off)
    f32x4_t s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        const uint4 &a = Kr[kk >> 1], &b = Kr[2 + (kk >> 1)];
        const uint4 A0 = (kk & 1) ? fp8x8_to_bf16x8(a.z, a.w) : fp8x8_to_bf16x8(a.x, a.y);
        const uint4 A1 = (kk & 1) ? fp8x8_to_bf16x8(b.z, b.w) : fp8x8_to_bf16x8(b.x, b.y);
        s0 = mfma_bf16(A0, Q[kk], s0);
        s1 = mfma_bf16(A1, Q[kk], s1);
    }
    const float c0 = ks[0] * scale_log2, c1 = ks[1] * scale_log2;
#pragma unroll
    for (int i = 0; i < 4; ++i) { sv[i] = s0[i] * c0; sv[4 + i] = s1[i] * c1; }
}

struct MfmaState {
    float m, l;
    f32x4_t acc[8];          // acc[e][i] = O^T[dim 32j + 8i + e][head lane%16]
};

// First half of a 32-token tile: the scores S^T = K Q^T of the tile, in the log2 domain.
__device__ __forceinline__ void mfma_scores(const uint4 (&K)[8], const uint4 (&Q)[4], float (&sv)[8], float scale_log2) {
    // Scores are rounded before the running max is subtracted (no fused multiply-subtract): s - max is then exactly
    // 0 for the maximal score, and a length-1 context returns its V row bit for bit.
#pragma clang fp contract(off)
    f32x4_t s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        s0 = mfma_bf16(K[kk], Q[kk], s0);
        s1 = mfma_bf16(K[4 + kk], Q[kk], s1);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) { sv[i] = s0[i] * scale_log2; sv[4 + i] = s1[i] * scale_log2; }
}

// Second half: online softmax over the tile's scores and the weighted V accumulation O^T += V^T P^T.
// `vs0` / `vs1` scale the weights of the tile's first / second 16 tokens on their way into the product (the V scales of
// an 8-bit cache; 1 otherwise): the sum of weights stays unscaled.
// t1: the request's length; t1col: tokens this lane's column may see (t1 less the query tokens after its own; = t1 in
// plain decode); t1min: the smallest t1col of the wave's columns.
// kMulti (several query tokens per request): the three differ; otherwise all are t1.
template <bool kScaled = false, bool kMulti = false>
__device__ __forceinline__ void mfma_softmax_pv(float (&sv)[8], uint4 (&V)[8], MfmaState &st, int tb, int t1, int t1col,
                                                int t1min, int j, float vs0 = 1.f, float vs1 = 1.f) {
#pragma clang fp contract(off)
    if (tb + 32 > (kMulti ? t1min : t1)) {               // last tiles of the request (uniform branch)
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            if (kMulti) {
                if (tb + slot_token(j, r) >= t1col) sv[r] = -INFINITY;      // not visible to this column
                if (tb + slot_token(j, r) >= t1) V[r] = make_uint4(0, 0, 0, 0);
            } else if (tb + slot_token(j, r) >= t1) {    // unowned slot: its K/V bits are arbitrary, possibly NaN
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
    // finite: in plain decode every tile holds a live token; with several query tokens a column may see none of a
    // tile's, and then keeps a finite stand-in (exp2 below sees -inf - finite, never -inf - -inf)
    const float mn = kMulti ? fmaxf(fmaxf(st.m, tmax), -1e30f) : fmaxf(st.m, tmax);
    const float alpha = fast_exp2(st.m - mn);
    float pw[8], psum = 0.f;
#pragma unroll
    for (int r = 0; r < 8; ++r) { pw[r] = fast_exp2(sv[r] - mn); psum += pw[r]; }
    st.l = st.l * alpha + psum;
    st.m = mn;
    if (kScaled) {
#pragma unroll
        for (int r = 0; r < 4; ++r) { pw[r] *= vs0; pw[4 + r] *= vs1; }
    }
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

constexpr int kMaxStates = 16;                         // states the ring holds at most
constexpr int kKStageBytes = 8192;                     // one 32-token K tile of a 16-bit cache (D = 128)

// Shared-memory layout for a batch of B requests and G columns per KV head: as many states (up to sixteen) as fit
// while two workgroups still share the 160 KB of a compute unit.  Four is the least the kernel works with (one state
// per wave: one request at a time); where not even four fit beside the plan's arrays (thousands of requests with 16
// columns), the layout keeps four and `two_per_cu` is false: the launch is still valid, with one workgroup per
// compute unit.
constexpr int kLdsPerWorkgroup = 80 * 1024 - 512;      // half a compute unit's shared memory less the kernel's own variables
inline MfmaLds mfma_lds_layout(int B, int G, bool kv8, bool staged, bool query_counts = false) {
    constexpr int D = 128;
    MfmaLds L;
    L.ring_off = (((query_counts ? 3 : 2) * B + 1) * 4 + 15) & ~15;      // E[B + 1], Lc[B] and, if asked for, Nc[B]
    L.state_floats = G * (D + 4) + 2 * kMaxGroup;
    L.static_bytes = staged ? kWaves * (kv8 ? kKStageBytes / 2 : kKStageBytes) : 0;   // the waves' K tiles
    const int budget = kLdsPerWorkgroup - L.ring_off - L.static_bytes;
    const int cap = budget / (L.state_floats * 4);
    L.two_per_cu = cap >= kWaves;
    L.ring_states = cap > kMaxStates ? kMaxStates : (cap < kWaves ? kWaves : cap);
    L.total = L.ring_off + L.ring_states * L.state_floats * 4;
    return L;
}

// A range (or a chunk of it) of `clen` tiles is dealt to the four waves in contiguous runs: wave w takes tiles
// run_start(w) .. run_start(w + 1) - 1 of the chunk.  With fewer than four tiles, waves 0 .. clen - 1 take one each.
__device__ __forceinline__ int run_start(int clen, int w) { return clen >= kWaves ? (clen * w) >> 2 : min(w, clen); }
// The wave whose run holds tile x of the chunk (0 <= x < clen).
__device__ __forceinline__ int wave_of_tile(int clen, int x) {
    return (x >= run_start(clen, 1)) + (x >= run_start(clen, 2)) + (x >= run_start(clen, 3));
}

// Combine the `cnt` consecutive states (m, l, o) that the waves left for one request's piece of a chunk and store the
// result: the normalised output if the request lies inside one range, else the unnormalised values (plus, once per
// head, the running max and sum) into the piece's partial-result slot.  Every thread owns four consecutive output
// elements.  All threads call it between barriers.
template <int D, bool MT>
__device__ __forceinline__ void mfma_combine_states(const float *first, int cnt, int state_floats, const AttnParams &p,
                                                    const Segment &seg, int kvh, int n_tokens = 1) {
    const int G = MT ? p.Gq : p.G;                       // columns: (query token, head) pairs of the KV head
    for (int idx = 4 * threadIdx.x; idx < G * D; idx += 4 * kThreads) {
        const int g = idx / D, d = idx - g * D;
        // a request's piece lies in at most four runs: all four reads are issued before any is used (a state that is
        // not part of the piece is read from the first one and dropped)
        float mu[kWaves], lu[kWaves];
        float4 ou[kWaves];
#pragma unroll
        for (int u = 0; u < kWaves; ++u) {
            const float *st = first + (u < cnt ? u : 0) * state_floats;
            mu[u] = st[G * (D + 4) + g];
            lu[u] = st[G * (D + 4) + kMaxGroup + g];
            ou[u] = *reinterpret_cast<const float4 *>(st + g * (D + 4) + d);
        }
        float M = -INFINITY;
#pragma unroll
        for (int u = 0; u < kWaves; ++u) {
            if (u >= cnt) mu[u] = -INFINITY;
            M = fmaxf(M, mu[u]);
        }
        float4 num = make_float4(0.f, 0.f, 0.f, 0.f);
        float den = 0.f;
#pragma unroll
        for (int u = 0; u < kWaves; ++u) {
            if (mu[u] > -INFINITY) {
                const float a = fast_exp2(mu[u] - M);
                num.x += a * ou[u].x; num.y += a * ou[u].y; num.z += a * ou[u].z; num.w += a * ou[u].w;
                den += a * lu[u];
            }
        }
        if (MT && p.t_off + g / p.G >= n_tokens) {           // no query token behind this column: zeros, weight 0
            num = make_float4(0.f, 0.f, 0.f, 0.f);
            den = 0.f;
        }
        if (seg.nparts == 1) {
            const size_t o0 = (MT ? out_row(p, seg.b, kvh, g) : (size_t)seg.b * p.Hq + kvh * G + g) * D + d;
            const bool live = den > 0.f;
            store_out4(p, o0, make_float4(live ? num.x / den : 0.f, live ? num.y / den : 0.f, live ? num.z / den : 0.f,
                                          live ? num.w / den : 0.f));
        } else {
            const size_t pi = MT ? partial_row(p, seg.slot, kvh, g) : (size_t)seg.slot * p.Hq + kvh * G + g;
            *reinterpret_cast<float4 *>(p.ws.part_o + pi * D + d) = num;
            if (d == 0) p.ws.part_ml[pi] = make_float2(M, den);
        }
    }
}

// The tiles of a range are dealt to the four waves in contiguous runs, so a wave holds one online-softmax state per
// request its run touches: four states plus one per request boundary that falls inside a run, whatever the number
// of requests (dealt round-robin, every request would leave four).  A wave leaves each finished state in shared memory
// and goes on; the workgroup meets once, when the range is done: one barrier, then every thread combines, request by
// request, the one to four consecutive states that belong to it.  A range that holds more requests than the states'
// area has room for (all but three of its states) is taken in chunks of that many requests, with the same meeting
// after each chunk.
// KV8: the pools hold 8-bit E4M3 bytes with one scale per (page, KV head); queries stay bf16.
// KST: K tiles go through the per-wave staging area in shared memory (the host chooses it where room for enough
// states is left beside it); otherwise they are loaded straight into the operand registers.
// MT: several query tokens per request (the columns are (query token, head) pairs with a causal limit each); the
// one-token kernel is compiled without any of it.
template <int PS, bool KV8 = false, bool KST = true, bool MT = false>
__global__ __launch_bounds__(kThreads, 2) void decode_mfma_kernel(AttnParams p) {
    constexpr int D = 128;
    constexpr int ES = KV8 ? 1 : 2;                          // bytes per cache element
    constexpr int kLog2Ps = (PS == 16) ? 4 : 5;
    __shared__ PlanSmem ps;
    extern __shared__ __align__(16) int E[];                 // E[B + 1] tile offsets, then Lc[B] lengths, then the ring
    __shared__ __align__(16) char kstage_all[KST ? kWaves * (KV8 ? kKStageBytes / 2 : kKStageBytes) : 16];  // a K tile per wave
    float *ring = reinterpret_cast<float *>(reinterpret_cast<char *>(E) + p.lds.ring_off);
    const int state_floats = p.lds.state_floats;
    const int max_seg = p.lds.ring_states - (kWaves - 1);    // requests a chunk may hold: the states then fit

    int w, kvh;
    wg_coords(p, &w, &kvh);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int col = lane & 15, j = lane >> 4;
    const int G = p.G, Gq = MT ? p.Gq : G;                       // heads per KV head; columns = query tokens x heads
    const int head0 = kvh * G;
    const int col_qi = (MT && col < Gq) ? col / G : 0;           // this lane's column: query token, head, and how many
    const int col_g = col - col_qi * G;                          // of the request's newest tokens it must not see
    const int tokens = MT ? p.Tq : 1;                            // query tokens per request, t_off .. in this launch
    const int t_off = MT ? p.t_off : 0;
    const int col_tok = t_off + col_qi;                          // which of the request's query tokens

    MfmaTileLoader<PS> ld;
    ld.page_stride = (size_t)p.Hkv * PS * D * ES;
    ld.kbase = reinterpret_cast<const char *>(p.k_cache) + (size_t)kvh * PS * D * ES;
    ld.vbase = reinterpret_cast<const char *>(p.v_cache) + (size_t)kvh * PS * D * ES;
    ld.koff = col * 256 + j * 16;
    ld.voff = col * 16 + (4 * j) * 256;
    ld.init_staging(lane);
    char *kstage = kstage_all + (KST ? wave * (KV8 ? kKStageBytes / 2 : kKStageBytes) : 0);
    Mfma8TileLoader<PS> ld8;
    ld8.page_stride = ld.page_stride; ld8.kbase = ld.kbase; ld8.vbase = ld.vbase;
    ld8.k_scale = KV8 ? p.k_scale + kvh : nullptr; ld8.v_scale = KV8 ? p.v_scale + kvh : nullptr;
    ld8.Hkv = p.Hkv;
    ld8.koff = col * 128 + j * 32;
    ld8.voff = col * 8 + (4 * j) * 128;
    ld8.init_staging(lane);

    // Several query tokens per request: Nc[b] = how many request b brings (behind E[] and Lc[] in shared memory).
    int *Nc = E + 2 * p.plan.B + 1;
    auto load_q = [&](int b, uint4 (&Q)[4]) {                    // B operand of K Q^T for request b
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) Q[kk] = make_uint4(0, 0, 0, 0);
        if (col < Gq && (!MT || t_off + col_qi < Nc[b])) {       // a column no query token stands behind keeps zeros
            const char *qrow = reinterpret_cast<const char *>(p.q) + (((size_t)b * tokens + t_off + col_qi) * p.Hq + head0 + col_g) * (D * 2);
#pragma unroll
            for (int kk = 0; kk < 4; ++kk)                      // dims of step kk: (4kk + j) * 8 .., or 32j + 8kk .. (KV8)
                Q[kk] = *reinterpret_cast<const uint4 *>(qrow + (KV8 ? 4 * j + kk : 4 * kk + j) * 16);
        }
    };

    // Tile offsets and lengths of all requests, in shared memory.
    const int *Lc = E + p.plan.B + 1;
    const bool wave_plan = p.plan.B <= kWavePlanMax;         // small batch: every wave plans for itself, no barrier
    WavePlan wp{0, 0, 0, 0};
    Plan pl;
    if (wave_plan) {
        unsigned long long T = 0;
        const bool first = blockIdx.x == 0 && wave == 0;
        pl = plan_build_wave(p.context_lens, p.plan, E, E + p.plan.B + 1, &wp, w == 0 && wave == 0,
                             [&](int b) { wave_zero_rows<D>(p, b, kvh); }, T);
        if (first && lane == 0) {
            p.ws.plan_words[0] = pl.S * kTile; p.ws.plan_words[1] = pl.nranges;
            p.ws.plan_words[2] = (int)(T & 0xffffffffULL); p.ws.plan_words[3] = (int)(T >> 32);
        }
    } else {
        pl = attn_prologue<D>(p, &ps, E, w, kvh);
    }
    if constexpr (MT) {                                          // every wave writes the same values: no barrier needed
        for (int b = lane; b < p.plan.B; b += 64) {
            const int n = p.q_lens ? p.q_lens[b] : tokens;
            Nc[b] = min(max(n, 0), tokens);
        }
    }

    for (int range = w; range < pl.nranges; range += p.plan.nw) {
        const int start = range * pl.S, end = min(pl.C, start + pl.S);
        int cs = start;                  // first tile of the chunk
        int cb = wave_plan ? wave_first_request(wp, start) : plan_first_request(p.plan, &ps, E, start);   // its request
      while (cs < end) {                 // chunks of the range: normally one
        // ---- the chunk: up to max_seg requests from tile cs on; nb = the request the next chunk starts with
        int ce = end, nb = cb;
        // (with the plan in registers the common case needs no walk: the requests up to the one that holds the range's
        // last tile, empty ones included, are no more than a chunk may hold)
        if (!(wave_plan && wave_first_request(wp, end - 1) - cb < max_seg)) {
            int bb = cb;
            for (int nseg = 1;; ++nseg) {
                const int e1 = __builtin_amdgcn_readfirstlane(E[bb + 1]);
                if (e1 >= end) break;                            // the request reaches the end of the range
                do { ++bb; } while (__builtin_amdgcn_readfirstlane(E[bb + 1]) == __builtin_amdgcn_readfirstlane(E[bb]));   // next request that owns tiles (one exists: e1 < C)
                if (nseg == max_seg) { ce = e1; nb = bb; break; }
            }
        }
        const int clen = ce - cs;
        const int r0 = run_start(clen, wave), nk = run_start(clen, wave + 1) - r0;     // this wave's run of the chunk's tiles
        const int first_b = cb;
        // the request that holds the chunk's last tile bounds every lane's search below: a chunk rarely spans more than
        // two or three requests, so the search takes one or two steps instead of log2(B)
        const int search_hi = wave_plan ? wave_first_request(wp, ce - 1) + 1 : p.plan.B;

        // ---- this wave's tiles: tile r0 + slot of the chunk, slot = 0 .. nk-1.  Lane s of the wave looks up
        // everything about slot s (of the current group of 64 slots) once: the request, the tile's index inside the
        // request and its physical pages.  The tile loop then only picks values out with v_readlane, so neither the
        // block table nor the plan sits between two tiles, also across request boundaries.
        int4 meta = make_int4(-1, 0, 0, 0);                      // request, tile in request, page of tokens 0-15, 16-31
        auto fetch_meta = [&](int first_slot) {
            const int slot = first_slot + lane;
            meta = make_int4(-1, 0, 0, 0);
            if (slot < nk) {
                const int pos = cs + r0 + slot;
                int lo = first_b, hi = search_hi;                // E[lo] <= pos < E[hi]
                while (hi - lo > 1) {
                    const int mid = (lo + hi) >> 1;
                    if (E[mid] <= pos) lo = mid; else hi = mid;
                }
                const int t = pos - E[lo];
                const int last_page = (Lc[lo] - 1) >> kLog2Ps;
                const int32_t *bt = p.block_table + (size_t)lo * p.MB;
                const int page = (t * kTile) >> kLog2Ps;
                meta.x = lo;
                // fused step: the tiles that hold the request's newest token(s) get their rows written first
                bool newest = t == ((Lc[lo] - 1) >> kLog2Tile);
                if (MT) newest = Nc[lo] > 0 && t <= ((Lc[lo] - 1) >> kLog2Tile) && t >= (max(Lc[lo] - Nc[lo], 0) >> kLog2Tile);
                meta.y = t | ((p.k_new != nullptr && newest) ? kAppendFlag : 0);
                if (PS == 16 && page < last_page) {              // both pages exist: one 8-byte read (page is even)
                    struct alignas(4) PagePair { int first, second; };   // rows of odd length keep 4-byte alignment
                    const PagePair pp2 = *reinterpret_cast<const PagePair *>(bt + page);
                    meta.z = pp2.first; meta.w = pp2.second;
                } else {                                         // never read beyond the request's pages
                    meta.z = bt[page]; meta.w = meta.z;
                }
            }
        };
        fetch_meta(0);
        struct SlotInfo { int req, tile, pg0, pg1; bool append; };
        auto slot_info = [&](int slot) {
            SlotInfo si{-1, 0, 0, 0, false};
            if (slot >= nk) return si;
            if ((slot & 63) == 0 && slot > 0) fetch_meta(slot);  // rare: more than 64 tiles per wave in a range
            const int l = slot & 63;
            const int ty = __builtin_amdgcn_readlane(meta.y, l);
            si.req = __builtin_amdgcn_readlane(meta.x, l); si.tile = ty & ~kAppendFlag; si.append = (ty & kAppendFlag) != 0;
            si.pg0 = __builtin_amdgcn_readlane(meta.z, l); si.pg1 = __builtin_amdgcn_readlane(meta.w, l);
            return si;
        };
        // Fused decode step, with several query tokens per request or K loaded straight into registers: the tile that
        // holds the request's last token gets the new K/V row written into its page (a bit copy, the first lanes the K
        // row, the next ones the V row, 16 bytes each) before the tile is requested; the wave waits for the write to be
        // acknowledged, so the loads that follow see it.  With several query tokens per request the new rows are
        // [B, T, Hkv, D] and each tile takes those of the request's last T positions that fall into it.
        constexpr int kRowPieces = D * ES / 16;                  // 16-byte pieces of a row: 16 (16-bit cache) or 8
        auto append_row = [&](const SlotInfo &si) {
            const int L = Lc[si.req];
            const int n_new = MT ? Nc[si.req] : 1;               // rows 0 .. n_new - 1 of the request's new rows
#pragma unroll 1
            for (int qi = 0; qi < n_new; ++qi) {
                const int pos = L - n_new + qi;
                if (MT && (pos < 0 || (pos >> kLog2Tile) != si.tile)) continue;      // uniform
                const int pg = (PS == 16 && (pos & 16)) ? si.pg1 : si.pg0;
                const size_t row = (size_t)pg * ld.page_stride + (size_t)(pos & (PS - 1)) * (D * ES);
                if (lane < 2 * kRowPieces) {
                    const bool is_v = lane >= kRowPieces;
                    const int piece = lane & (kRowPieces - 1);
                    const char *src = reinterpret_cast<const char *>(is_v ? p.v_new : p.k_new) +
                                      (((size_t)si.req * tokens + qi) * p.Hkv + kvh) * (D * ES) + piece * 16;
                    char *dst = const_cast<char *>(is_v ? ld.vbase : ld.kbase) + row + piece * 16;
                    *reinterpret_cast<uint4 *>(dst) = *reinterpret_cast<const uint4 *>(src);
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_s_waitcnt(0);           // all counters: the row is in memory before the tile is read
        };
        // One query token per request and K staged: no wait at all.  The new rows are asked for together with the
        // tile's loads (every lane one 16-byte piece of each); when the tile has arrived the K row is written over its
        // place in the staging area, the V row over the registers of the lanes that hold that token, and both go to
        // their page with stores nobody waits for: within this launch only this wave reads that row of that KV head.
        constexpr bool kPatchAppend = KST && !MT;
        int patch_row = -1;                                      // the new token's place in the tile in flight, or none
        size_t patch_dst = 0;                                    // byte offset of its row behind kbase / vbase
        uint4 Kn = make_uint4(0, 0, 0, 0), Vn = make_uint4(0, 0, 0, 0);
        auto request_new_row = [&](const SlotInfo &si) {
            const int pos = __builtin_amdgcn_readfirstlane(Lc[si.req]) - 1;
            patch_row = pos - si.tile * kTile;
            const int pg = (PS == 16 && (pos & 16)) ? si.pg1 : si.pg0;
            patch_dst = (size_t)pg * ld.page_stride + (size_t)(pos & (PS - 1)) * (D * ES);
            const size_t src = ((size_t)si.req * p.Hkv + kvh) * (D * ES);
            Kn = *reinterpret_cast<const uint4 *>(reinterpret_cast<const char *>(p.k_new) + src + (lane & (kRowPieces - 1)) * 16);
            if constexpr (KV8) {                                 // a lane's V piece is 8 bytes there: dims 8 col ..
                const uint2 v8 = *reinterpret_cast<const uint2 *>(reinterpret_cast<const char *>(p.v_new) + src + col * 8);
                Vn.x = v8.x; Vn.y = v8.y;
            } else {
                Vn = *reinterpret_cast<const uint4 *>(reinterpret_cast<const char *>(p.v_new) + src + col * 16);
            }
        };

        // Software pipeline of one wave (single K and V buffers): the K rows of the next tile are requested as soon
        // as the scores of the current tile have consumed K, its V rows as soon as the accumulation has consumed V,
        // and the next request's query as soon as the last scores of the current request are done.  The requests
        // stay in flight across the end-of-segment exchange below.
        uint4 K[KV8 ? 1 : 8], V[8], Q[4];
        uint4 Kr[KV8 ? 4 : 1];           // 8-bit cache: the raw bytes of a tile and the scales of its two pages
        uint2 Vr[KV8 ? 8 : 1];
        float ks[2] = {1.f, 1.f}, vs[2] = {1.f, 1.f};
        auto issue_k = [&](int pg0, int pg1) __attribute__((always_inline)) {
            if constexpr (KST) {
                if constexpr (KV8) ld8.issue_k_staged(pg0, pg1, kstage, ks); else ld.issue_k_staged(pg0, pg1, kstage);
            } else {
                if constexpr (KV8) ld8.issue_k(pg0, pg1, Kr, ks); else ld.issue_k(pg0, pg1, K);
            }
        };
        auto issue_v = [&](int pg0, int pg1) __attribute__((always_inline)) {
            if constexpr (KV8) ld8.issue_v(pg0, pg1, Vr, vs); else ld.issue_v(pg0, pg1, V);
        };
        int s = 0;                       // slot being computed; its loads are in flight
        SlotInfo cur = slot_info(0);
        if (cur.req >= 0) {
            if (cur.append) { if constexpr (kPatchAppend) request_new_row(cur); else append_row(cur); }
            issue_k(cur.pg0, cur.pg1);
            load_q(cur.req, Q);
            issue_v(cur.pg0, cur.pg1);
        }
        __builtin_amdgcn_sched_barrier(0);       // nothing below may move in front of the first tile's loads

        // where this wave's states go: behind those of the waves before it (one per wave with a run, and one more for
        // every request that begins inside a run); worked out while the first tile is on its way
        int wbase = 0;
        for (int ww = 0; ww < wave; ++ww) wbase += run_start(clen, ww + 1) > run_start(clen, ww) ? 1 : 0;
        if (wave_plan) {                 // from the plan in registers: the boundaries in front of this wave's run ...
            const int mine = run_start(clen, wave);
            wbase += wave_count_ends(wp, cs, cs + mine);
            for (int ww = 1; ww < wave; ++ww)                    // ... less those a run begins with
                if (run_start(clen, ww) < mine) wbase -= wave_count_ends(wp, cs + run_start(clen, ww) - 1, cs + run_start(clen, ww) + 1);
        } else {
            int bb = cb;
            while (true) {
                const int e1 = __builtin_amdgcn_readfirstlane(E[bb + 1]) - cs;   // where the next request begins, in the chunk
                if (e1 >= clen) break;
                const int ww = wave_of_tile(clen, e1);
                if (ww < wave && e1 != run_start(clen, ww)) ++wbase;
                do { ++bb; } while (__builtin_amdgcn_readfirstlane(E[bb + 1]) == __builtin_amdgcn_readfirstlane(E[bb]));
            }
        }
        int nstate = 0;                  // states this wave has left in shared memory for this chunk
        while (cur.req >= 0) {           // one pass per request the wave's run touches
            const int b = cur.req;
            const Segment seg = plan_segment(E, Lc, pl, b, range, start, end);
            // several query tokens: query i of the request's n sits at position L - n + i; a column with no query behind
            // it runs unmasked on zero queries and is dropped when the segment is combined
            const int seg_n = MT ? __builtin_amdgcn_readfirstlane(Nc[b]) : 1;
            const int col_back = (MT && col < Gq && col_tok < seg_n) ? seg_n - 1 - col_tok : 0;
            const int t1min = MT ? seg.L - max(seg_n - 1 - t_off, 0) : seg.L;
            MfmaState st;
            st.m = -INFINITY; st.l = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) st.acc[e] = f32x4_t{0.f, 0.f, 0.f, 0.f};
            while (cur.req == seg.b) {
                const SlotInfo nxt = slot_info(s + 1);
                const bool more = nxt.req >= 0;
                float sv[8];
                float ks_cur[2] = {ks[0], ks[1]};                // scales of this tile's K (8-bit cache)
                if constexpr (KST) {
                    // The copy into shared memory is complete when every load of this wave is (vmcnt = 0; the compiler
                    // does not order shared-memory reads behind such copies by itself).  This one wait also covers the V
                    // rows and the query asked for at the end of the previous tile, so nothing below waits for memory:
                    // the compiler would turn any wait for an older load into one for all loads while a copy into
                    // shared memory is in flight.
                    __builtin_amdgcn_s_waitcnt(0x0f70);
                    if constexpr (kPatchAppend) {
                        if (patch_row >= 0) {                    // this tile holds its request's new token (uniform)
                            const int blk = patch_row >> 4, row = patch_row & 15;
                            if (lane < kRowPieces) {             // piece `lane` of the K row: staging area, and its page
                                *reinterpret_cast<uint4 *>(kstage + blk * (kRowPieces * 256) + row * (D * ES) +
                                                           (((lane ^ row) & (kRowPieces - 1)) << 4)) = Kn;
                                *reinterpret_cast<uint4 *>(const_cast<char *>(ld.kbase) + patch_dst + lane * 16) = Kn;
                            }
                            if (lane < 16) {                     // piece `lane` of the V row to its page
                                char *vdst = const_cast<char *>(ld.vbase) + patch_dst;
                                if constexpr (KV8) *reinterpret_cast<uint2 *>(vdst + lane * 8) = make_uint2(Vn.x, Vn.y);
                                else *reinterpret_cast<uint4 *>(vdst + lane * 16) = Vn;
                            }
#pragma unroll
                            for (int r = 0; r < 8; ++r) {        // the lane group that holds the token takes the new V
                                if (slot_token(j, r) == patch_row) {
                                    if constexpr (KV8) Vr[r] = make_uint2(Vn.x, Vn.y); else V[r] = Vn;
                                }
                            }
                            patch_row = -1;
                        }
                    }
                    ks_cur[0] = ks[0]; ks_cur[1] = ks[1];
                    if constexpr (KV8) ld8.read_k_staged(kstage, Kr); else ld.read_k_staged(kstage, K);
                    __builtin_amdgcn_s_waitcnt(0xc07f);          // operands are in registers (lgkmcnt = 0) ...
                    if (more) {                                  // ... so the next tile may take their place
                        if (nxt.append) { if constexpr (kPatchAppend) request_new_row(nxt); else append_row(nxt); }
                        issue_k(nxt.pg0, nxt.pg1);
                    }
                    if constexpr (KV8) mfma_scores_fp8(Kr, Q, sv, p.scale_log2, ks_cur);
                    else mfma_scores(K, Q, sv, p.scale_log2);
                } else {
                    if constexpr (KV8) mfma_scores_fp8(Kr, Q, sv, p.scale_log2, ks);
                    else mfma_scores(K, Q, sv, p.scale_log2);
                    if (more) {
                        if (nxt.append) append_row(nxt);
                        issue_k(nxt.pg0, nxt.pg1);
                        if (nxt.req != seg.b) load_q(nxt.req, Q);
                    }
                }
                if constexpr (KV8) {
                    const float v0 = vs[0], v1 = vs[1];          // of the current tile: the next V request replaces them
#pragma unroll
                    for (int r = 0; r < 8; ++r) V[r] = fp8x8_to_bf16x8(Vr[r].x, Vr[r].y);
                    if (more) {                                  // the raw V bytes are consumed: request the next ones
                        if (KST && nxt.req != seg.b) load_q(nxt.req, Q);
                        issue_v(nxt.pg0, nxt.pg1);
                    }
                    mfma_softmax_pv<true, MT>(sv, V, st, cur.tile * kTile, seg.L, seg.L - col_back, t1min, j, v0, v1);
                } else {
                    mfma_softmax_pv<false, MT>(sv, V, st, cur.tile * kTile, seg.L, seg.L - col_back, t1min, j);
                    if (more) {
                        if (KST && nxt.req != seg.b) load_q(nxt.req, Q);
                        issue_v(nxt.pg0, nxt.pg1);
                    }
                }
                ++s; cur = nxt;
            }

            // ---- end of the wave's share of this request: it leaves its state in shared memory and goes on
            st.l += __shfl_xor(st.l, 16);                        // per-lane sums of the four lane groups; m is common
            st.l += __shfl_xor(st.l, 32);
            float *state = ring + (size_t)(wbase + nstate) * state_floats;
            ++nstate;
            if (col < Gq) {
                float *orow = state + col * (D + 4);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    float4 lo4 = make_float4(st.acc[0][i], st.acc[1][i], st.acc[2][i], st.acc[3][i]);
                    float4 hi4 = make_float4(st.acc[4][i], st.acc[5][i], st.acc[6][i], st.acc[7][i]);
                    *reinterpret_cast<float4 *>(orow + 32 * j + 8 * i) = lo4;
                    *reinterpret_cast<float4 *>(orow + 32 * j + 8 * i + 4) = hi4;
                }
                if (j == 0) {
                    float *sm_m = state + Gq * (D + 4);
                    sm_m[col] = st.m; sm_m[kMaxGroup + col] = st.l;
                }
            }
        }

        // ---- the chunk is done: the workgroup meets and combines, request by request, the states that belong to it
        // (consecutive ones: the runs are in tile order).  Which states a request has depends on the plan alone, so the
        // first request's are worked out before the meeting and each further one's while the stores of the one before
        // are on their way.
        {
            int bb = cb, at = 0, e1, cnt;
            Segment sg;
            auto piece = [&]() {
                const int e0 = __builtin_amdgcn_readfirstlane(E[bb]);
                e1 = __builtin_amdgcn_readfirstlane(E[bb + 1]);
                const int lo = max(e0, cs) - cs, hi = min(e1, ce) - cs;              // the request's tiles in the chunk
                cnt = wave_of_tile(clen, hi - 1) - wave_of_tile(clen, lo) + 1;
                sg = plan_segment(E, Lc, pl, bb, range, start, end);
            };
            piece();
            lds_barrier();
            while (true) {
                mfma_combine_states<D, MT>(ring + (size_t)at * state_floats, cnt, state_floats, p, sg, kvh, MT ? Nc[bb] : 1);   // nobody waits for its stores
                at += cnt;
                if (e1 >= ce) break;
                do { ++bb; } while (__builtin_amdgcn_readfirstlane(E[bb + 1]) == __builtin_amdgcn_readfirstlane(E[bb]));
                piece();
            }
        }
        lds_barrier();
        cs = ce; cb = nb;
      }
    }
    if (blockIdx.x == 0) write_merge_records(p, pl, E);
}

}  // namespace omni
