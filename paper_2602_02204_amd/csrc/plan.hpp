// Device-side work decomposition ("stream" split of the context), recomputed identically by every workgroup.
//
// The host never sees context_lens (they live on the device and the library never synchronises), so the launch grid is
// data-independent: nw workgroups per KV head.  Each workgroup derives the same plan from the lengths:
//   - request b owns c_b = ceil(L_b / 32) tiles of 32 tokens; the tiles of all requests are laid end to end
//     (E_b = tiles before request b, C = all tiles);
//   - the line of C tiles is cut into ranges of S tiles, S = max(s_min, ceil(C / nw)) unless forced, so every range
//     carries the same number of tiles whatever the mix of request lengths;
//   - workgroup w of a KV head takes range w (and w + nw, ... if there are more ranges than workgroups).
// A range crosses request boundaries wherever they fall: it is a list of segments (request, first tile, last tile).
// A request covered by one range is finished by that workgroup; a request cut by range boundaries yields one partial
// result per range that touches it, put together by the merge kernel that follows.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace omni {

constexpr int kThreads = 256;          // threads per workgroup in every kernel of the attention path
constexpr int kWaves = kThreads / 64;
constexpr int kTile = 32;              // tokens per tile: the granularity of ranges and segments
constexpr int kLog2Tile = 5;

struct PlanParams {
    int B;
    int nw;              // workgroups per KV head
    int s_min;           // smallest range length in tiles the plan may pick (>= 1)
    int s_force;         // > 0: use exactly this range length in tiles
};

// One piece of one request inside one range.
struct Segment {
    int b;               // request
    int lo, hi;          // tiles [lo, hi) of the request
    int L;               // context length of the request (tokens)
    int nparts;          // ranges that touch this request
    int slot;            // partial-result slot of this segment (range index + request index: unique, and
                         // consecutive over the ranges of one request)
    int slot_first;      // slot of the request's first segment
};

__device__ __forceinline__ int ceil_div(int a, int b) { return (a + b - 1) / b; }

// Barrier that orders shared-memory traffic only: global loads issued before it stay in flight across it.
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Shared-memory part of the plan.  The dynamic shared memory of the kernel holds E[0..B] (exclusive prefix of tile
// counts, E[B] = C) followed by Lc[0..B) (context lengths clamped at 0).
struct PlanSmem {
    int wave_tot[kWaves];
    int first_b;         // request holding the first tile of the current range
    unsigned long long total_tokens;
};

struct Plan {
    int S;               // range length in tiles
    int C;               // all tiles
    int nranges;
};

// The cut of a line of C tiles into ranges.
__device__ __forceinline__ Plan plan_cut(const PlanParams &pp, int C) {
    Plan pl;
    pl.C = C;
    const int S = pp.s_force > 0 ? pp.s_force : max(pp.s_min, ceil_div(C, pp.nw));
    pl.S = max(S, 1);
    pl.nranges = ceil_div(C, pl.S);
    return pl;
}

// Inclusive scan over the 256 threads of the workgroup (two shared-memory barriers).
__device__ __forceinline__ int block_inclusive_scan(int v, PlanSmem *ps, int *total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int t = __shfl_up(v, off);
        if (lane >= off) v += t;
    }
    lds_barrier();                         // wave_tot may still be read from the previous round
    if (lane == 63) ps->wave_tot[wave] = v;
    lds_barrier();
    int add = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        const int s = ps->wave_tot[w];
        if (w < wave) add += s;
        tot += s;
    }
    *total = tot;
    return v + add;
}

// Build E[] and Lc[] in shared memory and choose S.  All 256 threads call this.  Requests of length <= 0 own no
// tile; `zero_row(b)` is invoked for each of them by all lanes of one wave together (a wave-uniform call), so that the
// caller can write their all-zero output with whole-wave stores.
// `first_len` is context_lens[threadIdx.x] if the caller has already loaded it (have_first), so that the load can be
// issued ahead of other traffic.  Only shared memory is synchronised: global loads in flight are not waited for.
template <typename ZeroRow>
__device__ __forceinline__ Plan plan_build(const int32_t *__restrict__ lens, const PlanParams &pp, PlanSmem *ps, int *E,
                                           int *Lc, ZeroRow zero_row, int first_len = 0, bool have_first = false) {
    if (threadIdx.x == 0) ps->total_tokens = 0;
    int carry = 0;
    unsigned long long tokens = 0;
    for (int base = 0; base < pp.B; base += kThreads) {
        const int b = base + threadIdx.x;
        int c = 0, L = 0;
        bool empty = false;
        if (b < pp.B) {
            L = (have_first && base == 0) ? first_len : lens[b];
            if (L > 0) { c = (L + kTile - 1) >> kLog2Tile; tokens += (unsigned long long)L; }
            else empty = true;
        }
        for (unsigned long long em = __ballot(empty); em; em &= em - 1)       // each wave takes its own empty requests
            zero_row(base + (int)(threadIdx.x & ~63u) + (int)__builtin_ctzll(em));
        int tot;
        const int incl = block_inclusive_scan(c, ps, &tot) + carry;
        if (b < pp.B) { E[b] = incl - c; Lc[b] = c ? L : 0; }
        carry += tot;
    }
    if (threadIdx.x == 0) E[pp.B] = carry;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) tokens += __shfl_xor(tokens, off);
    if ((threadIdx.x & 63) == 0 && tokens) atomicAdd(&ps->total_tokens, tokens);
    lds_barrier();
    return plan_cut(pp, __builtin_amdgcn_readfirstlane(carry));
}

// ---- Plan without workgroup barriers, for batches of up to kWavePlanMax requests.
// Every wave loads all the lengths itself (lane l holds requests 4l .. 4l+3), scans them with cross-lane shuffles and
// writes E[] and Lc[] to shared memory.  The waves of a workgroup store identical values to the same words, so a wave
// may read the arrays as soon as its own stores are done: no wave waits for another before its first table read.
constexpr int kWavePlanMax = 256;

struct WavePlan {
    int i0, i1, i2, i3;  // tiles up to and including request 4*lane + i (requests beyond the batch own no tile)
    int owns;            // bit i: request 4*lane + i owns at least one tile
};

// `zero_row(b)` is called, by all lanes of the wave together, for each request of length <= 0 if `zero_rows`;
// `total_tokens` receives the sum of the lengths (in every lane).
template <typename ZeroRow>
__device__ __forceinline__ Plan plan_build_wave(const int32_t *__restrict__ lens, const PlanParams &pp, int *E, int *Lc,
                                                WavePlan *wp, bool zero_rows, ZeroRow zero_row,
                                                unsigned long long &total_tokens) {
    const int lane = threadIdx.x & 63;
    int L[4], c[4], incl[4];
    if ((reinterpret_cast<uintptr_t>(lens) & 15) == 0 && 4 * lane + 3 < pp.B) {   // one 16-byte load where it may be:
        const int4 v = *reinterpret_cast<const int4 *>(lens + 4 * lane);         // a quarter of the requests to the L2
        L[0] = v.x; L[1] = v.y; L[2] = v.z; L[3] = v.w;
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int b = 4 * lane + i;
            L[i] = b < pp.B ? lens[b] : 0;
        }
    }
    int run = 0;
    unsigned long long tokens = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int b = 4 * lane + i;
        if (L[i] > 0) { c[i] = (L[i] + kTile - 1) >> kLog2Tile; tokens += (unsigned long long)L[i]; }
        else { c[i] = 0; L[i] = 0; }
        if (zero_rows)
            for (unsigned long long em = __ballot(c[i] == 0 && b < pp.B); em; em &= em - 1)
                zero_row(4 * (int)__builtin_ctzll(em) + i);
        run += c[i];
        incl[i] = run;
    }
    int scan = run;                              // inclusive scan of the lanes' totals
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int t = __shfl_up(scan, off);
        if (lane >= off) scan += t;
    }
    const int before = scan - run;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int b = 4 * lane + i;
        incl[i] += before;
        if (b < pp.B) { E[b] = incl[i] - c[i]; Lc[b] = L[i]; }
    }
    wp->i0 = incl[0]; wp->i1 = incl[1]; wp->i2 = incl[2]; wp->i3 = incl[3];
    wp->owns = (c[0] > 0 ? 1 : 0) | (c[1] > 0 ? 2 : 0) | (c[2] > 0 ? 4 : 0) | (c[3] > 0 ? 8 : 0);
    const int C = __builtin_amdgcn_readlane(scan, 63);
    if (lane == 0) E[pp.B] = C;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) tokens += __shfl_xor(tokens, off);
    total_tokens = tokens;
    return plan_cut(pp, C);
}

// Request that holds tile `start` (0 <= start < C): the number of requests that end at or before it.
__device__ __forceinline__ int wave_first_request(const WavePlan &wp, int start) {
    return __popcll(__ballot(wp.i0 <= start)) + __popcll(__ballot(wp.i1 <= start)) +
           __popcll(__ballot(wp.i2 <= start)) + __popcll(__ballot(wp.i3 <= start));
}

// Requests that own tiles and end strictly between tiles lo and hi of the line (their last tile is p - 1, lo < p < hi):
// the request boundaries inside the stretch.
__device__ __forceinline__ int wave_count_ends(const WavePlan &wp, int lo, int hi) {
    return __popcll(__ballot((wp.owns & 1) && wp.i0 > lo && wp.i0 < hi)) + __popcll(__ballot((wp.owns & 2) && wp.i1 > lo && wp.i1 < hi)) +
           __popcll(__ballot((wp.owns & 4) && wp.i2 > lo && wp.i2 < hi)) + __popcll(__ballot((wp.owns & 8) && wp.i3 > lo && wp.i3 < hi));
}

// Request that holds tile `start` (0 <= start < C).  All 256 threads call this; E[] must be complete.
__device__ __forceinline__ int plan_first_request(const PlanParams &pp, PlanSmem *ps, const int *E, int start) {
    lds_barrier();                         // previous readers of first_b are done
    for (int b = threadIdx.x; b < pp.B; b += kThreads)
        if (E[b] <= start && start < E[b + 1]) ps->first_b = b;     // exactly one request matches
    lds_barrier();
    return __builtin_amdgcn_readfirstlane(ps->first_b);
}

// Segment of request b inside range `range` = tiles [start, end) of the line.
__device__ __forceinline__ Segment plan_segment(const int *E, const int *Lc, const Plan &pl, int b, int range, int start,
                                                int end) {
    Segment s;
    const int e0 = __builtin_amdgcn_readfirstlane(E[b]), e1 = __builtin_amdgcn_readfirstlane(E[b + 1]);
    s.b = b;
    s.lo = max(start, e0) - e0;
    s.hi = min(end, e1) - e0;
    s.L = __builtin_amdgcn_readfirstlane(Lc[b]);
    const int first_range = e0 / pl.S, last_range = (e1 - 1) / pl.S;
    s.nparts = last_range - first_range + 1;
    s.slot = range + b;
    s.slot_first = first_range + b;
    return s;
}

}  // namespace omni
