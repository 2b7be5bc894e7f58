// Device-side split-context plan, recomputed identically by every workgroup.
//
// The host never sees context_lens (they live on the device and the library never synchronises), so the grid is a
// host-known bound and each workgroup derives the same plan from the lengths:
//   PL      partition length in tokens (multiple of 32), chosen so that the number of (request, partition) pairs
//           R = sum_b max(1, ceil(L_b / PL)) does not exceed R_target when that is possible at all;
//   item r  -> (request b, partition index, partitions of b, first r of b).
// Partitions of one request are equalised: a request cut n ways uses pieces of roundup32(ceil(L / n)) tokens.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace omni {

constexpr int kThreads = 256;          // threads per workgroup in every kernel of the attention path
constexpr int kWaves = kThreads / 64;
constexpr int kTile = 32;              // token granularity of partitions

struct PlanParams {
    int B;
    int r_target;        // (request, partition) pairs the plan aims for; <= B means "never split"
    int pl_min;          // smallest partition length the plan may pick (multiple of 32)
    int pl_force;        // > 0: use exactly this partition length
};

struct Item {
    int b, part, nparts, start, L, PL;
};

__device__ __forceinline__ int ceil_div(int a, int b) { return (a + b - 1) / b; }

__device__ __forceinline__ int piece_len(int L, int nparts) {
    int x = ceil_div(L, nparts);
    return (x + kTile - 1) & ~(kTile - 1);
}

// Inclusive scan over the 256 threads of the workgroup.  sm needs kWaves ints.  Returns the scan value; *total = sum.
__device__ __forceinline__ int block_inclusive_scan(int v, int *sm, int *total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        int t = __shfl_up(v, off);
        if (lane >= off) v += t;
    }
    __syncthreads();                       // sm may still be read from a previous call
    if (lane == 63) sm[wave] = v;
    __syncthreads();
    int add = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        int s = sm[w];
        if (w < wave) add += s;
        tot += s;
    }
    *total = tot;
    return v + add;
}

// Partition length for this batch.  Every thread returns the same value.  sm needs kWaves*2 ints.
__device__ __forceinline__ int plan_partition_len(const int32_t *__restrict__ lens, const PlanParams &pp, int *sm,
                                                  long long *total_tokens) {
    long long sum = 0;
    for (int b = threadIdx.x; b < pp.B; b += kThreads) sum += max(lens[b], 0);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off);
    long long *sm64 = reinterpret_cast<long long *>(sm);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sm64[threadIdx.x >> 6] = sum;
    __syncthreads();
    long long T = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) T += sm64[w];
    *total_tokens = T;
    if (pp.pl_force > 0) return pp.pl_force;
    if (pp.r_target <= pp.B) return 0x3fffffe0;                     // no split: one partition per request
    long long per = (T + (pp.r_target - pp.B) - 1) / (pp.r_target - pp.B);
    if (per < pp.pl_min) per = pp.pl_min;
    per = (per + 127) & ~127LL;                                     // whole 128-token strips (4 waves x 32 tokens)
    if (per > 0x3fffffe0) per = 0x3fffffe0;
    return (int)per;
}

// Find the item with global index r.  All 256 threads must call this (it synchronises).  Returns false when r is
// beyond the last item.  sm needs 16 ints.  *R_out (optional) receives the number of items.
__device__ __forceinline__ bool plan_find(const int32_t *__restrict__ lens, const PlanParams &pp, int r, int *sm,
                                          Item *it, int *R_out, long long *T_out) {
    long long T;
    const int PL = plan_partition_len(lens, pp, sm, &T);
    if (T_out) *T_out = T;
    int carry = 0;
    __syncthreads();
    if (threadIdx.x == 0) sm[8] = -1;
    for (int base = 0; base < pp.B; base += kThreads) {
        const int b = base + threadIdx.x;
        int L = 0, n = 0;
        if (b < pp.B) {
            L = max(lens[b], 0);
            n = max(1, ceil_div(L, PL));
        }
        int tot;
        const int incl = block_inclusive_scan(n, sm, &tot) + carry;   // its barriers order the sm[8] init above
        const int excl = incl - n;
        if (n > 0 && r >= excl && r < incl) {
            sm[8] = b; sm[9] = r - excl; sm[10] = n; sm[11] = excl; sm[12] = L;
        }
        carry += tot;
    }
    __syncthreads();
    if (R_out) *R_out = carry;
    if (sm[8] < 0) return false;
    // the item is the same for every thread: keep it in scalar registers
    it->b = __builtin_amdgcn_readfirstlane(sm[8]);
    it->part = __builtin_amdgcn_readfirstlane(sm[9]);
    it->nparts = __builtin_amdgcn_readfirstlane(sm[10]);
    it->start = __builtin_amdgcn_readfirstlane(sm[11]);
    it->L = __builtin_amdgcn_readfirstlane(sm[12]);
    it->PL = __builtin_amdgcn_readfirstlane(PL);
    return true;
}

}  // namespace omni
