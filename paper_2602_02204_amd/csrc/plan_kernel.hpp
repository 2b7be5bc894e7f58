// Plan kernel: runs before the MFMA attention kernel of the same call and writes the tile list of every
// (range, wave) into the workspace, so that the attention kernel's first memory request already is a K/V tile.
#pragma once
#include "common.hpp"

namespace omni {

// One workgroup per range (looping if there are more ranges than workgroups).  For range r, wave v, slot s the tile is
// g = v + 4 s of the range; the entry holds (request, tile index inside the request, physical page of its first
// 16 tokens, physical page of its second 16 tokens).  Entries past the range's last tile, and all entries of ranges
// that do not exist for this batch, are written as request -1: the attention kernel reads the entries of range
// blockIdx before it knows how many ranges there are, so every entry it may read is rewritten by every call.
template <int PS>
__global__ __launch_bounds__(kThreads) void plan_kernel(AttnParams p, int ranges_to_clear) {
    constexpr int kLog2Ps = (PS == 16) ? 4 : 5;
    __shared__ PlanSmem ps;
    extern __shared__ int E[];                               // E[B + 1] tile offsets, then Lc[B] lengths
    const Plan pl = plan_build(p.context_lens, p.plan, &ps, E, E + p.plan.B + 1, [](int) {});
    const int *Lc = E + p.plan.B + 1;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        const unsigned long long T = ps.total_tokens;
        p.ws.plan_words[0] = pl.S * kTile; p.ws.plan_words[1] = pl.nranges;
        p.ws.plan_words[2] = (int)(T & 0xffffffffULL); p.ws.plan_words[3] = (int)(T >> 32);
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int nall = max(pl.nranges, ranges_to_clear);
    for (int range = blockIdx.x; range < nall; range += gridDim.x) {
        int nk = 0, start = 0, first_b = 0;
        if (range < pl.nranges) {                            // uniform
            start = range * pl.S;
            const int len = min(pl.C, start + pl.S) - start;
            nk = len > wave ? (len - wave + kWaves - 1) / kWaves : 0;
            first_b = plan_first_request(p.plan, &ps, E, start);
        }
        int4 *dst = p.ws.meta + ((size_t)range * kWaves + wave) * p.slots_cap;
        for (int slot = lane; slot < p.slots_cap; slot += 64) {
            int4 m = make_int4(-1, 0, 0, 0);
            if (slot < nk) {
                const int pos = start + wave + kWaves * slot;
                int lo = first_b, hi = p.plan.B;             // E[lo] <= pos < E[hi]
                while (hi - lo > 1) {
                    const int mid = (lo + hi) >> 1;
                    if (E[mid] <= pos) lo = mid; else hi = mid;
                }
                const int t = pos - E[lo];
                const int last_page = (Lc[lo] - 1) >> kLog2Ps;
                const int32_t *bt = p.block_table + (size_t)lo * p.MB;
                const int page = (t * kTile) >> kLog2Ps;
                m.x = lo; m.y = t;
                m.z = bt[page];
                m.w = (PS == 16) ? bt[min(page + 1, last_page)] : m.z;   // never read beyond the request's pages
            }
            dst[slot] = m;
        }
    }
}

}  // namespace omni
