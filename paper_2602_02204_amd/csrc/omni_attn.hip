// C ABI of the decode-attention library: argument validation, host-side plan state, kernel dispatch.
// See include/omni_attn.h for the contract of every entry point.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <cstdint>
#include <cstring>
#include <new>
#include <vector>

#include "omni_attn.h"
#include "aux_kernels.hpp"
#include "decode_mfma.hpp"
#include "decode_valu.hpp"
#include "prefill_mfma.hpp"
#include "prefill_valu.hpp"

using namespace omni;

namespace {

constexpr int kDefaultTargetWorkgroups = 512;     // two 4-wave workgroups per compute unit
constexpr int kDefaultMinPartition = 128;
constexpr int kMaxBatch = 4096;                      // the plan keeps 2 * batch + 1 words in shared memory
// Dynamic shared memory any layout of the matrix-core kernel may ask for: normally half a compute unit's 160 KB, and up
// to a whole one (less the static staging area and the kernel's own variables) for the largest batches with 16 columns.
constexpr int kMaxDynamicLds = 160 * 1024 - kWaves * kKStageBytes - 1024;

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

int ilog2(int x) { int l = 0; while ((1 << l) < x) ++l; return l; }

bool misaligned(const void *p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }

int elem_bytes(int dtype) { return dtype == OMNI_F32 ? 4 : (dtype == OMNI_BF16 ? 2 : 1); }

}  // namespace

struct omni_handle_s {
    omni_attn_desc_t d;
    int tune_kernel = 0;
    int tune_target_wgs = kDefaultTargetWorkgroups;
    int tune_min_partition = kDefaultMinPartition;
    int tune_force_partition = 0;
    int tune_prefill_splits = 0;
    int tune_prefill_min_split = kPrefillMinSplitTokens;
    int tune_query_tokens = 1;
    int tune_prefill_sort = 1;
    // derived
    int kernel = 1;              // 1 = vector ALU, 2 = MFMA
    int G = 1;
    int pass_tokens = 1;         // query tokens per request one launch of the attention kernel covers
    int max_ctx = 0;
    int nw = 1;                  // workgroups per KV head
    int r_cap = 0;               // bound on partial-result slots (range index + request index)
    size_t off_ml = 0, off_o = 0, off_e = 0, ws_bytes = 0;
    MfmaLds lds{};               // shared-memory layout of the matrix-core kernel
    bool k_staged = true;        // K tiles through shared memory (matrix-core kernel)
    bool lds_attr_set = false;   // the kernel has been told how much dynamic shared memory it may get
    void *ws = nullptr;
    size_t ws_given = 0;
    const int32_t *q_lens = nullptr;     // several query tokens per request: how many each request brings (null: all)
    // profiling aid: event pairs around the partition kernel
    std::vector<hipEvent_t> prof_events;
    int prof_used = 0, prof_stride = 1, prof_calls = 0;

    // Context split of the multi-token-query kernel for chunks of up to max_q_len tokens: where the query blocks fill
    // at most half of the compute units, as many workgroups per (query block, KV head, request) as it takes to fill
    // them, at most 16 and no more than the longest context the handle allows can use.  1 = no split.
    int prefill_splits(int max_q_len) const {
        const bool mfma = (d.kv_dtype == OMNI_BF16 && d.head_dim == 128 && tune_kernel != 1) || d.kv_dtype == OMNI_FP8_E4M3;
        if (!mfma || tune_prefill_splits == 1) return 1;
        const int qb = prefill_tokens_per_block(G);
        const long long wgs = (long long)((max_q_len + qb - 1) / qb) * d.num_kv_heads * d.batch;
        const int by_ctx = (max_ctx + 2 * kTile - 1) / (2 * kTile) / (tune_prefill_min_split / (2 * kTile));
        int ns = tune_prefill_splits > 1 ? tune_prefill_splits : (wgs > 128 ? 1 : (int)(256 / wgs));
        if (ns > 16) ns = 16;
        if (ns > by_ctx) ns = by_ctx;            // no context the handle allows would use more
        return ns < 1 ? 1 : ns;
    }
    static size_t prefill_ml_bytes(const omni_attn_desc_t &d, int max_q_len, int ns) {
        return align256((size_t)d.batch * max_q_len * d.num_q_heads * ns * sizeof(float2));
    }
    size_t prefill_ws_bytes(int max_q_len) const {
        const int ns = prefill_splits(max_q_len);
        if (ns <= 1) return 0;
        return prefill_ml_bytes(d, max_q_len, ns) + align256((size_t)d.batch * max_q_len * d.num_q_heads * ns * d.head_dim * sizeof(float));
    }

    void derive() {
        G = d.num_q_heads / d.num_kv_heads;
        const long long cap_ctx = (long long)d.max_blocks_per_seq * d.page_size;
        max_ctx = (d.max_context_hint > 0 && d.max_context_hint < cap_ctx) ? d.max_context_hint : (int)(cap_ctx > 0x3fffffe0 ? 0x3fffffe0 : cap_ctx);
        const bool fp8 = d.kv_dtype == OMNI_FP8_E4M3;
        const bool mfma_ok = (d.kv_dtype == OMNI_BF16 || fp8) && d.head_dim == 128;
        kernel = fp8 ? 2 : ((tune_kernel == 2 && mfma_ok) ? 2 : (tune_kernel == 1 ? 1 : (mfma_ok ? 2 : 1)));
        nw = tune_target_wgs / d.num_kv_heads;
        if (nw < 1) nw = 1;
        // query tokens one launch takes: as many as fit the 16 columns of a KV head's tiles; more go in several passes
        pass_tokens = tune_query_tokens;
        if (pass_tokens * G > kMaxGroup) pass_tokens = kMaxGroup / G;
        const int Gq = G * pass_tokens;          // columns of a KV head: (query token, head) pairs
        const bool mt = tune_query_tokens > 1;
        // K goes through the staging area wherever the states' area beside it still holds five states (two requests
        // per chunk) with two workgroups per compute unit
        const MfmaLds plain = mfma_lds_layout(d.batch, Gq, fp8, false, mt), staged = mfma_lds_layout(d.batch, Gq, fp8, true, mt);
        k_staged = staged.two_per_cu && staged.ring_states >= kWaves + 1;
        lds = k_staged ? staged : plain;
        lds_attr_set = false;
        long long ranges = nw;
        if (tune_force_partition > 0) {
            const long long tiles = (long long)d.batch * ((max_ctx + kTile - 1) / kTile);
            const long long s = tune_force_partition / kTile;
            ranges = (tiles + s - 1) / s;
        }
        long long cap = ranges + d.batch;
        if (cap > 0x3fffffff) cap = 0x3fffffff;
        r_cap = (int)cap;
        const size_t rows = (size_t)r_cap * d.num_q_heads * pass_tokens;             // partial-result rows
        off_ml = 256;
        off_o = align256(off_ml + rows * sizeof(float2));
        off_e = align256(off_o + rows * d.head_dim * sizeof(float));
        ws_bytes = align256(off_e + (size_t)d.batch * sizeof(int2));              // the merge kernel's records
    }
};

extern "C" {

const char *omni_status_string(omni_status_t s) {
    switch (s) {
        case OMNI_OK: return "ok";
        case OMNI_ERR_NULL: return "null pointer";
        case OMNI_ERR_SHAPE: return "bad shape";
        case OMNI_ERR_DTYPE: return "bad dtype";
        case OMNI_ERR_UNSUPPORTED: return "unsupported configuration";
        case OMNI_ERR_WORKSPACE: return "workspace missing or too small";
        case OMNI_ERR_HIP: return "HIP error";
        case OMNI_ERR_NOMEM: return "out of host memory";
    }
    return "unknown status";
}

omni_status_t omni_create(const omni_attn_desc_t *desc, omni_handle_t *out_handle) {
    if (out_handle) *out_handle = nullptr;
    if (!desc || !out_handle) return OMNI_ERR_NULL;
    if (desc->struct_size != sizeof(omni_attn_desc_t)) return OMNI_ERR_SHAPE;
    if (desc->batch <= 0 || desc->num_q_heads <= 0 || desc->num_kv_heads <= 0 || desc->num_pages <= 0 ||
        desc->max_blocks_per_seq <= 0 || desc->head_dim <= 0 || desc->page_size <= 0)
        return OMNI_ERR_SHAPE;
    if (desc->num_q_heads % desc->num_kv_heads != 0) return OMNI_ERR_SHAPE;
    auto known = [](int t) { return t == OMNI_F32 || t == OMNI_BF16; };
    const bool fp8 = desc->kv_dtype == OMNI_FP8_E4M3;
    if (!known(desc->q_dtype) || !(known(desc->kv_dtype) || fp8) || !known(desc->out_dtype)) return OMNI_ERR_DTYPE;
    if (fp8 ? desc->q_dtype != OMNI_BF16 : desc->q_dtype != desc->kv_dtype) return OMNI_ERR_DTYPE;
    if (desc->out_dtype == OMNI_BF16 && desc->q_dtype != OMNI_BF16) return OMNI_ERR_DTYPE;
    if (fp8 && desc->head_dim != 128) return OMNI_ERR_UNSUPPORTED;
    if (desc->head_dim != 64 && desc->head_dim != 128) return OMNI_ERR_UNSUPPORTED;
    if (desc->page_size != 16 && desc->page_size != 32) return OMNI_ERR_UNSUPPORTED;
    if (desc->num_q_heads / desc->num_kv_heads > kMaxGroup) return OMNI_ERR_UNSUPPORTED;
    if (desc->batch > kMaxBatch) return OMNI_ERR_UNSUPPORTED;
    omni_handle_s *h = new (std::nothrow) omni_handle_s();
    if (!h) return OMNI_ERR_NOMEM;
    h->d = *desc;
    h->derive();
    *out_handle = h;
    return OMNI_OK;
}

void omni_destroy(omni_handle_t h) {
    if (!h) return;
    for (hipEvent_t e : h->prof_events) (void)hipEventDestroy(e);
    delete h;
}

omni_status_t omni_set_tuning(omni_handle_t h, int32_t key, int32_t value) {
    if (!h) return OMNI_ERR_NULL;
    switch (key) {
        case OMNI_TUNE_KERNEL:
            if (value < 0 || value > 2) return OMNI_ERR_SHAPE;
            if (value == 2 && !(h->d.kv_dtype == OMNI_BF16 && h->d.head_dim == 128) && h->d.kv_dtype != OMNI_FP8_E4M3)
                return OMNI_ERR_UNSUPPORTED;
            if (value == 1 && (h->d.kv_dtype == OMNI_FP8_E4M3 || h->tune_query_tokens > 1)) return OMNI_ERR_UNSUPPORTED;
            h->tune_kernel = value; break;
        case OMNI_TUNE_TARGET_WORKGROUPS:
            if (value <= 0) return OMNI_ERR_SHAPE;
            h->tune_target_wgs = value; break;
        case OMNI_TUNE_MIN_PARTITION:
            if (value < kTile || value % kTile) return OMNI_ERR_SHAPE;
            h->tune_min_partition = value; break;
        case OMNI_TUNE_FORCE_PARTITION:
            if (value < 0 || value % kTile) return OMNI_ERR_SHAPE;
            h->tune_force_partition = value; break;
        case OMNI_TUNE_PREFILL_SPLITS:
            if (value < 0 || value > 16) return OMNI_ERR_SHAPE;
            h->tune_prefill_splits = value; break;
        case OMNI_TUNE_PREFILL_SORT:
            if (value < 0 || value > 1) return OMNI_ERR_SHAPE;
            h->tune_prefill_sort = value; break;
        case OMNI_TUNE_QUERY_TOKENS:
            if (value < 1) return OMNI_ERR_SHAPE;
            if (value > 1 && h->kernel != 2) return OMNI_ERR_UNSUPPORTED;
            h->tune_query_tokens = value; break;
        case OMNI_TUNE_PREFILL_MIN_SPLIT:
            if (value < 2 * kTile || value % (2 * kTile)) return OMNI_ERR_SHAPE;
            h->tune_prefill_min_split = value; break;
        default: return OMNI_ERR_SHAPE;
    }
    h->derive();
    h->ws = nullptr;             // layout may have changed: the caller registers the workspace again
    h->ws_given = 0;
    return OMNI_OK;
}

omni_status_t omni_workspace_bytes(omni_handle_t h, size_t *bytes) {
    if (!h || !bytes) return OMNI_ERR_NULL;
    *bytes = h->ws_bytes;
    return OMNI_OK;
}

omni_status_t omni_prefill_workspace_bytes(omni_handle_t h, int32_t max_q_len, size_t *bytes) {
    if (!h || !bytes) return OMNI_ERR_NULL;
    if (max_q_len <= 0) return OMNI_ERR_SHAPE;
    *bytes = h->prefill_ws_bytes(max_q_len);
    return OMNI_OK;
}

omni_status_t omni_set_workspace(omni_handle_t h, void *dev_ptr, size_t bytes) {
    if (!h || !dev_ptr) return OMNI_ERR_NULL;
    if (((uintptr_t)dev_ptr & 255) != 0 || bytes < h->ws_bytes) return OMNI_ERR_WORKSPACE;
    h->ws = dev_ptr;
    h->ws_given = bytes;
    return OMNI_OK;
}

omni_status_t omni_set_query_lens(omni_handle_t h, const int32_t *dev_q_lens) {
    if (!h) return OMNI_ERR_NULL;
    if (misaligned(dev_q_lens, 4)) return OMNI_ERR_SHAPE;
    h->q_lens = dev_q_lens;
    return OMNI_OK;
}

omni_status_t omni_get_plan(omni_handle_t h, int32_t *kernel, int32_t *partition_grid, int32_t *merge_grid,
                            int32_t *max_request_parts, int32_t *threads_per_workgroup) {
    if (!h) return OMNI_ERR_NULL;
    if (kernel) *kernel = h->kernel;
    if (partition_grid) *partition_grid = h->nw * h->d.num_kv_heads;
    if (merge_grid) *merge_grid = h->d.batch * h->d.num_kv_heads;
    if (max_request_parts) *max_request_parts = h->r_cap;
    if (threads_per_workgroup) *threads_per_workgroup = kThreads;
    return OMNI_OK;
}

}  // extern "C"

namespace {

template <typename T, int D>
void launch_valu(const AttnParams &p, dim3 grid, size_t dyn, hipStream_t s) {
    if (p.G <= 1) decode_valu_kernel<T, D, 1><<<grid, kThreads, dyn, s>>>(p);
    else if (p.G <= 2) decode_valu_kernel<T, D, 2><<<grid, kThreads, dyn, s>>>(p);
    else if (p.G <= 4) decode_valu_kernel<T, D, 4><<<grid, kThreads, dyn, s>>>(p);
    else if (p.G <= 8) decode_valu_kernel<T, D, 8><<<grid, kThreads, dyn, s>>>(p);
    else decode_valu_kernel<T, D, 16><<<grid, kThreads, dyn, s>>>(p);
}

}  // namespace

extern "C" {

static omni_status_t launch_append(omni_handle_t h, const void *k_new, const void *v_new, void *k_cache, void *v_cache,
                                   const int32_t *block_table, const int32_t *positions, int positions_are_lengths,
                                   void *stream);

// The variant of the matrix-core kernel a handle launches: page size, cache width, K staging, query tokens per request.
static const void *mfma_variant(const omni_handle_s *h) {
    const bool ps16 = h->d.page_size == 16, st = h->k_staged, fp8 = h->d.kv_dtype == OMNI_FP8_E4M3;
    if (h->tune_query_tokens > 1) {
        if (fp8) return ps16 ? (st ? (const void *)&decode_mfma_kernel<16, true, true, true> : (const void *)&decode_mfma_kernel<16, true, false, true>)
                             : (st ? (const void *)&decode_mfma_kernel<32, true, true, true> : (const void *)&decode_mfma_kernel<32, true, false, true>);
        return ps16 ? (st ? (const void *)&decode_mfma_kernel<16, false, true, true> : (const void *)&decode_mfma_kernel<16, false, false, true>)
                    : (st ? (const void *)&decode_mfma_kernel<32, false, true, true> : (const void *)&decode_mfma_kernel<32, false, false, true>);
    }
    if (fp8) return ps16 ? (st ? (const void *)&decode_mfma_kernel<16, true, true> : (const void *)&decode_mfma_kernel<16, true, false>)
                         : (st ? (const void *)&decode_mfma_kernel<32, true, true> : (const void *)&decode_mfma_kernel<32, true, false>);
    return ps16 ? (st ? (const void *)&decode_mfma_kernel<16, false, true> : (const void *)&decode_mfma_kernel<16, false, false>)
                : (st ? (const void *)&decode_mfma_kernel<32, false, true> : (const void *)&decode_mfma_kernel<32, false, false>);
}

// The attention launch shared by omni_paged_decode_attn (k_new = v_new = null) and omni_decode_step.
// `ws_base` = null: the workspace the caller registered with the handle; else a buffer of at least h->ws_bytes.
static omni_status_t launch_attention(omni_handle_t h, const void *q, const void *k_new, const void *v_new,
                                      const void *k_cache, const void *v_cache, const int32_t *block_table,
                                      const int32_t *context_lens, float scale, void *out, void *stream,
                                      const float *k_scale = nullptr, const float *v_scale = nullptr,
                                      void *ws_base = nullptr) {
    if (!h || !q || !k_cache || !v_cache || !block_table || !context_lens || !out) return OMNI_ERR_NULL;
    const bool fp8 = h->d.kv_dtype == OMNI_FP8_E4M3;
    if (fp8 != (k_scale != nullptr)) return OMNI_ERR_UNSUPPORTED;
    if (fp8 && (!v_scale || misaligned(k_scale, 4) || misaligned(v_scale, 4))) return v_scale ? OMNI_ERR_SHAPE : OMNI_ERR_NULL;
    if (!ws_base && (!h->ws || h->ws_given < h->ws_bytes)) return OMNI_ERR_WORKSPACE;
    if (misaligned(q, 16) || misaligned(k_cache, 16) || misaligned(v_cache, 16) || misaligned(out, 16) ||
        misaligned(k_new, 16) || misaligned(v_new, 16) || misaligned(block_table, 4) || misaligned(context_lens, 4))
        return OMNI_ERR_SHAPE;
    const omni_attn_desc_t &d = h->d;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);

    AttnParams p;
    p.q = q; p.k_cache = k_cache; p.v_cache = v_cache;
    p.k_new = k_new; p.v_new = v_new;
    p.k_scale = k_scale; p.v_scale = v_scale;
    p.block_table = block_table; p.context_lens = context_lens; p.out = out;
    p.q_lens = h->tune_query_tokens > 1 ? h->q_lens : nullptr;
    char *ws = reinterpret_cast<char *>(ws_base ? ws_base : h->ws);
    p.ws.plan_words = reinterpret_cast<int32_t *>(ws);
    p.ws.part_ml = reinterpret_cast<float2 *>(ws + h->off_ml);
    p.ws.part_o = reinterpret_cast<float *>(ws + h->off_o);
    p.ws.merge_rec = reinterpret_cast<int2 *>(ws + h->off_e);
    p.plan.B = d.batch;
    p.plan.nw = h->nw;
    p.plan.s_min = h->tune_min_partition / kTile;
    p.plan.s_force = h->tune_force_partition / kTile;
    p.scale_log2 = scale * kLog2e;
    p.Hq = d.num_q_heads; p.Hkv = d.num_kv_heads; p.G = h->G; p.MB = d.max_blocks_per_seq;
    p.Tq = h->tune_query_tokens;
    p.log2_ps = ilog2(d.page_size);
    p.out_bf16 = d.out_dtype == OMNI_BF16;
    p.lds = h->lds;

    // Several query tokens per request: one pass (attention + merge) per pass_tokens of them; the new rows of a fused
    // step are all written by the first pass.
    for (int t_off = 0; t_off < p.Tq; t_off += h->pass_tokens) {
        p.t_off = t_off;
        p.T = p.Tq - t_off < h->pass_tokens ? p.Tq - t_off : h->pass_tokens;
        p.Gq = p.T * h->G;
        if (t_off > 0) { p.k_new = nullptr; p.v_new = nullptr; }
        const dim3 grid((unsigned)(h->nw * d.num_kv_heads));
        const size_t dyn = (size_t)(2 * d.batch + 1) * sizeof(int);     // tile offsets and lengths of the plan
        (void)hipGetLastError();
        const bool prof = (size_t)(2 * h->prof_used + 1) < h->prof_events.size() && (h->prof_calls++ % h->prof_stride) == 0;
        // Profiled launches of the matrix-core kernel carry their event pair in the dispatch itself (the events then hold
        // the kernel's own start and stop times); around the other kernels the pair is recorded on the stream.
        const bool prof_in_dispatch = prof && h->kernel == 2;
        if (prof && !prof_in_dispatch && hipEventRecord(h->prof_events[2 * h->prof_used], s) != hipSuccess) return OMNI_ERR_HIP;
        if (h->kernel == 2) {
            const void *fn = mfma_variant(h);
            if (!h->lds_attr_set) {          // more than the default 64 KB of dynamic shared memory: the setting belongs to
                                             // the kernel, not to the handle, so every handle asks for the same bound (what
                                             // any layout may use) and none lowers what another one needs
                if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxDynamicLds) != hipSuccess) {
                    (void)hipGetLastError();
                    return OMNI_ERR_HIP;
                }
                h->lds_attr_set = true;
            }
            void *args[] = {&p};
            const hipError_t le = prof_in_dispatch
                ? hipExtLaunchKernel(fn, grid, dim3(kThreads), args, (size_t)h->lds.total, s, h->prof_events[2 * h->prof_used],
                                     h->prof_events[2 * h->prof_used + 1], 0)
                : hipLaunchKernel(fn, grid, dim3(kThreads), args, (size_t)h->lds.total, s);
            if (le != hipSuccess) {
                (void)hipGetLastError();
                return OMNI_ERR_HIP;
            }
        } else if (d.kv_dtype == OMNI_BF16) {
            if (d.head_dim == 128) launch_valu<uint16_t, 128>(p, grid, dyn, s);
            else launch_valu<uint16_t, 64>(p, grid, dyn, s);
        } else {
            if (d.head_dim == 128) launch_valu<float, 128>(p, grid, dyn, s);
            else launch_valu<float, 64>(p, grid, dyn, s);
        }
        if (hipGetLastError() != hipSuccess) return OMNI_ERR_HIP;
        if (prof) {
            if (!prof_in_dispatch && hipEventRecord(h->prof_events[2 * h->prof_used + 1], s) != hipSuccess) return OMNI_ERR_HIP;
            ++h->prof_used;
        }

        // Whether any request was cut by a range boundary is known only on the device: the merge kernel always runs, and
        // its workgroups return at once for requests that the attention kernel finished.
        const dim3 mgrid((unsigned)(d.batch * d.num_kv_heads));
        if (d.head_dim == 128) merge_kernel<128><<<mgrid, kThreads, 0, s>>>(p);
        else merge_kernel<64><<<mgrid, kThreads, 0, s>>>(p);
        if (hipGetLastError() != hipSuccess) return OMNI_ERR_HIP;
    }

    return OMNI_OK;
}

omni_status_t omni_paged_decode_attn(omni_handle_t h, const void *q, const void *k_cache, const void *v_cache,
                                     const int32_t *block_table, const int32_t *context_lens, float scale, void *out,
                                     void *stream) {
    return launch_attention(h, q, nullptr, nullptr, k_cache, v_cache, block_table, context_lens, scale, out, stream);
}

// ---- omni_paged_decode_attn without a workspace from the caller: the partial rows and plan words go to a static device
// array.  `scratch` is a host-side stand-in for the array, not a device address: host code uses only the address that
// hipGetSymbolAddress returns for the current device (every device holds its own copy of the array).
constexpr size_t kScratchBytes = (size_t)8 << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
constexpr int kMaxDevices = 64;
static void *g_scratch_ptr[kMaxDevices] = {};

omni_status_t omni_paged_decode_attn_static(omni_handle_t h, const void *q, const void *k_cache, const void *v_cache,
                                            const int32_t *block_table, const int32_t *context_lens, float scale,
                                            void *out, void *stream) {
    if (!h) return OMNI_ERR_NULL;
    if (h->d.kv_dtype == OMNI_FP8_E4M3) return OMNI_ERR_UNSUPPORTED;
    if (h->ws_bytes > kScratchBytes) return OMNI_ERR_WORKSPACE;      // larger problems need omni_set_workspace
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        (void)hipGetLastError();
        return OMNI_ERR_HIP;
    }
    if (!g_scratch_ptr[dev]) {                                       // first call on this device: look the array up
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
            (void)hipGetLastError();
            return OMNI_ERR_HIP;
        }
        g_scratch_ptr[dev] = ptr;
    }
    return launch_attention(h, q, nullptr, nullptr, k_cache, v_cache, block_table, context_lens, scale, out, stream,
                            nullptr, nullptr, g_scratch_ptr[dev]);
}

omni_status_t omni_paged_decode_attn_fp8(omni_handle_t h, const void *q, const void *k_cache, const void *v_cache,
                                         const float *k_scale, const float *v_scale, const int32_t *block_table,
                                         const int32_t *context_lens, float scale, void *out, void *stream) {
    if (!h || !k_scale || !v_scale) return OMNI_ERR_NULL;
    if (h->d.kv_dtype != OMNI_FP8_E4M3) return OMNI_ERR_UNSUPPORTED;
    return launch_attention(h, q, nullptr, nullptr, k_cache, v_cache, block_table, context_lens, scale, out, stream,
                            k_scale, v_scale);
}

omni_status_t omni_decode_step_fp8(omni_handle_t h, const void *q, const void *k_new, const void *v_new, void *k_cache,
                                   void *v_cache, const float *k_scale, const float *v_scale, const int32_t *block_table,
                                   const int32_t *context_lens, float scale, void *out, void *stream) {
    if (!h || !k_new || !v_new || !k_scale || !v_scale) return OMNI_ERR_NULL;
    if (h->d.kv_dtype != OMNI_FP8_E4M3) return OMNI_ERR_UNSUPPORTED;
    return launch_attention(h, q, k_new, v_new, k_cache, v_cache, block_table, context_lens, scale, out, stream, k_scale,
                            v_scale);
}

omni_status_t omni_decode_step(omni_handle_t h, const void *q, const void *k_new, const void *v_new, void *k_cache,
                               void *v_cache, const int32_t *block_table, const int32_t *context_lens, float scale,
                               void *out, void *stream) {
    if (!h || !k_new || !v_new) return OMNI_ERR_NULL;
    if (h->kernel == 2)          // the MFMA kernel writes the new rows itself, just before it reads their tiles
        return launch_attention(h, q, k_new, v_new, k_cache, v_cache, block_table, context_lens, scale, out, stream);
    if (!q || !k_cache || !v_cache || !block_table || !context_lens || !out) return OMNI_ERR_NULL;
    if (!h->ws || h->ws_given < h->ws_bytes) return OMNI_ERR_WORKSPACE;
    const omni_status_t st = launch_append(h, k_new, v_new, k_cache, v_cache, block_table, context_lens, 1, stream);
    if (st != OMNI_OK) return st;
    return launch_attention(h, q, nullptr, nullptr, k_cache, v_cache, block_table, context_lens, scale, out, stream);
}

omni_status_t omni_kv_append(omni_handle_t h, const void *k_new, const void *v_new, void *k_cache, void *v_cache,
                             const int32_t *block_table, const int32_t *positions, void *stream) {
    return launch_append(h, k_new, v_new, k_cache, v_cache, block_table, positions, 0, stream);
}

static omni_status_t launch_append(omni_handle_t h, const void *k_new, const void *v_new, void *k_cache, void *v_cache,
                                   const int32_t *block_table, const int32_t *positions, int positions_are_lengths,
                                   void *stream) {
    if (!h || !k_new || !v_new || !k_cache || !v_cache || !block_table || !positions) return OMNI_ERR_NULL;
    if (misaligned(k_new, 16) || misaligned(v_new, 16) || misaligned(k_cache, 16) || misaligned(v_cache, 16) ||
        misaligned(block_table, 4) || misaligned(positions, 4))
        return OMNI_ERR_SHAPE;
    const omni_attn_desc_t &d = h->d;
    AppendParams p;
    p.k_new = k_new; p.v_new = v_new; p.k_cache = k_cache; p.v_cache = v_cache;
    p.block_table = block_table; p.positions = positions;
    p.B = d.batch; p.Hkv = d.num_kv_heads; p.MB = d.max_blocks_per_seq; p.log2_ps = ilog2(d.page_size);
    p.row_vecs = d.head_dim * elem_bytes(d.kv_dtype) / 16;
    p.positions_are_lengths = positions_are_lengths;
    const long long total = (long long)p.B * p.Hkv * p.row_vecs;
    const dim3 grid((unsigned)((total + kThreads - 1) / kThreads));
    (void)hipGetLastError();
    kv_append_kernel<<<grid, kThreads, 0, reinterpret_cast<hipStream_t>(stream)>>>(p);
    if (hipGetLastError() != hipSuccess) return OMNI_ERR_HIP;
    return OMNI_OK;
}

omni_status_t omni_kv_append_quant_fp8(omni_handle_t h, const void *k_new, const void *v_new, void *k_cache, void *v_cache,
                                       float *k_scale, float *v_scale, const int32_t *block_table,
                                       const int32_t *positions, float headroom, void *stream) {
    if (!h || !k_new || !v_new || !k_cache || !v_cache || !k_scale || !v_scale || !block_table || !positions)
        return OMNI_ERR_NULL;
    if (h->d.kv_dtype != OMNI_FP8_E4M3) return OMNI_ERR_UNSUPPORTED;
    if (!(headroom >= 1.0f) || !(headroom <= 65536.0f)) return OMNI_ERR_SHAPE;
    if (misaligned(k_new, 16) || misaligned(v_new, 16) || misaligned(k_cache, 16) || misaligned(v_cache, 16) ||
        misaligned(k_scale, 4) || misaligned(v_scale, 4) || misaligned(block_table, 4) || misaligned(positions, 4))
        return OMNI_ERR_SHAPE;
    const omni_attn_desc_t &d = h->d;
    AppendQuantParams p;
    p.k_new = k_new; p.v_new = v_new; p.k_cache = k_cache; p.v_cache = v_cache;
    p.k_scale = k_scale; p.v_scale = v_scale;
    p.block_table = block_table; p.positions = positions;
    p.headroom = headroom;
    p.B = d.batch; p.Hkv = d.num_kv_heads; p.MB = d.max_blocks_per_seq; p.log2_ps = ilog2(d.page_size);
    const long long threads = 2LL * p.B * p.Hkv * 16;                      // 16 lanes per K row and per V row
    const dim3 grid((unsigned)((threads + kThreads - 1) / kThreads));
    (void)hipGetLastError();
    kv_append_quant_kernel<<<grid, kThreads, 0, reinterpret_cast<hipStream_t>(stream)>>>(p);
    if (hipGetLastError() != hipSuccess) return OMNI_ERR_HIP;
    return OMNI_OK;
}

omni_status_t omni_debug_last_plan(omni_handle_t h, int32_t host_out[4], void *stream) {
    if (!h || !host_out) return OMNI_ERR_NULL;
    if (!h->ws) return OMNI_ERR_WORKSPACE;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    if (hipStreamSynchronize(s) != hipSuccess) return OMNI_ERR_HIP;
    int32_t words[4];
    if (hipMemcpy(words, h->ws, sizeof(words), hipMemcpyDeviceToHost) != hipSuccess) return OMNI_ERR_HIP;
    host_out[0] = words[0]; host_out[1] = words[1]; host_out[2] = words[2]; host_out[3] = 0;
    return OMNI_OK;
}

omni_status_t omni_debug_lds_layout(omni_handle_t h, int32_t host_out[6]) {
    if (!h || !host_out) return OMNI_ERR_NULL;
    if (h->kernel != 2) return OMNI_ERR_UNSUPPORTED;
    host_out[0] = h->lds.total; host_out[1] = h->lds.static_bytes; host_out[2] = h->lds.ring_states;
    host_out[3] = h->k_staged ? 1 : 0; host_out[4] = h->lds.two_per_cu ? 1 : 0; host_out[5] = kMaxDynamicLds;
    return OMNI_OK;
}

omni_status_t omni_debug_kernel_resources(omni_handle_t h, int32_t which, int32_t host_out[6]) {
    if (!h || !host_out) return OMNI_ERR_NULL;
    const void *fn = nullptr;
    int dyn = 0;
    if (which == 0) {
        if (h->kernel != 2) return OMNI_ERR_UNSUPPORTED;
        fn = mfma_variant(h);
        dyn = h->lds.total;
    } else if (which == 1) {
        fn = h->d.head_dim == 128 ? (const void *)&merge_kernel<128> : (const void *)&merge_kernel<64>;
        dyn = 0;
    } else {
        return OMNI_ERR_SHAPE;
    }
    hipFuncAttributes a;
    if (hipFuncGetAttributes(&a, fn) != hipSuccess) {
        (void)hipGetLastError();
        return OMNI_ERR_HIP;
    }
    host_out[0] = a.numRegs; host_out[1] = (int32_t)a.sharedSizeBytes; host_out[2] = dyn;
    host_out[3] = a.maxThreadsPerBlock; host_out[4] = (int32_t)a.localSizeBytes; host_out[5] = kThreads;
    return OMNI_OK;
}

omni_status_t omni_debug_profile_begin(omni_handle_t h, int32_t capacity, int32_t stride) {
    if (!h) return OMNI_ERR_NULL;
    if (capacity <= 0 || stride <= 0) return OMNI_ERR_SHAPE;
    h->prof_stride = stride;
    h->prof_calls = 0;
    for (hipEvent_t e : h->prof_events) (void)hipEventDestroy(e);
    h->prof_events.clear();
    h->prof_used = 0;
    for (int i = 0; i < 2 * capacity; ++i) {
        hipEvent_t e;
        if (hipEventCreate(&e) != hipSuccess) return OMNI_ERR_HIP;
        h->prof_events.push_back(e);
    }
    return OMNI_OK;
}

omni_status_t omni_debug_profile_end(omni_handle_t h, float *host_ms, int32_t *count) {
    if (!h || !host_ms || !count) return OMNI_ERR_NULL;
    omni_status_t st = OMNI_OK;
    *count = 0;
    for (int i = 0; i < h->prof_used; ++i) {
        float ms = 0.f;
        if (hipEventSynchronize(h->prof_events[2 * i + 1]) != hipSuccess ||
            hipEventElapsedTime(&ms, h->prof_events[2 * i], h->prof_events[2 * i + 1]) != hipSuccess) {
            st = OMNI_ERR_HIP;
            break;
        }
        host_ms[(*count)++] = ms;
    }
    for (hipEvent_t e : h->prof_events) (void)hipEventDestroy(e);
    h->prof_events.clear();
    h->prof_used = 0;
    return st;
}

omni_status_t omni_debug_gather(omni_handle_t h, const void *cache, const int32_t *block_table,
                                const int32_t *context_lens, int32_t request, void *dense_out, void *stream) {
    if (!h || !cache || !block_table || !context_lens || !dense_out) return OMNI_ERR_NULL;
    const omni_attn_desc_t &d = h->d;
    if (request < 0 || request >= d.batch) return OMNI_ERR_SHAPE;
    GatherParams p;
    p.cache = cache; p.block_table = block_table; p.context_lens = context_lens; p.dense_out = dense_out;
    p.request = request; p.Hkv = d.num_kv_heads; p.MB = d.max_blocks_per_seq; p.log2_ps = ilog2(d.page_size);
    p.row_vecs = d.head_dim * elem_bytes(d.kv_dtype) / 16;
    const long long total = (long long)h->max_ctx * p.Hkv * p.row_vecs;
    const dim3 grid((unsigned)((total + kThreads - 1) / kThreads));
    (void)hipGetLastError();
    gather_kernel<<<grid, kThreads, 0, reinterpret_cast<hipStream_t>(stream)>>>(p);
    if (hipGetLastError() != hipSuccess) return OMNI_ERR_HIP;
    return OMNI_OK;
}

omni_status_t omni_debug_stream_read(const void *a, size_t a_bytes, const void *b, size_t b_bytes, void *sink,
                                     void *stream) {
    if (!a || !sink || (b_bytes && !b)) return OMNI_ERR_NULL;
    if (((a_bytes | b_bytes) & 15) || ((uintptr_t)a & 15) || ((uintptr_t)b & 15)) return OMNI_ERR_SHAPE;
    (void)hipGetLastError();
    stream_read_kernel<<<2 * 256, kThreads, 0, reinterpret_cast<hipStream_t>(stream)>>>(
        reinterpret_cast<const uint4 *>(a), a_bytes / 16, reinterpret_cast<const uint4 *>(b), b_bytes / 16,
        reinterpret_cast<unsigned *>(sink));
    if (hipGetLastError() != hipSuccess) return OMNI_ERR_HIP;
    return OMNI_OK;
}

static omni_status_t launch_pack(omni_handle_t h, bool unpack, const void *k_src, const void *v_src, void *k_dst,
                                 void *v_dst, const int32_t *block_table, const int32_t *context_lens,
                                 const int64_t *token_offsets, void *stream, const int32_t *q_lens = nullptr,
                                 int max_tokens = 0) {
    if (!h || !k_src || !v_src || !k_dst || !v_dst || !block_table || !context_lens || !token_offsets) return OMNI_ERR_NULL;
    if (misaligned(k_src, 16) || misaligned(v_src, 16) || misaligned(k_dst, 16) || misaligned(v_dst, 16) ||
        misaligned(block_table, 4) || misaligned(context_lens, 4) || misaligned(token_offsets, 8))
        return OMNI_ERR_SHAPE;
    const omni_attn_desc_t &d = h->d;
    PackParams p;
    p.k_src = k_src; p.v_src = v_src; p.k_dst = k_dst; p.v_dst = v_dst;
    p.block_table = block_table; p.context_lens = context_lens;
    p.token_offsets = reinterpret_cast<const long long *>(token_offsets);
    p.q_lens = q_lens;
    p.max_tokens = max_tokens;
    p.Hkv = d.num_kv_heads; p.MB = d.max_blocks_per_seq; p.log2_ps = ilog2(d.page_size);
    p.row_vecs = d.head_dim * elem_bytes(d.kv_dtype) / 16;
    const int span = q_lens ? max_tokens : h->max_ctx;                     // tokens per request the grid must cover
    const dim3 grid((unsigned)((span + kPackTokens - 1) / kPackTokens), (unsigned)d.batch);
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    (void)hipGetLastError();
    if (unpack) kv_pack_kernel<true><<<grid, kThreads, 0, s>>>(p);
    else kv_pack_kernel<false><<<grid, kThreads, 0, s>>>(p);
    if (hipGetLastError() != hipSuccess) return OMNI_ERR_HIP;
    return OMNI_OK;
}

omni_status_t omni_kv_pack(omni_handle_t h, const void *k_cache, const void *v_cache, const int32_t *block_table,
                           const int32_t *context_lens, const int64_t *token_offsets, void *k_dense, void *v_dense,
                           void *stream) {
    return launch_pack(h, false, k_cache, v_cache, k_dense, v_dense, block_table, context_lens, token_offsets, stream);
}

omni_status_t omni_kv_unpack(omni_handle_t h, const void *k_dense, const void *v_dense, void *k_cache, void *v_cache,
                             const int32_t *block_table, const int32_t *context_lens, const int64_t *token_offsets,
                             void *stream) {
    return launch_pack(h, true, k_dense, v_dense, k_cache, v_cache, block_table, context_lens, token_offsets, stream);
}

omni_status_t omni_kv_append_chunk(omni_handle_t h, const void *k_new, const void *v_new, void *k_cache, void *v_cache,
                                   const int32_t *block_table, const int32_t *context_lens, const int32_t *q_lens,
                                   const int64_t *q_offsets, int32_t max_q_len, void *stream) {
    if (!q_lens) return OMNI_ERR_NULL;
    if (max_q_len <= 0) return OMNI_ERR_SHAPE;
    if (misaligned(q_lens, 4)) return OMNI_ERR_SHAPE;
    return launch_pack(h, true, k_new, v_new, k_cache, v_cache, block_table, context_lens, q_offsets, stream, q_lens,
                       max_q_len);
}

// The launch shared by omni_paged_prefill_attn (k_scale = v_scale = null) and omni_paged_prefill_attn_fp8.
static omni_status_t launch_prefill(omni_handle_t h, const void *q, const void *k_cache, const void *v_cache,
                                    const float *k_scale, const float *v_scale, const int32_t *block_table,
                                    const int32_t *context_lens, const int32_t *q_lens, const int64_t *q_offsets,
                                    int32_t max_q_len, float scale, void *out, void *stream) {
    if (!h || !q || !k_cache || !v_cache || !block_table || !context_lens || !q_lens || !q_offsets || !out)
        return OMNI_ERR_NULL;
    const omni_attn_desc_t &d = h->d;
    const bool fp8 = d.kv_dtype == OMNI_FP8_E4M3;
    if (fp8 != (k_scale != nullptr)) return OMNI_ERR_UNSUPPORTED;
    if (fp8 && (!v_scale || misaligned(k_scale, 4) || misaligned(v_scale, 4))) return v_scale ? OMNI_ERR_SHAPE : OMNI_ERR_NULL;
    const bool mfma = fp8 || (d.kv_dtype == OMNI_BF16 && d.head_dim == 128 && h->tune_kernel != 1);
    if (max_q_len <= 0 || (mfma && !(scale > 0.f))) return OMNI_ERR_SHAPE;
    if (misaligned(q, 16) || misaligned(k_cache, 16) || misaligned(v_cache, 16) || misaligned(out, 16) ||
        misaligned(block_table, 4) || misaligned(context_lens, 4) || misaligned(q_lens, 4) || misaligned(q_offsets, 8))
        return OMNI_ERR_SHAPE;
    PrefillParams p;
    p.q = q; p.k_cache = k_cache; p.v_cache = v_cache;
    p.k_scale = k_scale; p.v_scale = v_scale;
    p.block_table = block_table; p.context_lens = context_lens; p.q_lens = q_lens;
    p.q_offsets = reinterpret_cast<const long long *>(q_offsets);
    p.out = out;
    p.scale_log2 = scale * kLog2e;
    p.Hq = d.num_q_heads; p.Hkv = d.num_kv_heads; p.G = h->G; p.MB = d.max_blocks_per_seq;
    p.out_bf16 = d.out_dtype == OMNI_BF16;
    const int qb = mfma ? prefill_tokens_per_block(h->G) : kWaves;       // query tokens per workgroup
    // The context is split only if the registered workspace holds the pieces (omni_prefill_workspace_bytes).
    int ns = mfma ? h->prefill_splits(max_q_len) : 1;
    if (ns > 1 && (!h->ws || h->ws_given < h->prefill_ws_bytes(max_q_len))) ns = 1;
    // With a registered workspace and more than one round of workgroups, the requests are taken longest first: a
    // one-workgroup kernel ranks them into the first words of the workspace (the pieces of a split follow).
    const long long wgs_all = (long long)((max_q_len + qb - 1) / qb) * d.num_kv_heads * d.batch;
    const bool sorted = mfma && h->ws && d.batch > 1 && d.batch <= kPrefillOrderMax && wgs_all > 256 && h->tune_prefill_sort != 0;
    const size_t order_bytes = sorted ? align256((size_t)d.batch * sizeof(int32_t)) : 0;
    if (ns > 1 && h->ws_given < order_bytes + h->prefill_ws_bytes(max_q_len)) ns = 1;
    p.order = sorted ? reinterpret_cast<const int32_t *>(h->ws) : nullptr;
    p.B = d.batch;
    p.num_splits = ns; p.max_q_len = max_q_len;
    p.min_split_steps = h->tune_prefill_min_split / (2 * kTile);
    p.part_ml = reinterpret_cast<float2 *>(reinterpret_cast<char *>(h->ws) + order_bytes);
    p.part_o = ns > 1 ? reinterpret_cast<float *>(reinterpret_cast<char *>(h->ws) + order_bytes + omni_handle_s::prefill_ml_bytes(d, max_q_len, ns)) : nullptr;
    const dim3 grid((unsigned)((max_q_len + qb - 1) / qb) * (unsigned)ns, (unsigned)d.num_kv_heads, (unsigned)d.batch);
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    (void)hipGetLastError();
    if (sorted) {
        prefill_order_kernel<<<1, kPrefillOrderMax, 0, s>>>(context_lens, d.batch, reinterpret_cast<int32_t *>(h->ws));
        if (hipGetLastError() != hipSuccess) return OMNI_ERR_HIP;
    }
    if (mfma) {
        if (fp8) {
            if (d.page_size == 16) prefill_mfma_kernel<16, true><<<grid, kPrefillThreads, 0, s>>>(p);
            else prefill_mfma_kernel<32, true><<<grid, kPrefillThreads, 0, s>>>(p);
        } else {
            if (d.page_size == 16) prefill_mfma_kernel<16><<<grid, kPrefillThreads, 0, s>>>(p);
            else prefill_mfma_kernel<32><<<grid, kPrefillThreads, 0, s>>>(p);
        }
        if (ns > 1) {
            if (hipGetLastError() != hipSuccess) return OMNI_ERR_HIP;
            const long long items = (long long)max_q_len * d.num_q_heads * 32;
            prefill_merge_kernel<<<dim3((unsigned)((items + kThreads - 1) / kThreads), (unsigned)d.batch), kThreads, 0, s>>>(p);
        }
    } else {
        const int l2 = ilog2(d.page_size);
        if (d.kv_dtype == OMNI_BF16) {
            if (d.head_dim == 128) prefill_valu_kernel<uint16_t, 128><<<grid, kThreads, 0, s>>>(p, l2);
            else prefill_valu_kernel<uint16_t, 64><<<grid, kThreads, 0, s>>>(p, l2);
        } else {
            if (d.head_dim == 128) prefill_valu_kernel<float, 128><<<grid, kThreads, 0, s>>>(p, l2);
            else prefill_valu_kernel<float, 64><<<grid, kThreads, 0, s>>>(p, l2);
        }
    }
    if (hipGetLastError() != hipSuccess) return OMNI_ERR_HIP;
    return OMNI_OK;
}

omni_status_t omni_paged_prefill_attn(omni_handle_t h, const void *q, const void *k_cache, const void *v_cache,
                                      const int32_t *block_table, const int32_t *context_lens, const int32_t *q_lens,
                                      const int64_t *q_offsets, int32_t max_q_len, float scale, void *out, void *stream) {
    return launch_prefill(h, q, k_cache, v_cache, nullptr, nullptr, block_table, context_lens, q_lens, q_offsets, max_q_len,
                          scale, out, stream);
}

omni_status_t omni_paged_prefill_attn_fp8(omni_handle_t h, const void *q, const void *k_cache, const void *v_cache,
                                          const float *k_scale, const float *v_scale, const int32_t *block_table,
                                          const int32_t *context_lens, const int32_t *q_lens, const int64_t *q_offsets,
                                          int32_t max_q_len, float scale, void *out, void *stream) {
    if (!h || !k_scale || !v_scale) return OMNI_ERR_NULL;
    if (h->d.kv_dtype != OMNI_FP8_E4M3) return OMNI_ERR_UNSUPPORTED;
    return launch_prefill(h, q, k_cache, v_cache, k_scale, v_scale, block_table, context_lens, q_lens, q_offsets, max_q_len,
                          scale, out, stream);
}

struct omni_graph_s {
    hipGraphExec_t exec = nullptr;
};

omni_status_t omni_graph_begin(void *stream) {
    if (!stream) return OMNI_ERR_UNSUPPORTED;
    (void)hipGetLastError();
    if (hipStreamBeginCapture(reinterpret_cast<hipStream_t>(stream), hipStreamCaptureModeThreadLocal) != hipSuccess) {
        (void)hipGetLastError();
        return OMNI_ERR_HIP;
    }
    return OMNI_OK;
}

omni_status_t omni_graph_end(void *stream, omni_graph_t *out_graph) {
    if (out_graph) *out_graph = nullptr;
    if (!stream) return OMNI_ERR_UNSUPPORTED;
    hipGraph_t graph = nullptr;
    const hipError_t e = hipStreamEndCapture(reinterpret_cast<hipStream_t>(stream), &graph);   // always ends the capture
    if (!out_graph) {
        if (graph) (void)hipGraphDestroy(graph);
        return OMNI_ERR_NULL;
    }
    if (e != hipSuccess || !graph) {
        (void)hipGetLastError();
        if (graph) (void)hipGraphDestroy(graph);
        return OMNI_ERR_HIP;
    }
    omni_graph_s *g = new (std::nothrow) omni_graph_s();
    if (!g || hipGraphInstantiate(&g->exec, graph, nullptr, nullptr, 0) != hipSuccess) {
        (void)hipGetLastError();
        (void)hipGraphDestroy(graph);
        const omni_status_t st = g ? OMNI_ERR_HIP : OMNI_ERR_NOMEM;
        delete g;
        return st;
    }
    (void)hipGraphDestroy(graph);
    *out_graph = g;
    return OMNI_OK;
}

omni_status_t omni_graph_launch(omni_graph_t g, void *stream) {
    if (!g || !g->exec) return OMNI_ERR_NULL;
    if (hipGraphLaunch(g->exec, reinterpret_cast<hipStream_t>(stream)) != hipSuccess) {
        (void)hipGetLastError();
        return OMNI_ERR_HIP;
    }
    return OMNI_OK;
}

void omni_graph_destroy(omni_graph_t g) {
    if (!g) return;
    if (g->exec) (void)hipGraphExecDestroy(g->exec);
    delete g;
}

}  // extern "C"
