/*
 * omni_attn.h - C ABI of the MI355X (gfx950) batched decode-attention library.
 *
 * The operation is the attention inside the forward step that the paper's
 * model runner executes once per decode iteration over the whole batch of an
 * autoregressive stage (Section 3.1, overview; Section 3.3, AR stage support:
 * every engine brings its own scheduler, KV manager and model runner), over
 * the paged KV cache the engine inherits (Section 5, LLM serving systems).  It is the same call for a Thinker-like text stage and a
 * Talker-like speech-token stage (Section 2.1).  One call = one attention
 * layer's decode step for the whole batch: every request contributes exactly
 * one query token, which attends to all context_lens[b] tokens of its request.
 *
 * Conventions for every entry point
 *   - Plain C, no exceptions, no errno.  Every function returns omni_status_t
 *     (except omni_status_string / omni_destroy).
 *   - All tensor arguments are DEVICE pointers unless the name says "host".
 *     The caller owns every tensor and the workspace.  The library allocates no
 *     device memory, frees none, and never synchronises the stream: calls are
 *     asynchronous with respect to the host (the omni_debug_* calls excepted).
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).
 *   - Only host-checkable conditions are reported (null pointers, shapes,
 *     dtypes, workspace size, launch errors).  Page ids or lengths stored in
 *     device arrays that point outside the pool are undefined behaviour.
 *   - A handle is not thread-safe; distinct handles are independent.
 *
 * Layouts (row-major, contiguous)
 *   q, out              [batch, num_q_heads, head_dim]
 *   k_new, v_new        [batch, num_kv_heads, head_dim]
 *                       (with OMNI_TUNE_QUERY_TOKENS = T > 1: q, out [batch, T, num_q_heads, head_dim] and
 *                       k_new, v_new [batch, T, num_kv_heads, head_dim], see omni_paged_decode_attn)
 *   k_cache, v_cache    [num_pages, num_kv_heads, page_size, head_dim]   (two separate pools)
 *   block_table         [batch, max_blocks_per_seq] int32; entry j of row b is the physical page of
 *                       tokens [j*page_size, (j+1)*page_size) of request b; entries at or beyond
 *                       ceil(context_lens[b] / page_size) are never read
 *   context_lens        [batch] int32; tokens the query attends to, INCLUDING a token appended in
 *                       this step; 0 is legal and yields an all-zero output row
 *   positions           [batch] int32; token index at which omni_kv_append writes; < 0 skips the request
 * Query head h reads KV head h / (num_q_heads / num_kv_heads).  No mask, bias, window or soft-cap.
 * Alignment: q, out, k_new, v_new, k_cache and v_cache must be 16-byte aligned (rows are moved in 16-byte pieces);
 * the int32 arrays 4-byte aligned.  A misaligned pointer is reported as OMNI_ERR_SHAPE.
 */
#ifndef OMNI_ATTN_H
#define OMNI_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    OMNI_OK = 0,
    OMNI_ERR_NULL = 1,          /* a required pointer is NULL */
    OMNI_ERR_SHAPE = 2,         /* a size is non-positive, or num_q_heads is not a multiple of num_kv_heads */
    OMNI_ERR_DTYPE = 3,         /* unknown dtype code or unsupported q/kv/out combination */
    OMNI_ERR_UNSUPPORTED = 4,   /* head_dim, page_size, group size or batch outside what the kernels cover */
    OMNI_ERR_WORKSPACE = 5,     /* workspace missing, misaligned or smaller than omni_workspace_bytes */
    OMNI_ERR_HIP = 6,           /* the HIP runtime reported an error at launch */
    OMNI_ERR_NOMEM = 7          /* host memory for a handle or a graph object could not be allocated */
} omni_status_t;

typedef enum {
    OMNI_F32 = 0,
    OMNI_BF16 = 1,
    OMNI_FP8_E4M3 = 2           /* kv_dtype only: OCP 8-bit float (1-4-3, bias 7, max 448, no infinity), see omni_paged_decode_attn_fp8 */
} omni_dtype_t;

/* Problem description, fixed for the lifetime of a handle.  Set struct_size = sizeof(omni_attn_desc_t). */
typedef struct {
    uint32_t struct_size;
    int32_t  batch;                 /* B, 1 .. 4096 */
    int32_t  num_q_heads;           /* Hq, multiple of num_kv_heads; group size Hq/Hkv <= 16 */
    int32_t  num_kv_heads;          /* Hkv */
    int32_t  head_dim;              /* 64 or 128 */
    int32_t  page_size;             /* 16 or 32 tokens */
    int32_t  num_pages;             /* P, pages in each pool */
    int32_t  max_blocks_per_seq;    /* row length of block_table */
    int32_t  q_dtype;               /* omni_dtype_t; must equal kv_dtype, except OMNI_BF16 queries over an OMNI_FP8_E4M3 cache */
    int32_t  kv_dtype;              /* omni_dtype_t */
    int32_t  out_dtype;             /* omni_dtype_t; OMNI_BF16 only with bf16 q/kv */
    int32_t  max_context_hint;      /* upper bound on any context_lens[b] if the caller knows one; <= 0: max_blocks_per_seq*page_size */
} omni_attn_desc_t;

typedef struct omni_handle_s *omni_handle_t;

/* Tuning keys for omni_set_tuning.  Defaults are chosen for 256 compute units. */
typedef enum {
    OMNI_TUNE_KERNEL = 0,           /* 0 = auto, 1 = vector-ALU kernel, 2 = matrix-core (MFMA) kernel (bf16, head_dim 128 only) */
    OMNI_TUNE_TARGET_WORKGROUPS = 1,/* workgroups the attention kernel is launched with (> 0; rounded down to a multiple of Hkv) */
    OMNI_TUNE_MIN_PARTITION = 2,    /* smallest range of context, in tokens, one workgroup may be given (multiple of 32) */
    OMNI_TUNE_FORCE_PARTITION = 3,  /* > 0: every workgroup range is exactly this many tokens (multiple of 32); 0 = plan decides */
    OMNI_TUNE_PREFILL_SPLITS = 4,   /* omni_paged_prefill_attn, matrix-core path: 0 = the library decides from the grid how many
                                       workgroups may share a query block's context, 1 = never split, 2 .. 16 = this many */
    OMNI_TUNE_PREFILL_MIN_SPLIT = 5,/* fewest tokens of context one of them takes (multiple of 64; default 256): a query
                                       block with a shorter context is shared by fewer, decided on the device */
    OMNI_TUNE_QUERY_TOKENS = 6,     /* T >= 1 (default 1): omni_paged_decode_attn and omni_paged_decode_attn_fp8 take T query
                                       tokens per request, see there.  Matrix-core kernel only, else UNSUPPORTED */
    OMNI_TUNE_PREFILL_SORT = 7      /* omni_paged_prefill_attn, matrix-core path with a registered workspace and more than 256
                                       workgroups: 1 (default) = requests are taken longest context first (one more tiny
                                       launch ranks them), 0 = in batch order */
} omni_tune_key_t;

/* Validate `desc` and create a handle holding host-side plan state only (no device memory).
 * Errors: NULL, SHAPE, DTYPE, UNSUPPORTED.  On error *out_handle is set to NULL. */
omni_status_t omni_create(const omni_attn_desc_t *desc, omni_handle_t *out_handle);

/* Release the host-side state.  NULL is ignored.  The workspace stays the caller's. */
void omni_destroy(omni_handle_t h);

/* Change a tuning value.  This may change the workspace size and layout, so it forgets the registered workspace:
 * query omni_workspace_bytes and call omni_set_workspace again afterwards.  Errors: NULL, SHAPE (bad value),
 * UNSUPPORTED (kernel not available for this description). */
omni_status_t omni_set_tuning(omni_handle_t h, int32_t key, int32_t value);

/* Bytes of device workspace omni_paged_decode_attn needs for this handle (split-context partials and plan words). */
omni_status_t omni_workspace_bytes(omni_handle_t h, size_t *bytes);

/* Bytes of workspace with which omni_paged_prefill_attn splits the context for chunks of up to max_q_len tokens
 * (0 where it would not split).  The one registered workspace serves both calls: register the larger of the two
 * sizes.  Errors: NULL, SHAPE (max_q_len <= 0). */
omni_status_t omni_prefill_workspace_bytes(omni_handle_t h, int32_t max_q_len, size_t *bytes);

/* With OMNI_TUNE_QUERY_TOKENS = T > 1: a DEVICE array [batch] int32 that says how many query tokens each request
 * brings in the calls that follow, 0 .. T (values outside are clamped): request b's are the last dev_q_lens[b] tokens of
 * its context, in rows 0 .. dev_q_lens[b] - 1 of its T rows of q / out / k_new / v_new; its other rows of out are
 * written as zeros and its other new rows are not appended.  The library keeps the pointer and reads the array on the
 * device at every launch (so a recorded graph follows its contents).  NULL (the default): every request brings T.
 * Errors: NULL (handle), SHAPE (alignment). */
omni_status_t omni_set_query_lens(omni_handle_t h, const int32_t *dev_q_lens);

/* Hand the library a caller-owned device buffer of at least omni_workspace_bytes, 256-byte aligned.
 * The library keeps the pointer only; contents need no initialisation.  The buffer must not be shared by calls that
 * run concurrently.  Errors: NULL, WORKSPACE. */
omni_status_t omni_set_workspace(omni_handle_t h, void *dev_ptr, size_t bytes);

/*
 * out[b, h, :] = sum_t softmax_t(scale * q[b, h, :] . K_t) V_t over the context_lens[b] tokens of request b,
 * K_t / V_t being row (t % page_size) of page block_table[b][t / page_size], KV head h / (Hq/Hkv).
 * Accumulation is fp32.  The batch's context, laid end to end in 32-token tiles, is cut on the device into equal
 * ranges, one per workgroup (split-context / flash-decoding with an online softmax per piece); a request that is cut
 * by a range boundary is put together again by a log-sum-exp merge.  Both are exact re-associations of the definition
 * above.  Two kernel launches (attention, merge).  Writes `out` and the workspace, nothing else.
 * For a fixed handle and tuning the result is bit-identical from run to run and under any physical page permutation.
 * Several query tokens per request (speculative decoding, multi-token prediction; OMNI_TUNE_QUERY_TOKENS = T > 1): q
 * and out are [batch, T, num_q_heads, head_dim]; the T tokens are the LAST T of the context_lens[b] tokens (their K/V
 * rows are in the pools: omni_kv_append_chunk), query i sees tokens 0 .. context_lens[b] - T + i.  The kernel treats
 * the (token, head) pairs of a KV head as the columns of its matrix-core tiles, 16 per pass: with T * (Hq / Hkv) <= 16
 * the cache is still read once and the call costs about what the one-token call costs; a larger T takes
 * ceil(T / floor(16 / (Hq / Hkv))) passes (launch pairs) over the cache.  Every request has T tokens unless
 * omni_set_query_lens says otherwise;
 * a query that would see no token at all (context_lens[b] < T) gets zeros.  omni_decode_step and omni_decode_step_fp8
 * then take k_new / v_new [batch, T, num_kv_heads, head_dim] and write row i of request b to position
 * context_lens[b] - T + i (rows whose position would be negative are skipped) before the attention reads it.
 * Ragged numbers of new tokens: omni_paged_prefill_attn.
 * Errors: NULL, WORKSPACE, HIP.
 */
omni_status_t omni_paged_decode_attn(omni_handle_t h,
                                     const void *q, const void *k_cache, const void *v_cache,
                                     const int32_t *block_table, const int32_t *context_lens,
                                     float scale, void *out, void *stream);

/*
 * omni_paged_decode_attn for callers that cannot allocate device memory and so have no workspace to register: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels, same
 * results bit for bit; the plan words and partial rows go to an 8 MiB array that lives in the library's device image
 * (each GPU the library runs on holds its copy until the process ends) instead of the handle's workspace, which need
 * not be set.  The call makes no hipMalloc / hipFree and calls no allocating routine; its first call on a device looks
 * up the array's address.  All handles and streams of a process share a GPU's array: calls that overlap in time on
 * one GPU (different streams or threads) race on it, so issue them on one stream or order them yourself.  Nothing in
 * the array needs clearing between calls.  16-bit and fp32 caches only.
 * Errors: NULL, UNSUPPORTED (fp8 handle), WORKSPACE (omni_workspace_bytes of the handle exceeds 8 MiB: register a
 * workspace and use omni_paged_decode_attn), SHAPE (alignment), HIP.
 */
omni_status_t omni_paged_decode_attn_static(omni_handle_t h,
                                            const void *q, const void *k_cache, const void *v_cache,
                                            const int32_t *block_table, const int32_t *context_lens,
                                            float scale, void *out, void *stream);

/*
 * The same attention over a quantised KV cache (the paper lists quantised attention only among its diffusion engine's
 * options, Section 3.3; here it halves the bytes the decode path streams).  The handle is created with
 * kv_dtype = OMNI_FP8_E4M3, q_dtype = OMNI_BF16, head_dim 128.  k_cache / v_cache hold one E4M3 byte per element in
 * the same [num_pages, num_kv_heads, page_size, head_dim] layout; k_scale / v_scale are DEVICE arrays
 * [num_pages, num_kv_heads] of fp32, and element (page, g, slot, d) stands for decode(byte) * scale[page, g].
 * Bytes are widened exactly to bf16 in registers, products and sums are fp32, the K scale joins the softmax scale and
 * the V scale the softmax weights.  NaN bytes in slots no live token owns never reach the result.
 * omni_kv_append, omni_kv_pack and omni_kv_unpack move the bytes of such a cache like any other (scales are the
 * caller's); omni_paged_decode_attn, omni_decode_step and omni_paged_prefill_attn return OMNI_ERR_UNSUPPORTED for it
 * (their forms for such a cache: omni_decode_step_fp8, omni_paged_prefill_attn_fp8).  Scales must be positive.
 * Errors: NULL, SHAPE (alignment), UNSUPPORTED (handle is not an fp8 one), WORKSPACE, HIP.
 */
omni_status_t omni_paged_decode_attn_fp8(omni_handle_t h,
                                         const void *q, const void *k_cache, const void *v_cache,
                                         const float *k_scale, const float *v_scale,
                                         const int32_t *block_table, const int32_t *context_lens,
                                         float scale, void *out, void *stream);

/*
 * Autoregressive decoding adds one token per request per iteration (Section 2.2, the AR decoding loop): copy, bit for
 * bit, k_new[b, g, :] and v_new[b, g, :] into row (positions[b] % page_size) of page
 * block_table[b][positions[b] / page_size], KV head g, of k_cache / v_cache.  Requests with positions[b] < 0 are
 * skipped.  Writes only the addressed rows.  Errors: NULL, HIP.
 */
omni_status_t omni_kv_append(omni_handle_t h,
                             const void *k_new, const void *v_new, void *k_cache, void *v_cache,
                             const int32_t *block_table, const int32_t *positions, void *stream);

/*
 * One decode iteration of an autoregressive stage for the whole batch (Section 3.1: the model runner takes one
 * forward step over the whole batch per iteration; Section 2.2: the AR decoding loop adds one token per request):
 * exactly omni_kv_append with
 * positions[b] = context_lens[b] - 1 (requests of length 0 are skipped) followed by omni_paged_decode_attn, but with
 * the append fused into the attention kernel where the hardware path allows it (bf16, head_dim 128): the wave that
 * reads a request's last tile takes the new K/V row from k_new / v_new in place of that row of the page and writes it
 * into the page.  Same results, bit for bit, as the two separate calls; k_cache / v_cache hold the new rows when the
 * call has completed in stream order.
 * Errors: NULL, WORKSPACE, HIP.
 */
omni_status_t omni_decode_step(omni_handle_t h,
                               const void *q, const void *k_new, const void *v_new, void *k_cache, void *v_cache,
                               const int32_t *block_table, const int32_t *context_lens,
                               float scale, void *out, void *stream);

/* The decode iteration over the quantised cache: k_new / v_new [batch, num_kv_heads, head_dim] hold E4M3 BYTES, already
 * divided by the scale of the page they go to (position context_lens[b] - 1); exactly omni_kv_append of those bytes
 * followed by omni_paged_decode_attn_fp8, in one launch of the attention kernel plus the merge.  Quantising the new
 * rows, and choosing a page's scale before its first row arrives, is the caller's.
 * Errors: NULL, SHAPE (alignment), UNSUPPORTED (handle is not an fp8 one), WORKSPACE, HIP. */
omni_status_t omni_decode_step_fp8(omni_handle_t h, const void *q, const void *k_new, const void *v_new, void *k_cache,
                                   void *v_cache, const float *k_scale, const float *v_scale, const int32_t *block_table,
                                   const int32_t *context_lens, float scale, void *out, void *stream);

/*
 * The append that quantises (Section 2.2: the AR decoding loop adds one token per request per iteration; here into the
 * quantised cache of omni_paged_decode_attn_fp8).  k_new / v_new [batch, num_kv_heads, head_dim] are bf16 rows; row
 * (b, g) goes to slot positions[b] % page_size of page block_table[b][positions[b] / page_size], KV head g, as
 *     byte = E4M3(clamp(x / scale, -448, 448)),  round to nearest even,  NaN -> 0x7f,
 * with the scale of that (page, KV head).  A row that lands in slot 0 opens its page and fixes that scale first:
 *     scale = max(amax * headroom, 2^-100) / 448,   amax = the row's largest magnitude
 * (written to k_scale / v_scale [num_pages, num_kv_heads]); every other row uses the scale its page already has, and
 * values beyond 448 * scale saturate.  headroom >= 1 leaves room for the page's later rows (1 = the opening row's
 * largest element maps to 448 exactly).  All arithmetic is fp32; K and V are treated alike.  Requests with
 * positions[b] < 0 are skipped; two requests must not write into the same page in one call.  One launch.
 * Errors: NULL, UNSUPPORTED (handle is not an fp8 one), SHAPE (headroom outside [1, 65536], alignment), HIP.
 */
omni_status_t omni_kv_append_quant_fp8(omni_handle_t h, const void *k_new, const void *v_new, void *k_cache, void *v_cache,
                                       float *k_scale, float *v_scale, const int32_t *block_table,
                                       const int32_t *positions, float headroom, void *stream);

/*
 * Dense copies of whole requests, the payload a connector ships when the KV cache of a request moves between a
 * prefill and a decode engine (Section 3.4, disaggregated data transfer: the connector also carries KV cache between
 * prefill and decode).  For every request b with token_offsets[b] >= 0 and every t < context_lens[b]:
 *   pack:    k_dense[token_offsets[b] + t, g, :] = k_cache[block_table[b][t / page_size], g, t % page_size, :]
 *   unpack:  the same assignment in the other direction
 * and likewise for V; bit copies.  k_dense / v_dense are [total tokens, num_kv_heads, head_dim] DEVICE buffers of the
 * cache dtype; token_offsets is a DEVICE array [batch] of int64 (first dense row of each request; < 0 skips the
 * request; the caller keeps the ranges of different requests apart).  Pack writes only the addressed dense rows,
 * unpack only the addressed pool rows.  Lengths above max_context_hint (if one was given) are not supported.
 * One launch each; grid (ceil(max context / 32), batch), data-independent.  Errors: NULL, SHAPE (alignment), HIP.
 */
omni_status_t omni_kv_pack(omni_handle_t h, const void *k_cache, const void *v_cache, const int32_t *block_table,
                           const int32_t *context_lens, const int64_t *token_offsets, void *k_dense, void *v_dense,
                           void *stream);
omni_status_t omni_kv_unpack(omni_handle_t h, const void *k_dense, const void *v_dense, void *k_cache, void *v_cache,
                             const int32_t *block_table, const int32_t *context_lens, const int64_t *token_offsets,
                             void *stream);

/*
 * Multi-token queries over the paged cache (chunked prefill, which Section 2.2 and Section 3.3 list among the AR
 * engine's features; also how a stage consumes a whole sequence of upstream hidden states in one pass).  Request b
 * brings q_lens[b] new tokens, the LAST q_lens[b] of its context_lens[b] tokens; their query rows are rows
 * q_offsets[b] .. q_offsets[b] + q_lens[b] - 1 of q [total rows, num_q_heads, head_dim] and their results go to the
 * same rows of out.  Query i of the chunk sits at position p = context_lens[b] - q_lens[b] + i and attends to tokens
 * 0 .. p: causal inside the chunk, everything before it.  With q_lens[b] = 1 this is omni_paged_decode_attn.
 *   out[q_offsets[b] + i, h, :] = sum_{t <= p} softmax_t(scale * q[q_offsets[b] + i, h, :] . K_t) V_t
 * The chunk's K/V rows must be in the pools already (omni_kv_append_chunk).  q_lens [batch] int32 and q_offsets
 * [batch] int64 are DEVICE arrays; max_q_len is a HOST upper bound on q_lens (it sizes the grid; longer chunks are
 * cut off).  Rows of out that no request owns are not written; requests with q_lens[b] <= 0 are skipped.
 * bf16 q/K/V with head_dim 128 run on the matrix cores (fp32 accumulation).  There V enters the weighted sum as
 * fp16: exact for 2^-14 <= |V| <= 65504; a smaller value carries an absolute error of at most 2^-25; a larger one (or a
 * non-finite one) makes non-finite outputs for the queries of its request whose tiles reach it, never wrong finite
 * ones; and scale must be positive.  Every other fp32 / bf16 configuration (and this one under OMNI_TUNE_KERNEL = 1)
 * runs a plain vector-ALU kernel in fp32 arithmetic, without those two conditions.  An 8-bit cache:
 * OMNI_ERR_UNSUPPORTED here, see omni_paged_prefill_attn_fp8.
 * One launch and no workspace, unless the call would leave most of the chip idle (few requests, short chunks: a
 * workgroup owns floor(256 / group size) query tokens of one request and KV head) and the registered workspace holds
 * at least omni_prefill_workspace_bytes(max_q_len): then the matrix-core path lets up to 16 workgroups share a
 * query block's context in equal runs of 64-token steps (as many as the context gives OMNI_TUNE_PREFILL_MIN_SPLIT
 * tokens each), and a second launch merges their pieces (log-sum-exp, in order of position: the same exact
 * re-association as in decode).  How a block is shared depends on the handle, its tuning, max_q_len and the lengths
 * only, so the result is bit-identical from run to run.  With a registered workspace and more than 256 workgroups a
 * one-workgroup launch first ranks the requests by context length, and the kernel takes them longest first (the order
 * changes when a workgroup runs, not what it computes).
 * Errors: NULL, SHAPE (max_q_len <= 0, scale <= 0 on the matrix-core path, alignment), UNSUPPORTED, HIP.
 */
omni_status_t omni_paged_prefill_attn(omni_handle_t h, const void *q, const void *k_cache, const void *v_cache,
                                      const int32_t *block_table, const int32_t *context_lens, const int32_t *q_lens,
                                      const int64_t *q_offsets, int32_t max_q_len, float scale, void *out, void *stream);

/* omni_paged_prefill_attn over the quantised cache of omni_paged_decode_attn_fp8 (same handle, pools and scales; same
 * matrix-core kernel, context split and workspace rule).  K bytes are widened exactly to bf16; a V element enters the
 * weighted sum as decode(byte) * scale rounded once to fp16 (relative error 2^-12; its magnitude must stay within the
 * fp16 range as above); the K scale of a page joins the softmax scale.  scale must be positive.
 * Errors: NULL, SHAPE, UNSUPPORTED (handle is not an fp8 one), HIP. */
omni_status_t omni_paged_prefill_attn_fp8(omni_handle_t h, const void *q, const void *k_cache, const void *v_cache,
                                          const float *k_scale, const float *v_scale, const int32_t *block_table,
                                          const int32_t *context_lens, const int32_t *q_lens, const int64_t *q_offsets,
                                          int32_t max_q_len, float scale, void *out, void *stream);

/* The multi-token form of omni_kv_append: row q_offsets[b] + i of k_new / v_new [total rows, num_kv_heads, head_dim]
 * is copied, bit for bit, to position context_lens[b] - q_lens[b] + i of request b, for i < q_lens[b].  Any dtype
 * the handle supports.  max_q_len as above.  Errors: NULL, SHAPE, HIP. */
omni_status_t omni_kv_append_chunk(omni_handle_t h, const void *k_new, const void *v_new, void *k_cache, void *v_cache,
                                   const int32_t *block_table, const int32_t *context_lens, const int32_t *q_lens,
                                   const int64_t *q_offsets, int32_t max_q_len, void *stream);

/* Host-known part of the launch plan: which kernel (OMNI_TUNE_KERNEL value actually used), the data-independent
 * grid (workgroups) of the attention kernel, the grid of the merge kernel that follows it, the number of
 * partial-result slots the workspace is sized for, and threads per workgroup.  The range length itself is chosen on the device from
 * context_lens; omni_debug_last_plan reads it back. */
omni_status_t omni_get_plan(omni_handle_t h, int32_t *kernel, int32_t *partition_grid, int32_t *merge_grid,
                            int32_t *max_request_parts, int32_t *threads_per_workgroup);

const char *omni_status_string(omni_status_t s);

/*
 * Execution graphs (Section 3.3 lists execution-graph compilation among the engine's options and Section 4 credits
 * it with the largest gains of the autoregressive stages).  Every launch above has a grid that does not depend on
 * device data, allocates nothing and never synchronises, so a sequence of omni_decode_step / omni_paged_decode_attn /
 * omni_kv_append calls (for instance one per layer) can be recorded once and replayed with one host call per token:
 *   omni_graph_begin(stream);  ... calls on `stream` ...;  omni_graph_end(stream, &g);  omni_graph_launch(g, stream);
 * The graph replays the recorded pointers and scalar arguments (scale); the CONTENTS of q, context_lens, block_table,
 * k_new / v_new and the pools may change between replays.  `stream` must be a created stream (not NULL: the null
 * stream cannot be captured).  Between begin and end the calling thread must make no synchronising or allocating HIP call on any
 * stream, and each handle used must have run once on this device before (its first launch configures the kernel).
 * A graph is replayed on one stream at a time (the handles' workspaces are in it).  omni_graph_end returns the
 * instantiated graph; omni_graph_destroy(NULL) is a no-op.
 * Errors: NULL, UNSUPPORTED (null stream), HIP (capture or instantiation failed; the capture is ended and dropped).
 */
typedef struct omni_graph_s *omni_graph_t;
omni_status_t omni_graph_begin(void *stream);
omni_status_t omni_graph_end(void *stream, omni_graph_t *out_graph);
omni_status_t omni_graph_launch(omni_graph_t g, void *stream);
void omni_graph_destroy(omni_graph_t g);

/* ---- test / debugging aids: these synchronise the stream and copy to HOST memory ---- */

/* After an omni_paged_decode_attn call on `stream`: host_out[0] = range length (tokens) the device chose,
 * host_out[1] = number of ranges, host_out[2] = total context tokens, host_out[3] = reserved. */
omni_status_t omni_debug_last_plan(omni_handle_t h, int32_t host_out[4], void *stream);

/* Dense copy of one request's rows of `cache` (k_cache or v_cache), in token order, into DEVICE buffer
 * dense_out [context_lens[request], num_kv_heads, head_dim] (a bit copy).  Launches on `stream`, no sync. */
omni_status_t omni_debug_gather(omni_handle_t h, const void *cache, const int32_t *block_table,
                                const int32_t *context_lens, int32_t request, void *dense_out, void *stream);

/* Measurement aid: a plain streaming read of a_bytes at a followed by b_bytes at b (device pointers, 16-byte aligned,
 * sizes multiples of 16; b may be null with b_bytes = 0), launched on `stream` like the attention kernel.  `sink`
 * points at 4 writable device bytes.  Timed on buffers of the KV pool's size it gives the memory system's ceiling for a
 * kernel of the attention kernel's duration, the figure the attention kernel's bandwidth is compared with.
 * Errors: OMNI_ERR_NULL, OMNI_ERR_SHAPE (alignment), OMNI_ERR_HIP. */
omni_status_t omni_debug_stream_read(const void *a, size_t a_bytes, const void *b, size_t b_bytes, void *sink,
                                     void *stream);

/* Host-only: the shared-memory layout the matrix-core kernel of this handle is launched with.  host_out[0] = bytes of
 * dynamic shared memory, [1] = bytes of the kernel variant's static K staging area, [2] = online-softmax states the
 * ring holds (4 .. 16), [3] = 1 if K
 * tiles are staged through shared memory, [4] = 1 if two workgroups fit one compute unit's 160 KB, [5] = the most
 * dynamic shared memory any launch may ask for.  Errors: NULL, UNSUPPORTED (the handle runs the vector-ALU kernel). */
omni_status_t omni_debug_lds_layout(omni_handle_t h, int32_t host_out[6]);

/* What the loaded code object says about a kernel of this handle (hipFuncGetAttributes; needs a device): which = 0 the
 * attention kernel variant the handle launches (matrix-core kernel only), 1 the merge kernel.  host_out[0] = registers
 * per lane, [1] = static shared memory in bytes, [2] = dynamic shared memory at launch, [3] = the kernel's thread
 * limit per workgroup, [4] = scratch (spill) bytes per lane, [5] = threads per workgroup the library launches.
 * Errors: NULL, SHAPE (which), UNSUPPORTED, HIP. */
omni_status_t omni_debug_kernel_resources(omni_handle_t h, int32_t which, int32_t host_out[6]);

/* Profiling aid for the benchmark.  After omni_debug_profile_begin(h, capacity, stride) every stride-th attention
 * call (omni_paged_decode_attn or omni_decode_step; the first one included) records a HIP event pair around its
 * attention kernel (the kernel that reads the KV cache) on the caller's stream, until `capacity` pairs are used;
 * for the matrix-core kernel the pair is attached to the kernel's dispatch, so it spans that kernel alone.  Do not
 * capture such calls into a graph.  An event pair costs a few microseconds of stream time, hence the stride.  omni_debug_profile_end synchronises the
 * recorded events, writes the elapsed milliseconds of each recorded launch to host_ms[0 .. *count) (host_ms must hold
 * `capacity` floats), destroys the events and switches recording off.  Errors: NULL, SHAPE (capacity or stride <= 0),
 * HIP. */
omni_status_t omni_debug_profile_begin(omni_handle_t h, int32_t capacity, int32_t stride);
omni_status_t omni_debug_profile_end(omni_handle_t h, float *host_ms, int32_t *count);

#ifdef __cplusplus
}
#endif
#endif /* OMNI_ATTN_H */
