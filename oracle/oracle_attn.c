/*
 * CPU oracle for batched single-token decode attention over a paged KV cache.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the HIP
 * path is checked against.  It shares no code, header, table or helper with the
 * HIP library, and the product path never calls it.
 *
 * What it follows.  The paper (Section 3.1 "Overview"; Section 3.3 "AR stage
 * support") has every autoregressive stage run one batched forward step per
 * iteration over the requests its scheduler picked, each engine with its own KV
 * manager; Section 5 ("LLM serving systems") names the attention it inherits as
 * paged attention over a managed KV cache.  The paper prints no formula for
 * attention, so the arithmetic below is the textbook definition of scaled
 * dot-product attention for one query token per request, taken over the rows
 * that the request's block table addresses:
 *
 *     s_t = scale * sum_d q[d] * k_t[d]
 *     out = sum_t softmax(s)_t * v_t
 *
 * All arithmetic is IEEE double.  Stored fp32 / bf16 values are widened exactly.
 * `scale` arrives as the caller's fp32 value and is widened, not recomputed.
 *
 * Layouts (row-major, contiguous):
 *   q, out        [B, Hq, D]
 *   k_cache, v_cache  [P, Hkv, ps, D]      one (page, KV head) tile is contiguous
 *   block_table   [B, MB] int32            entry j of row b = physical page of tokens [j*ps, (j+1)*ps)
 *   context_lens  [B] int32                tokens the query attends to (includes a token appended this step)
 * Query head h reads KV head h / (Hq / Hkv)  (contiguous groups).
 * A request of length 0 yields an all-zero output row.
 *
 * Pins (tests/test_oracle_pins.py, all CPU): dense unpaged brute force written
 * separately in numpy; length-1 context returns the V row bit-exactly; identical
 * keys (or a zero query) return the mean of V; closed form for length 2; a
 * hand-worked example under tests/golden/; key-shift invariance at |shift| ~ 80;
 * one dominant key; convex-hull bound; bit-identical output under physical page
 * permutation and under a change of page size; NaN poison in unowned slots never
 * reaches the output; split-and-merge equals the unsplit result; append touches
 * exactly one row per (request, KV head).
 * Behaviour for non-finite *live* inputs is not pinned ("parity unpinned").
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };

typedef struct {
    int32_t B, Hq, Hkv, D, ps, MB;
    int32_t q_dtype, kv_dtype;          /* ORACLE_F32 / ORACLE_BF16 */
} oracle_shape_t;

static double widen(const void *base, int64_t idx, int dtype)
{
    if (dtype == ORACLE_F32) {
        return (double)((const float *)base)[idx];
    } else {
        uint32_t bits = (uint32_t)((const uint16_t *)base)[idx] << 16;
        float f;
        memcpy(&f, &bits, sizeof f);
        return (double)f;
    }
}

static int elem_size(int dtype) { return dtype == ORACLE_F32 ? 4 : 2; }

/* element offset of row (token t of request b, KV head g) inside a cache pool */
static int64_t row_offset(const oracle_shape_t *s, const int32_t *block_table, int b, int g, int t)
{
    int64_t page = block_table[(int64_t)b * s->MB + t / s->ps];
    int64_t slot = t % s->ps;
    return ((page * s->Hkv + g) * s->ps + slot) * s->D;
}

/* Scores of tokens [t0, t1) for (request b, query head h) into s_out[0 .. t1-t0). */
static void scores(const oracle_shape_t *s, const void *q, const void *k_cache, const int32_t *block_table,
                   double scale, int b, int h, int t0, int t1, double *s_out)
{
    int G = s->Hq / s->Hkv, g = h / G;
    int64_t qoff = ((int64_t)b * s->Hq + h) * s->D;
    for (int t = t0; t < t1; ++t) {
        int64_t koff = row_offset(s, block_table, b, g, t);
        double acc = 0.0;
        for (int d = 0; d < s->D; ++d)
            acc += widen(q, qoff + d, s->q_dtype) * widen(k_cache, koff + d, s->kv_dtype);
        s_out[t - t0] = scale * acc;
    }
}

/*
 * Unnormalised attention of (b, h) over tokens [t0, t1):
 *   m = max_t s_t,  l = sum_t exp(s_t - m),  o[d] = sum_t exp(s_t - m) * v_t[d].
 * An empty range gives m = -inf, l = 0, o = 0.
 */
static void partial(const oracle_shape_t *s, const void *q, const void *k_cache, const void *v_cache,
                    const int32_t *block_table, double scale, int b, int h, int t0, int t1,
                    double *o, double *m_out, double *l_out)
{
    int G = s->Hq / s->Hkv, g = h / G;
    int n = t1 - t0;
    for (int d = 0; d < s->D; ++d) o[d] = 0.0;
    if (n <= 0) { *m_out = -INFINITY; *l_out = 0.0; return; }
    double *sc = (double *)malloc(sizeof(double) * (size_t)n);
    scores(s, q, k_cache, block_table, scale, b, h, t0, t1, sc);
    double m = sc[0];
    for (int i = 1; i < n; ++i) if (sc[i] > m) m = sc[i];
    double l = 0.0;
    for (int i = 0; i < n; ++i) {
        double p = exp(sc[i] - m);
        l += p;
        int64_t voff = row_offset(s, block_table, b, g, t0 + i);
        for (int d = 0; d < s->D; ++d) o[d] += p * widen(v_cache, voff + d, s->kv_dtype);
    }
    free(sc);
    *m_out = m; *l_out = l;
}

/*
 * out[b, h, :] = softmax(scale * q K^T) V for every (b, h), or only for the
 * npairs (b, h) pairs listed in `pairs` (then out is [npairs, D]).
 * Returns the number of threads that did the work.
 */
int oracle_paged_decode_attn(const oracle_shape_t *s, const void *q, const void *k_cache, const void *v_cache,
                             const int32_t *block_table, const int32_t *context_lens, float scale,
                             double *out, const int32_t *pairs, int32_t npairs, int32_t num_threads)
{
    int64_t total = pairs ? npairs : (int64_t)s->B * s->Hq;
    int used = 1;
#ifdef _OPENMP
    if (num_threads > 0) omp_set_num_threads(num_threads);
    #pragma omp parallel
    {
        #pragma omp single
        used = omp_get_num_threads();
    }
    #pragma omp parallel for schedule(dynamic, 1)
#endif
    for (int64_t i = 0; i < total; ++i) {
        int b = pairs ? pairs[2 * i] : (int)(i / s->Hq);
        int h = pairs ? pairs[2 * i + 1] : (int)(i % s->Hq);
        double m, l;
        double *o = out + i * s->D;
        partial(s, q, k_cache, v_cache, block_table, (double)scale, b, h, 0, context_lens[b], o, &m, &l);
        if (l > 0.0)
            for (int d = 0; d < s->D; ++d) o[d] /= l;
    }
    return used;
}

/* Unnormalised (o, m, l) of one (b, h) over tokens [t0, t1): the quantity a split-context partition holds. */
void oracle_partial(const oracle_shape_t *s, const void *q, const void *k_cache, const void *v_cache,
                    const int32_t *block_table, float scale, int32_t b, int32_t h, int32_t t0, int32_t t1,
                    double *o, double *m, double *l)
{
    partial(s, q, k_cache, v_cache, block_table, (double)scale, b, h, t0, t1, o, m, l);
}

/*
 * Log-sum-exp merge of n partitions: with M = max_j m_j,
 *   out = sum_j exp(m_j - M) o_j / sum_j exp(m_j - M) l_j.
 * Partitions with l_j = 0 (empty) carry weight 0 and exp is never taken of
 * (-inf) - (-inf).  If every partition is empty the output is 0.
 */
void oracle_merge(int32_t n, int32_t D, const double *o /*[n, D]*/, const double *m, const double *l, double *out)
{
    double M = -INFINITY;
    for (int j = 0; j < n; ++j) if (l[j] > 0.0 && m[j] > M) M = m[j];
    double den = 0.0;
    for (int d = 0; d < D; ++d) out[d] = 0.0;
    for (int j = 0; j < n; ++j) {
        if (!(l[j] > 0.0)) continue;
        double w = exp(m[j] - M);
        den += w * l[j];
        for (int d = 0; d < D; ++d) out[d] += w * o[(int64_t)j * D + d];
    }
    if (den > 0.0) for (int d = 0; d < D; ++d) out[d] /= den;
}

/*
 * Write the new token's K and V rows of every request into its page:
 * page = block_table[b][pos / ps], slot = pos % ps, for every KV head; a bit copy.
 * positions[b] < 0 skips request b.  k_new, v_new are [B, Hkv, D].
 */
void oracle_kv_append(const oracle_shape_t *s, const void *k_new, const void *v_new, void *k_cache, void *v_cache,
                      const int32_t *block_table, const int32_t *positions)
{
    size_t es = (size_t)elem_size(s->kv_dtype), row = es * (size_t)s->D;
    for (int b = 0; b < s->B; ++b) {
        int pos = positions[b];
        if (pos < 0) continue;
        for (int g = 0; g < s->Hkv; ++g) {
            int64_t dst = row_offset(s, block_table, b, g, pos);
            int64_t src = ((int64_t)b * s->Hkv + g) * s->D;
            memcpy((char *)k_cache + (size_t)dst * es, (const char *)k_new + (size_t)src * es, row);
            memcpy((char *)v_cache + (size_t)dst * es, (const char *)v_new + (size_t)src * es, row);
        }
    }
}

/* Dense copy of request b's rows, in token order: dense_out is [L_b, Hkv, D], a bit copy. */
void oracle_gather(const oracle_shape_t *s, const void *cache, const int32_t *block_table,
                   const int32_t *context_lens, int32_t b, void *dense_out)
{
    size_t es = (size_t)elem_size(s->kv_dtype), row = es * (size_t)s->D;
    int L = context_lens[b];
    for (int t = 0; t < L; ++t)
        for (int g = 0; g < s->Hkv; ++g) {
            int64_t src = row_offset(s, block_table, b, g, t);
            int64_t dst = ((int64_t)t * s->Hkv + g) * s->D;
            memcpy((char *)dense_out + (size_t)dst * es, (const char *)cache + (size_t)src * es, row);
        }
}

/*
 * Multi-token queries over the paged cache (chunked prefill: Section 2.2 and Section 3.3 name chunked prefill among
 * the AR engine's scheduling features; a Talker prefill consumes the Thinker's hidden states in one such pass).
 * Request b contributes q_lens[b] query rows, stored at rows q_offsets[b] .. q_offsets[b] + q_lens[b] - 1 of
 * q [Tq, Hq, D]; query i of the chunk sits at position p = context_lens[b] - q_lens[b] + i of the request and attends
 * to tokens 0 .. p (causal inside the chunk, everything before it), context_lens[b] counting the chunk's own tokens:
 *
 *     out[q_offsets[b] + i, h, :] = sum_{t <= p} softmax_t(scale * q_row . k_t) v_t
 *
 * With q_lens[b] = 1 this is the decode definition above.  `rows` (optional) lists nrows triples (b, i, h) to compute
 * instead of everything; out is then [nrows, D], else [Tq, Hq, D].  Returns the number of threads used.
 * Pins: equals oracle_paged_decode_attn for one-token chunks; dense causal brute force in numpy; rows after a
 * query's position never influence it (NaN poison); the first token of a request returns its own V row.
 */
int oracle_paged_prefill_attn(const oracle_shape_t *s, const void *q, const void *k_cache, const void *v_cache,
                              const int32_t *block_table, const int32_t *context_lens, const int32_t *q_lens,
                              const int64_t *q_offsets, float scale, double *out, const int32_t *rows, int64_t nrows,
                              int32_t num_threads)
{
    int G = s->Hq / s->Hkv;
    int64_t total = nrows;
    int64_t *first = NULL;          /* without `rows`: prefix of q_lens, to enumerate (b, i) */
    if (!rows) {
        first = (int64_t *)malloc(sizeof(int64_t) * (size_t)(s->B + 1));
        first[0] = 0;
        for (int b = 0; b < s->B; ++b) first[b + 1] = first[b] + (q_lens[b] > 0 ? q_lens[b] : 0);
        total = first[s->B] * s->Hq;
    }
    int used = 1;
#ifdef _OPENMP
    if (num_threads > 0) omp_set_num_threads(num_threads);
    #pragma omp parallel
    {
        #pragma omp single
        used = omp_get_num_threads();
    }
    #pragma omp parallel for schedule(dynamic, 1)
#endif
    for (int64_t r = 0; r < total; ++r) {
        int b, i, h;
        if (rows) { b = rows[3 * r]; i = rows[3 * r + 1]; h = rows[3 * r + 2]; }
        else {
            int64_t row = r / s->Hq;
            h = (int)(r % s->Hq);
            b = 0;
            while (first[b + 1] <= row) ++b;
            i = (int)(row - first[b]);
        }
        int g = h / G;
        int n = context_lens[b] - q_lens[b] + i + 1;              /* tokens 0 .. p */
        int64_t qoff = ((q_offsets[b] + i) * s->Hq + h) * s->D;
        double *o = rows ? out + r * s->D : out + ((q_offsets[b] + i) * s->Hq + h) * s->D;
        for (int d = 0; d < s->D; ++d) o[d] = 0.0;
        if (n <= 0) continue;
        double *sc = (double *)malloc(sizeof(double) * (size_t)n);
        double m = -INFINITY;
        for (int t = 0; t < n; ++t) {
            int64_t koff = row_offset(s, block_table, b, g, t);
            double acc = 0.0;
            for (int d = 0; d < s->D; ++d)
                acc += widen(q, qoff + d, s->q_dtype) * widen(k_cache, koff + d, s->kv_dtype);
            sc[t] = (double)scale * acc;
            if (sc[t] > m) m = sc[t];
        }
        double l = 0.0;
        for (int t = 0; t < n; ++t) {
            double p = exp(sc[t] - m);
            l += p;
            int64_t voff = row_offset(s, block_table, b, g, t);
            for (int d = 0; d < s->D; ++d) o[d] += p * widen(v_cache, voff + d, s->kv_dtype);
        }
        for (int d = 0; d < s->D; ++d) o[d] /= l;
        free(sc);
    }
    free(first);
    return used;
}

/*
 * Quantised KV cache (8-bit floating point with one scale per page and KV head).  The stored byte is an OCP
 * "E4M3" number: 1 sign bit, 4 exponent bits (bias 7), 3 mantissa bits; exponent 0 holds subnormals m/8 * 2^-6;
 * there is no infinity and only the all-ones exponent with all-ones mantissa is NaN, so the largest finite value is
 * 1.75 * 2^8 = 448.  A cache element stands for   decode(byte) * scale[page, kv head].
 * The attention itself is the definition at the top of this file, taken over the de-quantised rows.
 * Pins: the decode against an independent conversion routine for all 256 bytes; with power-of-two scales the result
 * equals, bit for bit, the fp32 oracle run on the de-quantised pools; general scales to 1e-12.
 */
double oracle_fp8_e4m3_decode(uint8_t byte)
{
    int sign = byte >> 7, e = (byte >> 3) & 15, mant = byte & 7;
    double v;
    if (e == 15 && mant == 7) return NAN;
    if (e == 0) v = ldexp((double)mant / 8.0, -6);
    else v = ldexp(1.0 + (double)mant / 8.0, e - 7);
    return sign ? -v : v;
}

/* out[b, h, :] for every (b, h), or for the npairs listed pairs; k_scale / v_scale are [P, Hkv] fp32. */
int oracle_paged_decode_attn_fp8(const oracle_shape_t *s, const void *q, const uint8_t *k_cache, const uint8_t *v_cache,
                                 const float *k_scale, const float *v_scale, const int32_t *block_table,
                                 const int32_t *context_lens, float scale, double *out, const int32_t *pairs,
                                 int32_t npairs, int32_t num_threads)
{
    int G = s->Hq / s->Hkv;
    int64_t total = pairs ? npairs : (int64_t)s->B * s->Hq;
    int used = 1;
#ifdef _OPENMP
    if (num_threads > 0) omp_set_num_threads(num_threads);
    #pragma omp parallel
    {
        #pragma omp single
        used = omp_get_num_threads();
    }
    #pragma omp parallel for schedule(dynamic, 1)
#endif
    for (int64_t r = 0; r < total; ++r) {
        int b = pairs ? pairs[2 * r] : (int)(r / s->Hq);
        int h = pairs ? pairs[2 * r + 1] : (int)(r % s->Hq);
        int g = h / G, n = context_lens[b];
        double *o = out + r * s->D;
        for (int d = 0; d < s->D; ++d) o[d] = 0.0;
        if (n <= 0) continue;
        int64_t qoff = ((int64_t)b * s->Hq + h) * s->D;
        double *sc = (double *)malloc(sizeof(double) * (size_t)n);
        double m = -INFINITY;
        for (int t = 0; t < n; ++t) {
            int64_t page = block_table[(int64_t)b * s->MB + t / s->ps];
            int64_t koff = row_offset(s, block_table, b, g, t);
            double ks = (double)k_scale[page * s->Hkv + g], acc = 0.0;
            for (int d = 0; d < s->D; ++d)
                acc += widen(q, qoff + d, s->q_dtype) * (oracle_fp8_e4m3_decode(k_cache[koff + d]) * ks);
            sc[t] = (double)scale * acc;
            if (sc[t] > m) m = sc[t];
        }
        double l = 0.0;
        for (int t = 0; t < n; ++t) {
            double p = exp(sc[t] - m);
            l += p;
            int64_t page = block_table[(int64_t)b * s->MB + t / s->ps];
            int64_t voff = row_offset(s, block_table, b, g, t);
            double vs = (double)v_scale[page * s->Hkv + g];
            for (int d = 0; d < s->D; ++d) o[d] += p * (oracle_fp8_e4m3_decode(v_cache[voff + d]) * vs);
        }
        for (int d = 0; d < s->D; ++d) o[d] /= l;
        free(sc);
    }
    return used;
}

/*
 * Multi-token queries over the quantised cache: the chunk definition above (query i of request b at position
 * p = context_lens[b] - q_lens[b] + i attends to tokens 0 .. p), taken over the de-quantised rows
 * decode(byte) * scale[page, kv head].  `rows` as above.
 * Pins: one-token chunks equal oracle_paged_decode_attn_fp8; with power-of-two scales the result equals, bit for
 * bit, oracle_paged_prefill_attn on the de-quantised fp32 pools; general scales against a dense causal brute force.
 */
int oracle_paged_prefill_attn_fp8(const oracle_shape_t *s, const void *q, const uint8_t *k_cache, const uint8_t *v_cache,
                                  const float *k_scale, const float *v_scale, const int32_t *block_table,
                                  const int32_t *context_lens, const int32_t *q_lens, const int64_t *q_offsets,
                                  float scale, double *out, const int32_t *rows, int64_t nrows, int32_t num_threads)
{
    int G = s->Hq / s->Hkv;
    int64_t total = nrows;
    int64_t *first = NULL;
    if (!rows) {
        first = (int64_t *)malloc(sizeof(int64_t) * (size_t)(s->B + 1));
        first[0] = 0;
        for (int b = 0; b < s->B; ++b) first[b + 1] = first[b] + (q_lens[b] > 0 ? q_lens[b] : 0);
        total = first[s->B] * s->Hq;
    }
    int used = 1;
#ifdef _OPENMP
    if (num_threads > 0) omp_set_num_threads(num_threads);
    #pragma omp parallel
    {
        #pragma omp single
        used = omp_get_num_threads();
    }
    #pragma omp parallel for schedule(dynamic, 1)
#endif
    for (int64_t r = 0; r < total; ++r) {
        int b, i, h;
        if (rows) { b = rows[3 * r]; i = rows[3 * r + 1]; h = rows[3 * r + 2]; }
        else {
            int64_t row = r / s->Hq;
            h = (int)(r % s->Hq);
            b = 0;
            while (first[b + 1] <= row) ++b;
            i = (int)(row - first[b]);
        }
        int g = h / G;
        int n = context_lens[b] - q_lens[b] + i + 1;              /* tokens 0 .. p */
        int64_t qoff = ((q_offsets[b] + i) * s->Hq + h) * s->D;
        double *o = rows ? out + r * s->D : out + ((q_offsets[b] + i) * s->Hq + h) * s->D;
        for (int d = 0; d < s->D; ++d) o[d] = 0.0;
        if (n <= 0) continue;
        double *sc = (double *)malloc(sizeof(double) * (size_t)n);
        double m = -INFINITY;
        for (int t = 0; t < n; ++t) {
            int64_t page = block_table[(int64_t)b * s->MB + t / s->ps];
            int64_t koff = row_offset(s, block_table, b, g, t);
            double ks = (double)k_scale[page * s->Hkv + g], acc = 0.0;
            for (int d = 0; d < s->D; ++d)
                acc += widen(q, qoff + d, s->q_dtype) * (oracle_fp8_e4m3_decode(k_cache[koff + d]) * ks);
            sc[t] = (double)scale * acc;
            if (sc[t] > m) m = sc[t];
        }
        double l = 0.0;
        for (int t = 0; t < n; ++t) {
            double p = exp(sc[t] - m);
            l += p;
            int64_t page = block_table[(int64_t)b * s->MB + t / s->ps];
            int64_t voff = row_offset(s, block_table, b, g, t);
            double vs = (double)v_scale[page * s->Hkv + g];
            for (int d = 0; d < s->D; ++d) o[d] += p * (oracle_fp8_e4m3_decode(v_cache[voff + d]) * vs);
        }
        for (int d = 0; d < s->D; ++d) o[d] /= l;
        free(sc);
    }
    free(first);
    return used;
}


/*
 * Writing new rows into the quantised cache (the 8-bit form of oracle_kv_append; Section 2.2: the AR decoding loop adds
 * one token per request per iteration).  The paper names no quantisation rule; the one defined here:
 *   - the row that OPENS a page (slot 0) fixes the page's scale for that KV head:
 *         scale = max(amax * headroom, 2^-100) / 448        amax = largest |x| of the row, all in fp32
 *     (headroom >= 1 leaves room for later rows of the page; 448 is the largest finite E4M3 value);
 *   - every other row uses the scale its page already has;
 *   - byte = E4M3 code nearest to clamp(x / scale, -448, 448), ties to the even code; NaN gives the NaN byte 0x7f.
 * The quotient decides an integer code, so it is taken in the precision the GPU kernel uses: x (bf16, widened exactly)
 * and scale are fp32, the products and quotients above are single IEEE fp32 operations.
 * Pins: the encoder against the framework's own E4M3 cast on every representable value, every midpoint and random
 * values; hand-worked rounding cases (tests/golden/e4m3_rounding_cases.txt); decode(encode(v)) = v for all finite
 * codes; the append against a numpy brute force built on the framework's cast, with a whole-pool comparison.
 */
uint8_t oracle_fp8_e4m3_encode(float x)
{
    if (x != x) return 0x7f;
    uint8_t sign = signbit(x) ? 0x80 : 0x00;
    double a = fabs((double)x);
    if (a > 448.0) a = 448.0;
    int best = 0;
    double best_err = a;                                   /* code 0 stands for 0 */
    for (int code = 1; code <= 0x7e; ++code) {             /* the finite non-negative codes, ascending in value */
        double err = fabs(oracle_fp8_e4m3_decode((uint8_t)code) - a);
        if (err < best_err || (err == best_err && (code & 1) == 0)) { best = code; best_err = err; }
    }
    return (uint8_t)(sign | best);
}

void oracle_kv_append_quant_fp8(const oracle_shape_t *s, const uint16_t *k_new, const uint16_t *v_new, uint8_t *k_cache,
                                uint8_t *v_cache, float *k_scale, float *v_scale, const int32_t *block_table,
                                const int32_t *positions, float headroom)
{
    for (int which = 0; which < 2; ++which) {
        const uint16_t *src = which ? v_new : k_new;
        uint8_t *cache = which ? v_cache : k_cache;
        float *scales = which ? v_scale : k_scale;
        for (int b = 0; b < s->B; ++b) {
            int pos = positions[b];
            if (pos < 0) continue;
            int64_t page = block_table[(int64_t)b * s->MB + pos / s->ps];
            int slot = pos % s->ps;
            for (int g = 0; g < s->Hkv; ++g) {
                const uint16_t *row = src + ((int64_t)b * s->Hkv + g) * s->D;
                float sc;
                if (slot == 0) {
                    float amax = 0.0f;
                    for (int d = 0; d < s->D; ++d) {
                        float v = fabsf((float)widen(row, d, ORACLE_BF16));
                        if (v > amax) amax = v;                /* a NaN element never raises amax */
                    }
                    float top = amax * headroom;
                    if (!(top > 0x1p-100f)) top = 0x1p-100f;
                    sc = top / 448.0f;
                    scales[page * s->Hkv + g] = sc;
                } else {
                    sc = scales[page * s->Hkv + g];
                }
                uint8_t *dst = cache + (((page * s->Hkv + g) * s->ps) + slot) * (int64_t)s->D;
                for (int d = 0; d < s->D; ++d) {
                    float qv = (float)widen(row, d, ORACLE_BF16) / sc;
                    if (qv > 448.0f) qv = 448.0f;
                    if (qv < -448.0f) qv = -448.0f;
                    dst[d] = oracle_fp8_e4m3_encode(qv);
                }
            }
        }
    }
}
