/*
 * ta_oracle.c -- reference oracle for attention over a paged KV cache.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It exists so that the GPU
 * library can be checked against something plain, slow and obviously correct.
 * Nothing in the product path may call it; it shares no code, header, table or
 * helper with the HIP sources.
 *
 * What it computes.  The paper (ThunderAgent, Sec. 2.1, 4.2 and 4.3) describes
 * multi-turn agent programs whose context c_{t+1} extends c_t as a prefix, so
 * the backend keeps each program's KV cache, decodes against it, prefills only
 * the new tool-output tokens (the incremental-prefill term of the cost
 * decomposition, Eq. 3) and, after a Pause has released a program's KV cache
 * (Sec. 4.3, Eq. 5), must bring the pages back when it is Restored (Eq. 4;
 * the offloading variant is discussed in App. A.2).  The paper treats these
 * as black-box backend operations; what they compute is standard
 * scaled-dot-product attention,
 *
 *      out = softmax(q K^T * scale) V,
 *
 * taken over the cached tokens of one program, where token j of program b
 * lives in physical page block_table[b][j / page_size], row j % page_size.
 * The oracle is that definition written out token by token in fp64 with a
 * two-pass softmax (max, then exp and sum, then normalise).  There is no
 * blocking, no online rescaling, no split over the key axis.
 *
 * Readings where the paper is silent:
 *   - grouped-query attention: query head h reads kv head h / (Hq / Hkv);
 *   - context_lens[b] counts every cached token including the newest one;
 *   - append-prefill: new token i (0-based) of a program with n new tokens and
 *     L cached tokens in total sees keys 0 .. (L - n) + i, itself included;
 *   - rows of the last page beyond the context length are never read;
 *   - a row with zero visible keys has output 0 and lse = -inf;
 *   - lse is the natural-log sum: max + ln(sum exp(s - max)).
 *
 * All bf16 inputs are widened exactly to fp64.  Element type of q and the
 * pools is uint16_t holding the bf16 bit pattern.
 *
 * FP8 KV cache (the paper serves its large models in FP8, Sec. 5.1; it says nothing
 * about the cache format, so this is a reading): keys and values may be stored
 * as 8-bit codes in the OCP "E4M3" format (1 sign, 4 exponent bits with bias 7,
 * 3 mantissa bits; no infinities; S.1111.111 is NaN; exponent field 0 holds the
 * subnormals m * 2^-9; largest finite value 448) together with one fp32 scale
 * for all keys and one for all values of the call.  The cached key is
 * code_value * k_scale, the cached value code_value * v_scale, both exact in
 * fp64, and attention over them is the same definition as above.  Queries
 * stay bf16.
 * Writing such a cache (the new tokens of a program arrive as bf16 rows): the
 * code of an element x is the E4M3 value nearest to x / scale, the quotient
 * taken in fp32 as the GPU takes it (x is exact in fp32), ties going to the
 * code whose mantissa is even; a quotient beyond the largest value becomes
 * +-448 (a cache must never acquire a NaN the model did not produce), NaN
 * stays NaN, and the sign of zero is kept.  Written below as that definition:
 * a search over all finite codes for the nearest value.
 *
 * Every function here is pinned by tests that compare it with an independent
 * numpy evaluation on contiguous arrays, closed forms (single key, equal keys,
 * two keys = logistic), invariants (probabilities sum to one, page permutation,
 * key shift) and a brute-force sweep of boundary sizes.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int32_t num_q_heads;
    int32_t num_kv_heads;
    int32_t head_dim;
    int32_t page_size;
    double scale;         /* multiplies q.k; caller passes 1/sqrt(head_dim) */
    int64_t stride_page;  /* pool strides in elements; head_dim is contiguous */
    int64_t stride_head;
    int64_t stride_token;
} oracle_geom;

static double widen_bf16(uint16_t bits)
{
    uint32_t u = ((uint32_t)bits) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

static const uint16_t *token_row(const oracle_geom *ge, const uint16_t *pool,
                                 const int32_t *table_row, int32_t kv_head, int64_t j)
{
    int64_t page = table_row[j / ge->page_size];
    int64_t row = j % ge->page_size;
    return pool + page * ge->stride_page + (int64_t)kv_head * ge->stride_head + row * ge->stride_token;
}

/*
 * One output row: query vector q (head_dim bf16 values) of query head h of a
 * program whose block-table row is table_row, attending keys 0 .. visible-1.
 * weights must hold `visible` doubles; on return it holds the softmax
 * probabilities p_j.  out holds head_dim doubles.
 */
static void attend_row(const oracle_geom *ge, const uint16_t *q, int32_t h,
                       const uint16_t *k_pool, const uint16_t *v_pool,
                       const int32_t *table_row, int64_t visible,
                       double *weights, double *out, double *lse)
{
    const int32_t d = ge->head_dim;
    const int32_t group = ge->num_q_heads / ge->num_kv_heads;
    const int32_t g = h / group;

    for (int32_t c = 0; c < d; ++c) out[c] = 0.0;
    if (visible <= 0) {
        *lse = -INFINITY;
        return;
    }
    /* scores s_j = scale * <q, k_j> */
    double top = -INFINITY;
    for (int64_t j = 0; j < visible; ++j) {
        const uint16_t *k = token_row(ge, k_pool, table_row, g, j);
        double dot = 0.0;
        for (int32_t c = 0; c < d; ++c) dot += widen_bf16(q[c]) * widen_bf16(k[c]);
        weights[j] = dot * ge->scale;
        if (weights[j] > top) top = weights[j];
    }
    /* softmax, two passes */
    double total = 0.0;
    for (int64_t j = 0; j < visible; ++j) {
        weights[j] = exp(weights[j] - top);
        total += weights[j];
    }
    for (int64_t j = 0; j < visible; ++j) weights[j] /= total;
    /* out = sum_j p_j v_j */
    for (int64_t j = 0; j < visible; ++j) {
        const uint16_t *v = token_row(ge, v_pool, table_row, g, j);
        const double p = weights[j];
        for (int32_t c = 0; c < d; ++c) out[c] += p * widen_bf16(v[c]);
    }
    *lse = top + log(total);
}

/* Value of an OCP E4M3 code (see the header): exact in fp64. */
static double widen_e4m3(uint8_t code)
{
    const int sign = code >> 7;
    const int exponent = (code >> 3) & 15;
    const int mantissa = code & 7;
    double magnitude;
    if (exponent == 15 && mantissa == 7) return NAN;
    if (exponent == 0)
        magnitude = ldexp((double)mantissa, -9);               /* subnormal: (m / 8) * 2^(1 - 7) */
    else
        magnitude = ldexp(1.0 + (double)mantissa / 8.0, exponent - 7);
    return sign ? -magnitude : magnitude;
}

/* The values of n codes, for checking the format against its specification. */
void ta_oracle_widen_e4m3(const uint8_t *codes, int64_t n, double *values)
{
    for (int64_t i = 0; i < n; ++i) values[i] = widen_e4m3(codes[i]);
}

/*
 * The E4M3 code nearest to q (see the header): a search over the 127 positive
 * finite codes 0x00 .. 0x7e for the smallest distance, exact in fp64; of two
 * codes at the same distance the even one wins (adjacent codes alternate in
 * parity, also across a change of exponent).
 */
static uint8_t quantise_e4m3(float q)
{
    const uint8_t sign = signbit(q) ? 0x80 : 0x00;
    if (isnan(q)) return (uint8_t)(sign | 0x7f);
    const double a = fabs((double)q);
    if (a >= 448.0) return (uint8_t)(sign | 0x7e);             /* beyond the largest value: saturate */
    int best = 0;
    double best_dist = a;                                      /* distance to code 0 */
    for (int code = 1; code <= 0x7e; ++code) {
        const double dist = fabs(a - widen_e4m3((uint8_t)code));
        if (dist < best_dist || (dist == best_dist && (code & 1) == 0)) {
            best = code;
            best_dist = dist;
        }
    }
    return (uint8_t)(sign | best);
}

/* Codes of n values x[i] / scale (x given as fp32, the division in fp32). */
void ta_oracle_quantise_e4m3(const float *x, int64_t n, float scale, uint8_t *codes)
{
    for (int64_t i = 0; i < n; ++i) {
        const volatile float q = x[i] / scale;                 /* rounded to fp32 here, not kept wider */
        codes[i] = quantise_e4m3(q);
    }
}

/*
 * attend_row for an FP8 cache: the same steps, with keys and values read as
 * E4M3 codes times their scale.  Pools are uint8_t, strides in elements.
 */
static void attend_row_fp8(const oracle_geom *ge, const uint16_t *q, int32_t h,
                           const uint8_t *k_pool, const uint8_t *v_pool, double k_scale, double v_scale,
                           const int32_t *table_row, int64_t visible,
                           double *weights, double *out, double *lse)
{
    const int32_t d = ge->head_dim;
    const int32_t group = ge->num_q_heads / ge->num_kv_heads;
    const int32_t g = h / group;

    for (int32_t c = 0; c < d; ++c) out[c] = 0.0;
    if (visible <= 0) {
        *lse = -INFINITY;
        return;
    }
    double top = -INFINITY;
    for (int64_t j = 0; j < visible; ++j) {
        const int64_t page = table_row[j / ge->page_size], row = j % ge->page_size;
        const uint8_t *k = k_pool + page * ge->stride_page + (int64_t)g * ge->stride_head + row * ge->stride_token;
        double dot = 0.0;
        for (int32_t c = 0; c < d; ++c) dot += widen_bf16(q[c]) * (widen_e4m3(k[c]) * k_scale);
        weights[j] = dot * ge->scale;
        if (weights[j] > top) top = weights[j];
    }
    double total = 0.0;
    for (int64_t j = 0; j < visible; ++j) {
        weights[j] = exp(weights[j] - top);
        total += weights[j];
    }
    for (int64_t j = 0; j < visible; ++j) weights[j] /= total;
    for (int64_t j = 0; j < visible; ++j) {
        const int64_t page = table_row[j / ge->page_size], row = j % ge->page_size;
        const uint8_t *v = v_pool + page * ge->stride_page + (int64_t)g * ge->stride_head + row * ge->stride_token;
        const double p = weights[j];
        for (int32_t c = 0; c < d; ++c) out[c] += p * (widen_e4m3(v[c]) * v_scale);
    }
    *lse = top + log(total);
}

/*
 * Decode over an FP8 cache: as ta_oracle_paged_decode, with
 *   k_pool, v_pool  uint8 E4M3 codes, layout per ge (strides in elements)
 *   k_scale, v_scale  the fp32 scales of the call, widened by the caller
 */
void ta_oracle_paged_decode_fp8(const oracle_geom *ge, const uint16_t *q,
                                const uint8_t *k_pool, const uint8_t *v_pool, double k_scale, double v_scale,
                                const int32_t *block_table, int64_t table_stride,
                                const int32_t *context_lens, int32_t batch,
                                double *out, double *lse)
{
    const int32_t Hq = ge->num_q_heads, d = ge->head_dim;
    int64_t longest = 1;
    for (int32_t b = 0; b < batch; ++b)
        if (context_lens[b] > longest) longest = context_lens[b];
    const int64_t rows = (int64_t)batch * Hq;
#pragma omp parallel
    {
        double *weights = (double *)malloc((size_t)longest * sizeof(double));
#pragma omp for schedule(dynamic, 1)
        for (int64_t r = 0; r < rows; ++r) {
            const int32_t b = (int32_t)(r / Hq), h = (int32_t)(r % Hq);
            attend_row_fp8(ge, q + r * d, h, k_pool, v_pool, k_scale, v_scale,
                           block_table + (int64_t)b * table_stride, context_lens[b], weights,
                           out + r * d, lse + r);
        }
        free(weights);
    }
}

int ta_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * Decode: one query token per program.
 *   q            bf16 [batch][Hq][d]
 *   block_table  int32 [batch][table_stride]
 *   context_lens int32 [batch]
 *   out          f64  [batch][Hq][d]
 *   lse          f64  [batch][Hq]
 */
void ta_oracle_paged_decode(const oracle_geom *ge, const uint16_t *q,
                            const uint16_t *k_pool, const uint16_t *v_pool,
                            const int32_t *block_table, int64_t table_stride,
                            const int32_t *context_lens, int32_t batch,
                            double *out, double *lse)
{
    const int32_t Hq = ge->num_q_heads, d = ge->head_dim;
    int64_t longest = 1;
    for (int32_t b = 0; b < batch; ++b)
        if (context_lens[b] > longest) longest = context_lens[b];
    const int64_t rows = (int64_t)batch * Hq;
#pragma omp parallel
    {
        double *weights = (double *)malloc((size_t)longest * sizeof(double));
#pragma omp for schedule(dynamic, 1)
        for (int64_t r = 0; r < rows; ++r) {
            const int32_t b = (int32_t)(r / Hq), h = (int32_t)(r % Hq);
            attend_row(ge, q + r * d, h, k_pool, v_pool, block_table + (int64_t)b * table_stride,
                       context_lens[b], weights, out + r * d, lse + r);
        }
        free(weights);
    }
}

/*
 * Append-prefill: program b contributes n_b = cu_q_lens[b+1] - cu_q_lens[b]
 * query tokens, packed back to back; their keys and values already sit in the
 * pages (context_lens[b] = prefix + n_b).  New token i sees
 * context_lens[b] - n_b + i + 1 keys.
 *   q    bf16 [total_q][Hq][d]
 *   out  f64  [total_q][Hq][d]
 *   lse  f64  [total_q][Hq]
 */
void ta_oracle_append_prefill(const oracle_geom *ge, const uint16_t *q,
                              const int32_t *cu_q_lens,
                              const uint16_t *k_pool, const uint16_t *v_pool,
                              const int32_t *block_table, int64_t table_stride,
                              const int32_t *context_lens, int32_t batch,
                              double *out, double *lse)
{
    const int32_t Hq = ge->num_q_heads, d = ge->head_dim;
    int64_t longest = 1;
    for (int32_t b = 0; b < batch; ++b)
        if (context_lens[b] > longest) longest = context_lens[b];
    const int64_t total_q = batch > 0 ? cu_q_lens[batch] : 0;
    /* program of each packed token */
    int32_t *owner = (int32_t *)malloc((size_t)(total_q > 0 ? total_q : 1) * sizeof(int32_t));
    for (int32_t b = 0; b < batch; ++b)
        for (int64_t t = cu_q_lens[b]; t < cu_q_lens[b + 1]; ++t) owner[t] = b;
    const int64_t rows = total_q * Hq;
#pragma omp parallel
    {
        double *weights = (double *)malloc((size_t)longest * sizeof(double));
#pragma omp for schedule(dynamic, 1)
        for (int64_t r = 0; r < rows; ++r) {
            const int64_t t = r / Hq;
            const int32_t h = (int32_t)(r % Hq);
            const int32_t b = owner[t];
            const int64_t n = cu_q_lens[b + 1] - cu_q_lens[b];
            const int64_t i = t - cu_q_lens[b];
            const int64_t visible = (int64_t)context_lens[b] - n + i + 1;
            attend_row(ge, q + r * d, h, k_pool, v_pool, block_table + (int64_t)b * table_stride,
                       visible, weights, out + r * d, lse + r);
        }
        free(weights);
    }
    free(owner);
}

/*
 * Append-prefill over an FP8 cache: as ta_oracle_append_prefill, the keys and values (the new
 * tokens' own included: they were quantised when they were appended) read as E4M3 codes times
 * their scale, as in ta_oracle_paged_decode_fp8.
 */
void ta_oracle_append_prefill_fp8(const oracle_geom *ge, const uint16_t *q, const int32_t *cu_q_lens,
                                  const uint8_t *k_pool, const uint8_t *v_pool, double k_scale, double v_scale,
                                  const int32_t *block_table, int64_t table_stride,
                                  const int32_t *context_lens, int32_t batch, double *out, double *lse)
{
    const int32_t Hq = ge->num_q_heads, d = ge->head_dim;
    int64_t longest = 1;
    for (int32_t b = 0; b < batch; ++b)
        if (context_lens[b] > longest) longest = context_lens[b];
    const int64_t total_q = batch > 0 ? cu_q_lens[batch] : 0;
    int32_t *owner = (int32_t *)malloc((size_t)(total_q > 0 ? total_q : 1) * sizeof(int32_t));
    for (int32_t b = 0; b < batch; ++b)
        for (int64_t t = cu_q_lens[b]; t < cu_q_lens[b + 1]; ++t) owner[t] = b;
    const int64_t rows = total_q * Hq;
#pragma omp parallel
    {
        double *weights = (double *)malloc((size_t)longest * sizeof(double));
#pragma omp for schedule(dynamic, 1)
        for (int64_t r = 0; r < rows; ++r) {
            const int64_t t = r / Hq;
            const int32_t h = (int32_t)(r % Hq);
            const int32_t b = owner[t];
            const int64_t n = cu_q_lens[b + 1] - cu_q_lens[b];
            const int64_t i = t - cu_q_lens[b];
            const int64_t visible = (int64_t)context_lens[b] - n + i + 1;
            attend_row_fp8(ge, q + r * d, h, k_pool, v_pool, k_scale, v_scale,
                           block_table + (int64_t)b * table_stride, visible, weights, out + r * d, lse + r);
        }
        free(weights);
    }
    free(owner);
}

/*
 * Selected rows only (for checking sampled outputs of a large workload).
 * Row r is (program row_b[r], packed query token row_t[r], query head row_h[r])
 * and sees row_visible[r] keys.  q is the full packed bf16 [.][Hq][d] array.
 *   out f64 [n_rows][d], lse f64 [n_rows]
 */
void ta_oracle_attend_rows(const oracle_geom *ge, const uint16_t *q,
                           const uint16_t *k_pool, const uint16_t *v_pool,
                           const int32_t *block_table, int64_t table_stride,
                           int64_t n_rows, const int32_t *row_b, const int64_t *row_t,
                           const int32_t *row_h, const int64_t *row_visible,
                           double *out, double *lse)
{
    const int32_t Hq = ge->num_q_heads, d = ge->head_dim;
    int64_t longest = 1;
    for (int64_t r = 0; r < n_rows; ++r)
        if (row_visible[r] > longest) longest = row_visible[r];
#pragma omp parallel
    {
        double *weights = (double *)malloc((size_t)longest * sizeof(double));
#pragma omp for schedule(dynamic, 1)
        for (int64_t r = 0; r < n_rows; ++r) {
            const uint16_t *qr = q + (row_t[r] * Hq + row_h[r]) * d;
            attend_row(ge, qr, row_h[r], k_pool, v_pool,
                       block_table + (int64_t)row_b[r] * table_stride, row_visible[r],
                       weights, out + r * d, lse + r);
        }
        free(weights);
    }
}

/*
 * Softmax probabilities of one row, for checking that they are non-negative
 * and sum to one.  probs must hold `visible` doubles.
 */
void ta_oracle_row_probs(const oracle_geom *ge, const uint16_t *q_row, int32_t h,
                         const uint16_t *k_pool, const uint16_t *v_pool,
                         const int32_t *table_row, int64_t visible,
                         double *probs, double *out, double *lse)
{
    attend_row(ge, q_row, h, k_pool, v_pool, table_row, visible, probs, out, lse);
}

/*
 * KV page restore (the device-side consequence of the paper's Restore after a
 * Pause, Sec. 4.3, Eq. 4-5): pool[dst_slots[i]] = host[i] for K and for V, bytes only.
 * Returns 0, or -1 when a slot is out of range or named twice (nothing is
 * written in that case).
 */
int ta_oracle_kv_page_restore(uint8_t *k_pool, uint8_t *v_pool, int64_t page_bytes,
                              const uint8_t *host_k, const uint8_t *host_v,
                              const int32_t *dst_slots, int32_t n_pages, int32_t pool_pages)
{
    if (n_pages < 0 || pool_pages < 0 || page_bytes < 0) return -1;
    uint8_t *seen = (uint8_t *)calloc((size_t)(pool_pages > 0 ? pool_pages : 1), 1);
    for (int32_t i = 0; i < n_pages; ++i) {
        const int32_t s = dst_slots[i];
        if (s < 0 || s >= pool_pages || seen[s]) {
            free(seen);
            return -1;
        }
        seen[s] = 1;
    }
    free(seen);
    for (int32_t i = 0; i < n_pages; ++i) {
        memcpy(k_pool + (int64_t)dst_slots[i] * page_bytes, host_k + (int64_t)i * page_bytes, (size_t)page_bytes);
        memcpy(v_pool + (int64_t)dst_slots[i] * page_bytes, host_v + (int64_t)i * page_bytes, (size_t)page_bytes);
    }
    return 0;
}

/*
 * KV page evict (the device-side consequence of the paper's Pause, Sec. 4.3:
 * a paused program's KV cache leaves the pool; App. A.2 and A.4 keep it in host
 * memory): host[i] = pool[src_slots[i]] for K and for V, bytes only.  The pool
 * is not modified.  A slot may be named more than once.  Returns 0, or -1 when
 * a slot is out of range (nothing is written in that case).
 */
int ta_oracle_kv_page_evict(const uint8_t *k_pool, const uint8_t *v_pool, int64_t page_bytes,
                            uint8_t *host_k, uint8_t *host_v,
                            const int32_t *src_slots, int32_t n_pages, int32_t pool_pages)
{
    if (n_pages < 0 || pool_pages < 0 || page_bytes < 0) return -1;
    for (int32_t i = 0; i < n_pages; ++i)
        if (src_slots[i] < 0 || src_slots[i] >= pool_pages) return -1;
    for (int32_t i = 0; i < n_pages; ++i) {
        memcpy(host_k + (int64_t)i * page_bytes, k_pool + (int64_t)src_slots[i] * page_bytes, (size_t)page_bytes);
        memcpy(host_v + (int64_t)i * page_bytes, v_pool + (int64_t)src_slots[i] * page_bytes, (size_t)page_bytes);
    }
    return 0;
}

/*
 * KV append (Sec. 2.1: the context c_{t+1} extends c_t, so the cache of a
 * program grows at its tail; Sec. 4.2: the new tokens are the ones an
 * incremental prefill or a decode step attends from).  Program b's n_b new
 * tokens, n_b = cu_new[b + 1] - cu_new[b], become its tokens
 * context_lens[b] - n_b ... context_lens[b] - 1 (context_lens counts them
 * already): row (cu_new[b] + i) of new_k / new_v, laid out [token][Hkv][d], is
 * written to the pool at the place the block table gives token
 * context_lens[b] - n_b + i.  Bit patterns are copied; nothing else changes.
 */
void ta_oracle_kv_append(const oracle_geom *ge, const uint16_t *new_k, const uint16_t *new_v,
                         const int32_t *cu_new, uint16_t *k_pool, uint16_t *v_pool,
                         const int32_t *block_table, int64_t table_stride,
                         const int32_t *context_lens, int32_t batch)
{
    const int64_t d = ge->head_dim, Hkv = ge->num_kv_heads, S = ge->page_size;
    for (int32_t b = 0; b < batch; ++b) {
        const int64_t n = cu_new[b + 1] - cu_new[b];
        const int64_t first = (int64_t)context_lens[b] - n;
        for (int64_t i = 0; i < n; ++i) {
            const int64_t token = first + i;
            const int64_t page = block_table[(int64_t)b * table_stride + token / S];
            const int64_t row = token % S;
            for (int64_t g = 0; g < Hkv; ++g) {
                const int64_t dst = page * ge->stride_page + g * ge->stride_head + row * ge->stride_token;
                const int64_t src = ((int64_t)(cu_new[b] + i) * Hkv + g) * d;
                for (int64_t c = 0; c < d; ++c) {
                    k_pool[dst + c] = new_k[src + c];
                    v_pool[dst + c] = new_v[src + c];
                }
            }
        }
    }
}

/*
 * The same for an FP8 cache: the new tokens' bf16 rows are quantised on the way in,
 * keys with k_scale and values with v_scale (pools uint8, strides in elements).
 */
void ta_oracle_kv_append_fp8(const oracle_geom *ge, const uint16_t *new_k, const uint16_t *new_v,
                             const int32_t *cu_new, uint8_t *k_pool, uint8_t *v_pool, float k_scale, float v_scale,
                             const int32_t *block_table, int64_t table_stride,
                             const int32_t *context_lens, int32_t batch)
{
    const int64_t d = ge->head_dim, Hkv = ge->num_kv_heads, S = ge->page_size;
    for (int32_t b = 0; b < batch; ++b) {
        const int64_t n = cu_new[b + 1] - cu_new[b];
        const int64_t first = (int64_t)context_lens[b] - n;
        for (int64_t i = 0; i < n; ++i) {
            const int64_t token = first + i;
            const int64_t page = block_table[(int64_t)b * table_stride + token / S];
            const int64_t row = token % S;
            for (int64_t g = 0; g < Hkv; ++g) {
                const int64_t dst = page * ge->stride_page + g * ge->stride_head + row * ge->stride_token;
                const int64_t src = ((int64_t)(cu_new[b] + i) * Hkv + g) * d;
                for (int64_t c = 0; c < d; ++c) {
                    const volatile float kq = (float)widen_bf16(new_k[src + c]) / k_scale;
                    const volatile float vq = (float)widen_bf16(new_v[src + c]) / v_scale;
                    k_pool[dst + c] = quantise_e4m3(kq);
                    v_pool[dst + c] = quantise_e4m3(vq);
                }
            }
        }
    }
}
