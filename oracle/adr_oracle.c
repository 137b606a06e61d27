/*
 * adr_oracle.c -- plain fp64 CPU definition of batched decode attention over a
 * paged KV cache.  TEST INFRASTRUCTURE ONLY: the tests, the smoke check and the
 * CPU-baseline leg of the benchmark call it; the product library never does,
 * and the two share no code.
 *
 * What it follows.  The paper (Sec. 2.1, "Transformer Architecture" and
 * "Prefill and Decoding Phases") states the operation only in words: step (2)
 * of a transformer layer is the attention computation over the KV caches; the
 * caches hold the K and V of every earlier token of a request; a decode step
 * computes K and V for the one new token only and attends over everything
 * cached.  The attention executor of Sec. 3.1 / 3.2.1 keeps that cache in
 * "cache blocks" (pages) with per-request metadata (length).  The arithmetic
 * is therefore textbook scaled-dot-product softmax attention of ONE query
 * vector per head against the request's cached keys and values, written out
 * here as its definition:
 *
 *     s_t  = scale * <q, k_t>                 t = 0 .. L-1
 *     m    = max_t s_t
 *     w_t  = exp(s_t - m),   Z = sum_t w_t
 *     out  = (sum_t w_t v_t) / Z,   lse = m + ln Z
 *
 * Two passes over the gathered tokens, plain loops, no online softmax, no
 * tiling, no partitioning.  Grouped-query heads: q-head h reads kv-head
 * h / (Hq/Hkv).  Token t of request b lives in physical page
 * block_table[b][t / page_size] at slot t % page_size; cache layout is
 * [num_pages][page_size][Hkv][d] for K and for V.
 *
 * All inputs are widened exactly: bf16 -> fp64 is a bit shift; an fp8 byte
 * (OCP E4M3, finite-only variant) is decoded from the format's definition and
 * multiplied by its page's fp32 scale in fp64.  The softmax scale is the
 * fp32 number the caller passes, widened.
 *
 * Every function here is pinned by tests that do not go through this file's
 * own formulas (closed forms, a dense numpy brute force, a library attention
 * routine on tiny inputs, the split/merge identity, format tables).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_BF16 = 0, ORACLE_FP8_E4M3 = 1 };

/* ---- exact widening of stored element types --------------------------- */

static double bf16_to_f64(uint16_t bits)
{
    /* bf16 is the upper half of an IEEE binary32 */
    uint32_t u = (uint32_t)bits << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* OCP 8-bit float E4M3 (the finite-only "FN" flavour): 1 sign, 4 exponent
 * (bias 7), 3 mantissa bits.  Exponent field 0 is subnormal: m * 2^-9.
 * There is no infinity; S.1111.111 is NaN; largest finite is 1.75 * 2^8 = 448. */
double oracle_fp8_e4m3_decode(uint8_t byte)
{
    int sign = byte >> 7;
    int e = (byte >> 3) & 0xF;
    int m = byte & 0x7;
    double mag;
    if (e == 0xF && m == 0x7)
        return NAN;
    if (e == 0)
        mag = ldexp((double)m, -9);
    else
        mag = ldexp(1.0 + (double)m / 8.0, e - 7);
    return sign ? -mag : mag;
}

/* Round-to-nearest-even, saturating, of a real number to E4M3.  Written as a
 * search over the finite codes so that it shares nothing with any bit-trick
 * converter: the nearest representable magnitude wins, ties go to the code
 * with an even mantissa field, magnitudes beyond 448 clamp to 448. */
uint8_t oracle_fp8_e4m3_encode(double x)
{
    uint8_t sign = 0;
    int best = 0;
    double best_err;
    int c;
    if (isnan(x))
        return 0x7F;
    if (signbit(x)) {
        sign = 0x80;
        x = -x;
    }
    if (x >= 448.0)
        return (uint8_t)(sign | 0x7E);
    best_err = fabs(x - 0.0);
    for (c = 1; c <= 0x7E; ++c) {
        double err = fabs(x - oracle_fp8_e4m3_decode((uint8_t)c));
        if (err < best_err || (err == best_err && (c & 1) == 0)) {
            best_err = err;
            best = c;
        }
    }
    return (uint8_t)(sign | best);
}

typedef struct {
    const void *k, *v;                 /* [num_pages][page_size][Hkv][d] */
    const float *k_scale, *v_scale;    /* [num_pages][Hkv], fp8 only */
    int num_pages, page_size, Hkv, d, dtype;
} oracle_cache;

static double cache_elem(const void *base, const float *scales, const oracle_cache *c,
                         int64_t page, int slot, int head, int j)
{
    int64_t idx = (((int64_t)page * c->page_size + slot) * c->Hkv + head) * c->d + j;
    if (c->dtype == ORACLE_BF16)
        return bf16_to_f64(((const uint16_t *)base)[idx]);
    return oracle_fp8_e4m3_decode(((const uint8_t *)base)[idx]) *
           (double)scales[(int64_t)page * c->Hkv + head];
}

/* ---- attention for one (request, q-head) ------------------------------ */

/* Scores s_t for request row b, q-head h.  q is bf16 [B][Hq][d] with a row
 * stride (elements) between requests. */
static void scores_one(double *s, const oracle_cache *c, const uint16_t *q, int64_t q_row_stride,
                       const int32_t *block_table, int max_pages, int b, int h, int Hq, int L,
                       double scale)
{
    int G = Hq / c->Hkv;
    int kvh = h / G;
    const uint16_t *qv = q + (int64_t)b * q_row_stride + (int64_t)h * c->d;
    int t, j;
    for (t = 0; t < L; ++t) {
        int32_t page = block_table[(int64_t)b * max_pages + t / c->page_size];
        int slot = t % c->page_size;
        double dot = 0.0;
        for (j = 0; j < c->d; ++j)
            dot += bf16_to_f64(qv[j]) * cache_elem(c->k, c->k_scale, c, page, slot, kvh, j);
        s[t] = scale * dot;
    }
}

static void attend_one(double *out, double *lse, double *weights_or_null, double *s,
                       const oracle_cache *c, const uint16_t *q, int64_t q_row_stride,
                       const int32_t *block_table, int max_pages, int b, int h, int Hq, int L,
                       double scale)
{
    int G = Hq / c->Hkv;
    int kvh = h / G;
    int t, j;
    double m, Z;
    if (L <= 0) { /* a padded row attends nothing */
        for (j = 0; j < c->d; ++j)
            out[j] = 0.0;
        *lse = -INFINITY;
        return;
    }
    scores_one(s, c, q, q_row_stride, block_table, max_pages, b, h, Hq, L, scale);
    m = s[0];
    for (t = 1; t < L; ++t)
        if (s[t] > m)
            m = s[t];
    Z = 0.0;
    for (t = 0; t < L; ++t) {
        s[t] = exp(s[t] - m); /* s now holds w_t */
        Z += s[t];
    }
    for (j = 0; j < c->d; ++j)
        out[j] = 0.0;
    for (t = 0; t < L; ++t) {
        int32_t page = block_table[(int64_t)b * max_pages + t / c->page_size];
        int slot = t % c->page_size;
        for (j = 0; j < c->d; ++j)
            out[j] += s[t] * cache_elem(c->v, c->v_scale, c, page, slot, kvh, j);
    }
    for (j = 0; j < c->d; ++j)
        out[j] /= Z;
    *lse = m + log(Z);
    if (weights_or_null)
        for (t = 0; t < L; ++t)
            weights_or_null[t] = s[t] / Z;
}

/* out [B][Hq][d] fp64, lse [B][Hq] fp64 (natural log).  Rows listed in
 * row_subset (n_rows of them) are computed; NULL means all B rows.  Returns
 * the number of threads used, or a negative number on a bad argument. */
int oracle_decode_attention(double *out, double *lse, const uint16_t *q, int64_t q_row_stride,
                            const oracle_cache *c, const int32_t *block_table, int max_pages,
                            const int32_t *seq_lens, int B, int Hq, float scale,
                            const int32_t *row_subset, int n_rows, int num_threads)
{
    int max_L = 0, r, used = 1;
    int64_t item, n_items;
    if (!out || !lse || !q || !c || !block_table || !seq_lens || Hq % c->Hkv != 0)
        return -1;
    if (!row_subset)
        n_rows = B;
    for (r = 0; r < n_rows; ++r) {
        int b = row_subset ? row_subset[r] : r;
        if (b < 0 || b >= B)
            return -2;
        if (seq_lens[b] > max_L)
            max_L = seq_lens[b];
        if (seq_lens[b] > (int64_t)max_pages * c->page_size)
            return -3;
    }
    n_items = (int64_t)n_rows * Hq;
#ifdef _OPENMP
    if (num_threads > 0)
        omp_set_num_threads(num_threads);
#pragma omp parallel
#endif
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)(max_L > 0 ? max_L : 1));
#ifdef _OPENMP
#pragma omp single
        used = omp_get_num_threads();
#pragma omp for schedule(dynamic, 1)
#endif
        for (item = 0; item < n_items; ++item) {
            int b = row_subset ? row_subset[item / Hq] : (int)(item / Hq);
            int h = (int)(item % Hq);
            attend_one(out + ((int64_t)b * Hq + h) * c->d, lse + (int64_t)b * Hq + h, NULL, s, c, q,
                       q_row_stride, block_table, max_pages, b, h, Hq, seq_lens[b], (double)scale);
        }
        free(s);
    }
    return used;
}

/* Softmax weights w_t / Z of one (request, q-head): weights[0 .. seq_lens[b]). */
int oracle_attention_weights(double *weights, const uint16_t *q, int64_t q_row_stride,
                             const oracle_cache *c, const int32_t *block_table, int max_pages,
                             const int32_t *seq_lens, int Hq, float scale, int b, int h)
{
    int L = seq_lens[b];
    double *s = (double *)malloc(sizeof(double) * (size_t)(L > 0 ? L : 1));
    double *o = (double *)malloc(sizeof(double) * (size_t)c->d);
    double lse;
    attend_one(o, &lse, weights, s, c, q, q_row_stride, block_table, max_pages, b, h, Hq, L,
               (double)scale);
    free(s);
    free(o);
    return 0;
}

/* ---- append ------------------------------------------------------------ */

/* The decode step's new token: request b's K and V vectors (all kv-heads) are
 * stored at token index positions[b] of that request, i.e. page
 * block_table[b][pos / page_size], slot pos % page_size.  positions[b] < 0
 * skips the row.  bf16 cache: a bit-for-bit copy.  k_new/v_new are bf16
 * [B][Hkv][d] with a row stride in elements.  Returns 0, or negative when a
 * position falls outside the row's block table or names a page outside the pool. */
int oracle_kv_append_bf16(uint16_t *K, uint16_t *V, int num_pages, int page_size, int Hkv, int d,
                          const uint16_t *k_new, const uint16_t *v_new, int64_t new_row_stride,
                          const int32_t *block_table, int max_pages, const int32_t *positions,
                          int B)
{
    int b, h, j;
    for (b = 0; b < B; ++b) {
        int pos = positions[b];
        int32_t page;
        int slot;
        if (pos < 0)
            continue;
        if (pos / page_size >= max_pages)
            return -1;
        page = block_table[(int64_t)b * max_pages + pos / page_size];
        slot = pos % page_size;
        if (page < 0 || page >= num_pages)
            return -2;
        for (h = 0; h < Hkv; ++h)
            for (j = 0; j < d; ++j) {
                int64_t dst = (((int64_t)page * page_size + slot) * Hkv + h) * d + j;
                int64_t src = (int64_t)b * new_row_stride + (int64_t)h * d + j;
                K[dst] = k_new[src];
                V[dst] = v_new[src];
            }
    }
    return 0;
}

/* fp8 cache with one fp32 scale per (page, kv-head), separately for K and V.
 * The rule (this build's own reading; the paper has no fp8 cache): the token
 * that lands in slot 0 of a page fixes that page's scale to
 * 2 * amax(token, head) / 448 (amax over the d elements, floor 2^-20 on amax so a zero vector still gets a usable scale);
 * later slots reuse the stored scale.  Each element is stored as
 * encode(x / scale) with round-to-nearest-even and saturation, the division
 * carried out in fp32 as the product x * (1/scale) with 1/scale rounded to
 * fp32 once -- the precision the GPU path uses -- so the byte is decided by
 * the same number on both sides. */
static void append_fp8_one(uint8_t *C, float *S, int page, int slot, int page_size, int Hkv, int d,
                           const uint16_t *src_row)
{
    int h, j;
    for (h = 0; h < Hkv; ++h) {
        float scale, inv;
        if (slot == 0) {
            float amax = 0.0f;
            for (j = 0; j < d; ++j) {
                float a = fabsf((float)bf16_to_f64(src_row[h * d + j]));
                if (a > amax)
                    amax = a;
            }
            if (amax < 9.5367431640625e-07f) /* 2^-20 */
                amax = 9.5367431640625e-07f;
            scale = amax * (2.0f / 448.0f);
            S[(int64_t)page * Hkv + h] = scale;
        } else {
            scale = S[(int64_t)page * Hkv + h];
        }
        inv = 1.0f / scale;
        for (j = 0; j < d; ++j) {
            float x = (float)bf16_to_f64(src_row[h * d + j]);
            float y = x * inv; /* fp32 product, one rounding */
            C[(((int64_t)page * page_size + slot) * Hkv + h) * d + j] =
                oracle_fp8_e4m3_encode((double)y);
        }
    }
}

int oracle_kv_append_fp8(uint8_t *K, uint8_t *V, float *k_scale, float *v_scale, int num_pages,
                         int page_size, int Hkv, int d, const uint16_t *k_new,
                         const uint16_t *v_new, int64_t new_row_stride, const int32_t *block_table,
                         int max_pages, const int32_t *positions, int B)
{
    int b;
    for (b = 0; b < B; ++b) {
        int pos = positions[b];
        int32_t page;
        if (pos < 0)
            continue;
        if (pos / page_size >= max_pages)
            return -1;
        page = block_table[(int64_t)b * max_pages + pos / page_size];
        if (page < 0 || page >= num_pages)
            return -2;
        append_fp8_one(K, k_scale, page, pos % page_size, page_size, Hkv, d,
                       k_new + (int64_t)b * new_row_stride);
        append_fp8_one(V, v_scale, page, pos % page_size, page_size, Hkv, d,
                       v_new + (int64_t)b * new_row_stride);
    }
    return 0;
}

/* ---- combining partitions ---------------------------------------------- */

/* If a request's tokens are cut into disjoint partitions p and each partition
 * reports its own normalised attention output o_p and its own log-sum-exp
 * lse_p = m_p + ln Z_p, the attention over the union is
 *     lse = ln sum_p exp(lse_p),   out = sum_p exp(lse_p - lse) * o_p
 * (each partition's share of the total softmax mass times its own average).
 * part_o [total_parts][heads][d], part_lse [total_parts][heads], request b
 * owns partitions [part_offsets[b], part_offsets[b+1]).  A partition with
 * lse = -inf carries no mass.  A request with no mass at all gives zeros and
 * lse = -inf. */
int oracle_lse_merge(double *out, double *lse_out, const double *part_o, const double *part_lse,
                     const int32_t *part_offsets, int B, int heads, int d)
{
    int b, h, j, p;
    for (b = 0; b < B; ++b)
        for (h = 0; h < heads; ++h) {
            double top = -INFINITY, total = 0.0, lse;
            double *o = out + ((int64_t)b * heads + h) * d;
            for (j = 0; j < d; ++j)
                o[j] = 0.0;
            for (p = part_offsets[b]; p < part_offsets[b + 1]; ++p)
                if (part_lse[(int64_t)p * heads + h] > top)
                    top = part_lse[(int64_t)p * heads + h];
            if (top == -INFINITY) {
                if (lse_out)
                    lse_out[(int64_t)b * heads + h] = -INFINITY;
                continue;
            }
            for (p = part_offsets[b]; p < part_offsets[b + 1]; ++p)
                total += exp(part_lse[(int64_t)p * heads + h] - top);
            lse = top + log(total);
            for (p = part_offsets[b]; p < part_offsets[b + 1]; ++p) {
                double share = exp(part_lse[(int64_t)p * heads + h] - lse);
                const double *po = part_o + ((int64_t)p * heads + h) * d;
                if (share == 0.0)
                    continue; /* also keeps a -inf partition's payload (possibly NaN) out */
                for (j = 0; j < d; ++j)
                    o[j] += share * po[j];
            }
            if (lse_out)
                lse_out[(int64_t)b * heads + h] = lse;
        }
    return 0;
}

int oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
