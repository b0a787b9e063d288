/*
 * CPU oracle for paged grouped-query attention with ALiBi biases.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the yardstick the GPU library is
 * compared against; nothing in the product path may call it.  It shares no
 * code, header, table or helper with the HIP kernels: its index arithmetic and
 * its fp16 / bf16 decoding are its own.
 *
 * It is the plain definition written out in fp64, because paging, grouping and
 * partitioning are re-organisations of the same sum, not approximations
 * (Section II on the key-value pair shared by a group; Section III-A on pages and blocks):
 *
 *   score      eq. (3):  s_j = scale * <q_h, k_j> + bias(i, j)
 *   bias       Section II, the ALiBi paragraph:
 *                        bias(i, j) = slope_h * (j - pos_i), linear in the
 *                        relative position of key j and query i
 *   softmax    eq. (4):  w_j = exp(s_j) / sum_j exp(s_j)
 *   output     Section III-A, paragraph after eq. (4): out = sum_j w_j v_j
 *   grouping   Section I / II: the G = Hq/Hkv query heads of a group share one
 *                        K/V head; head h reads KV head floor(h / G)
 *   cache      eq. (2), Alg. 1 (the cache-store step):
 *                        new tokens' K/V rows are appended to the paged cache
 *   causality  Alg. 1 (prompt branch): query i sees keys 0..pos_i only
 *
 * Readings taken where the text leaves a choice (all listed in the design
 * notes of the repository):
 *   - the bias is added after scaling the dot product and is not itself scaled;
 *   - the softmax is evaluated with the maximum subtracted (same value);
 *   - context_lens counts the token being decoded; a zero-length context
 *     yields an all-zero output row;
 *   - a negative slot means "padding token, skip".
 *
 * Parity pins: tests/test_oracle_pins.py (closed forms, library attention in
 * fp64, brute force, invariants, planted-mistake checks).  The unscaled-bias
 * reading and the head->group map for 1 < Hkv < Hq are conventions the paper
 * does not fix by any printed number: parity unpinned for those two choices
 * beyond agreement with the library routine's convention.
 *
 * Cache layout (both caches): [num_blocks][num_kv_heads][block_size][head_dim],
 * 2-byte elements, head_dim innermost.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F16 = 0, ORACLE_BF16 = 1 };

/* ---- exact widening of 2-byte floats to double ------------------------- */
static double widen_f16(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1F;
    int m = h & 0x3FF;
    double v;
    if (e == 0)
        v = ldexp((double)m, -24);                 /* zero and subnormals */
    else if (e == 31)
        v = m ? NAN : INFINITY;
    else
        v = ldexp((double)(m + 1024), e - 25);
    return sign ? -v : v;
}

static double widen_bf16(uint16_t h)
{
    uint32_t u = ((uint32_t)h) << 16;              /* bf16 is the top half of an fp32 */
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

static double widen(uint16_t h, int dtype)
{
    return dtype == ORACLE_F16 ? widen_f16(h) : widen_bf16(h);
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* ---- cache write: eq. (2), Alg. 1 (the cache-store step) -------------- */
void oracle_reshape_and_cache(const uint16_t *k, const uint16_t *v,
                              uint16_t *k_cache, uint16_t *v_cache,
                              const int64_t *slot_mapping,
                              int num_tokens, int num_kv_heads, int head_dim, int block_size,
                              int64_t k_token_stride, int64_t v_token_stride)
{
    for (int t = 0; t < num_tokens; ++t) {
        int64_t slot = slot_mapping[t];
        if (slot < 0) continue;                                   /* padding token */
        int64_t block = slot / block_size;
        int64_t row = slot % block_size;
        for (int g = 0; g < num_kv_heads; ++g) {
            int64_t dst = ((block * num_kv_heads + g) * block_size + row) * head_dim;
            for (int d = 0; d < head_dim; ++d) {
                k_cache[dst + d] = k[t * k_token_stride + (int64_t)g * head_dim + d];
                v_cache[dst + d] = v[t * v_token_stride + (int64_t)g * head_dim + d];
            }
        }
    }
}

/* ---- one query row against the first n_keys tokens of sequence b -------- */
static void attend_row(double *out_row, const uint16_t *q_row,
                       const uint16_t *k_cache, const uint16_t *v_cache,
                       const int32_t *table_row, int n_keys, int pos_q,
                       int kv_head, double slope, double scale,
                       int num_kv_heads, int head_dim, int block_size, int dtype)
{
    for (int d = 0; d < head_dim; ++d) out_row[d] = 0.0;
    if (n_keys <= 0) return;

    double *s = (double *)malloc(sizeof(double) * (size_t)n_keys);
    double m = -INFINITY;
    for (int j = 0; j < n_keys; ++j) {
        int64_t block = table_row[j / block_size];
        int64_t row = j % block_size;
        const uint16_t *k_j = k_cache + ((block * num_kv_heads + kv_head) * block_size + row) * head_dim;
        double dot = 0.0;
        for (int d = 0; d < head_dim; ++d)
            dot += widen(q_row[d], dtype) * widen(k_j[d], dtype);
        s[j] = scale * dot + slope * (double)(j - pos_q);         /* eq. (3) with the ALiBi bias */
        if (s[j] > m) m = s[j];
    }
    double denom = 0.0;
    for (int j = 0; j < n_keys; ++j) {                            /* eq. (4) */
        s[j] = exp(s[j] - m);
        denom += s[j];
    }
    for (int j = 0; j < n_keys; ++j) {                            /* weighted sum of V */
        int64_t block = table_row[j / block_size];
        int64_t row = j % block_size;
        const uint16_t *v_j = v_cache + ((block * num_kv_heads + kv_head) * block_size + row) * head_dim;
        double w = s[j] / denom;
        for (int d = 0; d < head_dim; ++d)
            out_row[d] += w * widen(v_j[d], dtype);
    }
    free(s);
}

/* ---- decode: one query token per sequence, all keys are in the past ----- */
void oracle_paged_attention(double *out,                 /* [B, Hq, D] fp64 */
                            const uint16_t *q,           /* [B, Hq, D] */
                            const uint16_t *k_cache, const uint16_t *v_cache,
                            const int32_t *block_tables, /* [B, max_blocks_per_seq] */
                            const int32_t *context_lens, /* [B] */
                            const float *alibi_slopes,   /* [Hq] or NULL */
                            float scale, int num_seqs, int num_heads, int num_kv_heads,
                            int head_dim, int block_size, int max_blocks_per_seq, int dtype)
{
    int group = num_heads / num_kv_heads;
    int units = num_seqs * num_heads;
#pragma omp parallel for schedule(dynamic, 1)
    for (int u = 0; u < units; ++u) {
        int b = u / num_heads, h = u % num_heads;
        int L = context_lens[b];
        double slope = alibi_slopes ? (double)alibi_slopes[h] : 0.0;
        attend_row(out + (int64_t)u * head_dim, q + (int64_t)u * head_dim, k_cache, v_cache,
                   block_tables + (int64_t)b * max_blocks_per_seq, L, L - 1, h / group,
                   slope, (double)scale, num_kv_heads, head_dim, block_size, dtype);
    }
}

/* Same as above for a chosen list of (sequence, head) pairs; out is [n_rows, D]. */
void oracle_paged_attention_rows(double *out, const int32_t *row_seq, const int32_t *row_head,
                                 int n_rows, const uint16_t *q,
                                 const uint16_t *k_cache, const uint16_t *v_cache,
                                 const int32_t *block_tables, const int32_t *context_lens,
                                 const float *alibi_slopes, float scale, int num_heads,
                                 int num_kv_heads, int head_dim, int block_size,
                                 int max_blocks_per_seq, int dtype)
{
    int group = num_heads / num_kv_heads;
#pragma omp parallel for schedule(dynamic, 1)
    for (int r = 0; r < n_rows; ++r) {
        int b = row_seq[r], h = row_head[r];
        int L = context_lens[b];
        double slope = alibi_slopes ? (double)alibi_slopes[h] : 0.0;
        attend_row(out + (int64_t)r * head_dim, q + ((int64_t)b * num_heads + h) * head_dim,
                   k_cache, v_cache, block_tables + (int64_t)b * max_blocks_per_seq, L, L - 1,
                   h / group, slope, (double)scale, num_kv_heads, head_dim, block_size, dtype);
    }
}

/* ---- split context: Section III-A (a block's result is kept and carried into the next
 * block's computation).  Each run of partition_size tokens
 * yields its own maximum m_p, sum l_p and normalised output o_p; they combine as
 *   m = max_p m_p,   out = sum_p e^{m_p-m} l_p o_p / sum_p e^{m_p-m} l_p,
 * which equals the unpartitioned result.  Written out literally so that the
 * identity can be tested; decode only. */
void oracle_paged_attention_partitioned(double *out, const uint16_t *q,
                                        const uint16_t *k_cache, const uint16_t *v_cache,
                                        const int32_t *block_tables, const int32_t *context_lens,
                                        const float *alibi_slopes, float scale, int num_seqs,
                                        int num_heads, int num_kv_heads, int head_dim,
                                        int block_size, int max_blocks_per_seq,
                                        int partition_size, int dtype)
{
    int group = num_heads / num_kv_heads;
    for (int b = 0; b < num_seqs; ++b)
        for (int h = 0; h < num_heads; ++h) {
            double *o = out + ((int64_t)b * num_heads + h) * head_dim;
            const uint16_t *q_row = q + ((int64_t)b * num_heads + h) * head_dim;
            const int32_t *table_row = block_tables + (int64_t)b * max_blocks_per_seq;
            int L = context_lens[b];
            int g = h / group;
            double slope = alibi_slopes ? (double)alibi_slopes[h] : 0.0;
            int n_part = (L + partition_size - 1) / partition_size;
            for (int d = 0; d < head_dim; ++d) o[d] = 0.0;
            if (n_part == 0) continue;
            double *m_p = (double *)malloc(sizeof(double) * n_part);
            double *l_p = (double *)malloc(sizeof(double) * n_part);
            double *o_p = (double *)calloc((size_t)n_part * head_dim, sizeof(double));
            for (int p = 0; p < n_part; ++p) {
                int j0 = p * partition_size;
                int j1 = j0 + partition_size < L ? j0 + partition_size : L;
                double *s = (double *)malloc(sizeof(double) * (j1 - j0));
                m_p[p] = -INFINITY;
                for (int j = j0; j < j1; ++j) {
                    int64_t block = table_row[j / block_size];
                    const uint16_t *k_j = k_cache + ((block * num_kv_heads + g) * block_size + j % block_size) * head_dim;
                    double dot = 0.0;
                    for (int d = 0; d < head_dim; ++d)
                        dot += widen(q_row[d], dtype) * widen(k_j[d], dtype);
                    s[j - j0] = (double)scale * dot + slope * (double)(j - (L - 1));
                    if (s[j - j0] > m_p[p]) m_p[p] = s[j - j0];
                }
                l_p[p] = 0.0;
                for (int j = j0; j < j1; ++j) {
                    int64_t block = table_row[j / block_size];
                    const uint16_t *v_j = v_cache + ((block * num_kv_heads + g) * block_size + j % block_size) * head_dim;
                    double e = exp(s[j - j0] - m_p[p]);
                    l_p[p] += e;
                    for (int d = 0; d < head_dim; ++d)
                        o_p[(int64_t)p * head_dim + d] += e * widen(v_j[d], dtype);
                }
                for (int d = 0; d < head_dim; ++d) o_p[(int64_t)p * head_dim + d] /= l_p[p];
                free(s);
            }
            double m = -INFINITY, denom = 0.0;
            for (int p = 0; p < n_part; ++p) if (m_p[p] > m) m = m_p[p];
            for (int p = 0; p < n_part; ++p) denom += exp(m_p[p] - m) * l_p[p];
            for (int p = 0; p < n_part; ++p) {
                double w = exp(m_p[p] - m) * l_p[p] / denom;
                for (int d = 0; d < head_dim; ++d) o[d] += w * o_p[(int64_t)p * head_dim + d];
            }
            free(m_p); free(l_p); free(o_p);
        }
}

/* ---- prefill over the paged cache: q_len new tokens per sequence, causal + ALiBi.
 * Query row i of sequence b sits at position pos = context_lens[b] - q_len_b + i and
 * sees keys 0..pos (Alg. 1 prompt branch; Section II on ALiBi). */
void oracle_paged_prefill(double *out,                   /* [T, Hq, D] fp64 */
                          const uint16_t *q,             /* [T, Hq, D] */
                          const uint16_t *k_cache, const uint16_t *v_cache,
                          const int32_t *block_tables, const int32_t *context_lens,
                          const int32_t *cu_q_lens,      /* [B+1] */
                          const float *alibi_slopes, float scale, int num_seqs, int num_heads,
                          int num_kv_heads, int head_dim, int block_size,
                          int max_blocks_per_seq, int dtype)
{
    int group = num_heads / num_kv_heads;
    int total = cu_q_lens[num_seqs];
    int units = total * num_heads;
#pragma omp parallel for schedule(dynamic, 4)
    for (int u = 0; u < units; ++u) {
        int t = u / num_heads, h = u % num_heads;
        int b = 0;
        while (cu_q_lens[b + 1] <= t) ++b;
        int q_len = cu_q_lens[b + 1] - cu_q_lens[b];
        int pos = context_lens[b] - q_len + (t - cu_q_lens[b]);
        double slope = alibi_slopes ? (double)alibi_slopes[h] : 0.0;
        attend_row(out + (int64_t)u * head_dim, q + (int64_t)u * head_dim, k_cache, v_cache,
                   block_tables + (int64_t)b * max_blocks_per_seq, pos + 1, pos, h / group,
                   slope, (double)scale, num_kv_heads, head_dim, block_size, dtype);
    }
}

/* Prefill for a chosen list of (query token, head) pairs; out is [n_rows, D]. */
void oracle_paged_prefill_rows(double *out, const int32_t *row_token, const int32_t *row_head,
                               int n_rows, const uint16_t *q,
                               const uint16_t *k_cache, const uint16_t *v_cache,
                               const int32_t *block_tables, const int32_t *context_lens,
                               const int32_t *cu_q_lens, const float *alibi_slopes, float scale,
                               int num_seqs, int num_heads, int num_kv_heads, int head_dim,
                               int block_size, int max_blocks_per_seq, int dtype)
{
    int group = num_heads / num_kv_heads;
#pragma omp parallel for schedule(dynamic, 1)
    for (int r = 0; r < n_rows; ++r) {
        int t = row_token[r], h = row_head[r];
        int b = 0;
        while (b + 1 < num_seqs && cu_q_lens[b + 1] <= t) ++b;
        int q_len = cu_q_lens[b + 1] - cu_q_lens[b];
        int pos = context_lens[b] - q_len + (t - cu_q_lens[b]);
        double slope = alibi_slopes ? (double)alibi_slopes[h] : 0.0;
        attend_row(out + (int64_t)r * head_dim, q + ((int64_t)t * num_heads + h) * head_dim,
                   k_cache, v_cache, block_tables + (int64_t)b * max_blocks_per_seq, pos + 1, pos,
                   h / group, slope, (double)scale, num_kv_heads, head_dim, block_size, dtype);
    }
}
