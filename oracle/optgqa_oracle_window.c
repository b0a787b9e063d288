/*
 * CPU oracle, local-attention variant: causal mask plus a sliding window over the paged cache.
 *
 * TEST INFRASTRUCTURE ONLY (see optgqa_oracle.c).  Shares nothing with the HIP kernels; written
 * again from the definitions so that it stands alone.
 *
 * Alg. 1 builds a causal and a local attention mask for the bias term when no ALiBi slopes are
 * given, and eq. (4) adds the mask inside the softmax.  The paper gives no window size and does
 * not say which side of the boundary is kept; the reading taken here (the usual one for sliding
 * windows): with window W > 0 the query at position pos sees exactly the W keys
 *
 *        pos - W < j <= pos          (fewer when pos + 1 < W),
 *
 * W <= 0 means no local mask.  The definition is written out as the paper's formula, mask
 * matrix and all:
 *
 *        M_j  = 0 if pos - W < j <= pos, else -infinity
 *        s_j  = scale * <q_h, k_j> + slope_h * (j - pos) + M_j          eq. (3) with eq. (4)'s mask
 *        out  = sum_j softmax(s)_j v_j                                   over ALL keys 0 .. L-1
 *
 * so masked keys are still scored and take part in the softmax with weight exp(-inf) = 0.  The
 * slope term stays defined relative to the query position, not to the window's first key.  The
 * window composes with ALiBi (slopes may be given or not).
 *
 * Pins (tests/pins_window.py): W >= context reduces to the pinned oracle; a windowed row equals
 * the pinned oracle on a cache that holds only the window's tokens; W = 1 returns the token's
 * own V row; a dense numpy/scipy formulation with a banded mask matrix on small cases.
 *
 * Cache layout: [num_blocks][num_kv_heads][block_size][head_dim], 2-byte elements.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { WIN_F16 = 0, WIN_BF16 = 1 };

static double elem_value_formula(uint16_t h, int dtype)
{
    int sign = (h >> 15) & 1;
    double v;
    if (dtype == WIN_F16) {
        int e = (h >> 10) & 0x1F, m = h & 0x3FF;
        if (e == 0) v = ldexp((double)m, -24);
        else if (e == 31) v = m ? NAN : INFINITY;
        else v = ldexp(1.0 + (double)m / 1024.0, e - 15);
    } else {
        int e = (h >> 7) & 0xFF, m = h & 0x7F;
        if (e == 0) v = ldexp((double)m, -133);
        else if (e == 255) v = m ? NAN : INFINITY;
        else v = ldexp(1.0 + (double)m / 128.0, e - 127);
    }
    return sign ? -v : v;
}

/* The decoder above, tabulated once per process for all 65 536 patterns of both types (the
 * attention loops decode every cache element once per query row; nothing is computed differently,
 * each entry is elem_value_formula's own result). */
static double *g_elem_value_table[2];

static void elem_value_tabulate(void)
{
    for (int dt = 0; dt < 2; ++dt) {
        if (g_elem_value_table[dt]) continue;
        double *t = (double *)malloc(sizeof(double) * 65536);
        for (int h = 0; h < 65536; ++h) t[h] = elem_value_formula((uint16_t)h, dt);
        g_elem_value_table[dt] = t;
    }
}

static double elem_value(uint16_t h, int dtype) { return g_elem_value_table[dtype][h]; }

/* One query row at position pos of a sequence whose cache holds n_ctx tokens (n_ctx > pos). */
static void attend_row_window(double *out_row, const uint16_t *q_row,
                              const uint16_t *k_cache, const uint16_t *v_cache,
                              const int32_t *table_row, int n_ctx, int pos, int window, int kv_head,
                              double slope, double scale, int num_kv_heads, int head_dim,
                              int block_size, int dtype)
{
    for (int d = 0; d < head_dim; ++d) out_row[d] = 0.0;
    if (n_ctx <= 0) return;
    double *s = (double *)malloc(sizeof(double) * (size_t)n_ctx);
    double m = -INFINITY;
    for (int j = 0; j < n_ctx; ++j) {
        int64_t at = (((int64_t)table_row[j / block_size] * num_kv_heads + kv_head) * block_size
                      + j % block_size) * head_dim;
        double dot = 0.0;
        for (int d = 0; d < head_dim; ++d)
            dot += elem_value(q_row[d], dtype) * elem_value(k_cache[at + d], dtype);
        int causal_ok = j <= pos;
        int local_ok = window <= 0 || j > pos - window;
        double mask = (causal_ok && local_ok) ? 0.0 : -INFINITY;
        s[j] = scale * dot + slope * (double)(j - pos) + mask;
        if (s[j] > m) m = s[j];
    }
    double denom = 0.0;
    for (int j = 0; j < n_ctx; ++j) {
        s[j] = exp(s[j] - m);              /* exp(-inf) = 0 for masked keys */
        denom += s[j];
    }
    for (int j = 0; j < n_ctx; ++j) {
        int64_t at = (((int64_t)table_row[j / block_size] * num_kv_heads + kv_head) * block_size
                      + j % block_size) * head_dim;
        double w = s[j] / denom;
        if (w == 0.0) continue;            /* a masked key's V row may hold anything, also NaN */
        for (int d = 0; d < head_dim; ++d) out_row[d] += w * elem_value(v_cache[at + d], dtype);
    }
    free(s);
}

/* Decode: the query of sequence b sits at position context_lens[b] - 1.  For a list of
 * (sequence, head) pairs (row_seq == NULL: all pairs in order); out is [n_rows, D]. */
void oracle_paged_attention_window(double *out, const int32_t *row_seq, const int32_t *row_head,
                                   int n_rows, const uint16_t *q,
                                   const uint16_t *k_cache, const uint16_t *v_cache,
                                   const int32_t *block_tables, const int32_t *context_lens,
                                   const float *alibi_slopes, float scale, int window,
                                   int num_heads, int num_kv_heads, int head_dim, int block_size,
                                   int max_blocks_per_seq, int dtype)
{
    elem_value_tabulate();
    int group = num_heads / num_kv_heads;
#pragma omp parallel for schedule(dynamic, 1)
    for (int r = 0; r < n_rows; ++r) {
        int b = row_seq ? row_seq[r] : r / num_heads;
        int h = row_seq ? row_head[r] : r % num_heads;
        int L = context_lens[b];
        double slope = alibi_slopes ? (double)alibi_slopes[h] : 0.0;
        attend_row_window(out + (int64_t)r * head_dim, q + ((int64_t)b * num_heads + h) * head_dim,
                          k_cache, v_cache, block_tables + (int64_t)b * max_blocks_per_seq, L, L - 1,
                          window, h / group, slope, (double)scale, num_kv_heads, head_dim,
                          block_size, dtype);
    }
}

/* Prefill (Alg. 1 prompt branch): query token t of sequence b sits at position
 * pos = context_lens[b] - q_len_b + (t - cu_q_lens[b]); the cache already holds the whole
 * sequence, the causal mask hides the keys after pos.  For a list of (query token, head) pairs
 * (row_token == NULL: all pairs in order); out is [n_rows, D]. */
void oracle_paged_prefill_window(double *out, const int32_t *row_token, const int32_t *row_head,
                                 int n_rows, const uint16_t *q,
                                 const uint16_t *k_cache, const uint16_t *v_cache,
                                 const int32_t *block_tables, const int32_t *context_lens,
                                 const int32_t *cu_q_lens, const float *alibi_slopes, float scale,
                                 int window, int num_seqs, int num_heads, int num_kv_heads,
                                 int head_dim, int block_size, int max_blocks_per_seq, int dtype)
{
    elem_value_tabulate();
    int group = num_heads / num_kv_heads;
#pragma omp parallel for schedule(dynamic, 1)
    for (int r = 0; r < n_rows; ++r) {
        int t = row_token ? row_token[r] : r / num_heads;
        int h = row_token ? row_head[r] : r % num_heads;
        int b = 0;
        while (b + 1 < num_seqs && cu_q_lens[b + 1] <= t) ++b;
        int new_tokens = cu_q_lens[b + 1] - cu_q_lens[b];
        int pos = context_lens[b] - new_tokens + (t - cu_q_lens[b]);
        double slope = alibi_slopes ? (double)alibi_slopes[h] : 0.0;
        attend_row_window(out + (int64_t)r * head_dim, q + ((int64_t)t * num_heads + h) * head_dim,
                          k_cache, v_cache, block_tables + (int64_t)b * max_blocks_per_seq,
                          context_lens[b], pos, window, h / group, slope, (double)scale,
                          num_kv_heads, head_dim, block_size, dtype);
    }
}
