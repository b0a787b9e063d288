/*
 * CPU oracle, whole-prompt clause: attention of a prompt over its own K and V, before any of
 * it is in the cache.
 *
 * TEST INFRASTRUCTURE ONLY (see optgqa_oracle.c).  Shares nothing with the HIP kernels; written
 * again from the definitions so that it stands alone.
 *
 * Alg. 1, prompt branch with empty caches: Q, K, V of the prompt arrive as contiguous
 * [tokens, heads, head_size] tensors, K and V are grouped for GQA, the bias is causal (+ ALiBi
 * when slopes are given), and attention is computed on these inputs directly; the cache store
 * of the same K, V is a separate statement of the algorithm (checked with the cache-write
 * oracle).  Sequence b owns tokens cu_seq_lens[b] .. cu_seq_lens[b+1] - 1; token i of a
 * sequence (0-based inside it) sits at position i:
 *
 *        s_j  = scale * <q_{i,h}, k_{j, h div G}> + slope_h * (j - i)     for j <= i   eq. (3)
 *        out_{i,h} = sum_{j <= i} softmax(s)_j v_{j, h div G}                            eq. (4)
 *
 * Pins (tests/pins_prompt.py): equal to the pinned paged prefill oracle on a cache that was
 * filled with the same tokens; a dense numpy / scipy formulation with a lower-triangular mask;
 * token 0 returns its own V row; sequences do not see each other.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { PROMPT_F16 = 0, PROMPT_BF16 = 1 };

static double prompt_elem_formula(uint16_t h, int dtype)
{
    int sign = (h >> 15) & 1;
    double v;
    if (dtype == PROMPT_F16) {
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
 * each entry is prompt_elem_formula's own result). */
static double *g_prompt_elem_table[2];

static void prompt_elem_tabulate(void)
{
    for (int dt = 0; dt < 2; ++dt) {
        if (g_prompt_elem_table[dt]) continue;
        double *t = (double *)malloc(sizeof(double) * 65536);
        for (int h = 0; h < 65536; ++h) t[h] = prompt_elem_formula((uint16_t)h, dt);
        g_prompt_elem_table[dt] = t;
    }
}

static double prompt_elem(uint16_t h, int dtype) { return g_prompt_elem_table[dtype][h]; }

/* q: [T][num_heads][D]; k, v: [T][num_kv_heads][D], all dense.  For a list of (token, head) pairs
 * (row_token == NULL: all pairs in order, n_rows = T * num_heads); out is [n_rows, D] fp64. */
void oracle_prompt_attention(double *out, const int32_t *row_token, const int32_t *row_head,
                             int n_rows, const uint16_t *q, const uint16_t *k, const uint16_t *v,
                             const int32_t *cu_seq_lens, const float *alibi_slopes, float scale,
                             int num_seqs, int num_heads, int num_kv_heads, int head_dim, int dtype)
{
    prompt_elem_tabulate();
    int group = num_heads / num_kv_heads;
#pragma omp parallel for schedule(dynamic, 1)
    for (int r = 0; r < n_rows; ++r) {
        int t = row_token ? row_token[r] : r / num_heads;
        int h = row_token ? row_head[r] : r % num_heads;
        int b = 0;
        while (b + 1 < num_seqs && cu_seq_lens[b + 1] <= t) ++b;
        int first = cu_seq_lens[b];            /* the sequence's token 0 */
        int i = t - first;                     /* this query's position */
        int g = h / group;
        double slope = alibi_slopes ? (double)alibi_slopes[h] : 0.0;
        const uint16_t *q_row = q + ((int64_t)t * num_heads + h) * head_dim;
        double *o = out + (int64_t)r * head_dim;
        double *s = (double *)malloc(sizeof(double) * (size_t)(i + 1));
        double m = -INFINITY;
        for (int j = 0; j <= i; ++j) {
            const uint16_t *k_row = k + ((int64_t)(first + j) * num_kv_heads + g) * head_dim;
            double dot = 0.0;
            for (int d = 0; d < head_dim; ++d) dot += prompt_elem(q_row[d], dtype) * prompt_elem(k_row[d], dtype);
            s[j] = (double)scale * dot + slope * (double)(j - i);
            if (s[j] > m) m = s[j];
        }
        double denom = 0.0;
        for (int j = 0; j <= i; ++j) {
            s[j] = exp(s[j] - m);
            denom += s[j];
        }
        for (int d = 0; d < head_dim; ++d) o[d] = 0.0;
        for (int j = 0; j <= i; ++j) {
            const uint16_t *v_row = v + ((int64_t)(first + j) * num_kv_heads + g) * head_dim;
            double w = s[j] / denom;
            for (int d = 0; d < head_dim; ++d) o[d] += w * prompt_elem(v_row[d], dtype);
        }
        free(s);
    }
}
