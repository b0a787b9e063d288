/*
 * CPU oracle, 8-bit KV-cache variant: the cache holds E4M3 codes and two per-tensor scales.
 *
 * TEST INFRASTRUCTURE ONLY (see optgqa_oracle.c).  Shares nothing with the HIP kernels: own
 * encoder, own decoder, own index arithmetic.
 *
 * The paper's title and Section I name quantisation next to grouped-query attention as the two
 * levers on KV-cache memory traffic, without fixing a cache format; this file states the
 * variant this build takes ("dequantise, then attend"), so that it has a definition to be
 * checked against:
 *
 *   format    E4M3 ("FN" flavour of the open 8-bit floating-point formats): 1 sign bit, 4 exponent
 *             bits with bias 7, 3 mantissa bits; no infinities; exponent 15 with mantissa 7 is
 *             NaN; largest finite magnitude 448; subnormals m * 2^-9.
 *   store     eq. (2) / Alg. 1 (the cache-store step) with a quantiser in front:
 *                 code = nearest_e4m3( fp32(k) * fp32(1 / k_scale) )
 *             The product is ONE fp32 multiplication (the reciprocal is one fp32 division), the
 *             rounding to E4M3 is to nearest, ties to the even code, magnitudes above 448
 *             (infinities included) saturate to +-448, NaN gives the code 0x7f.  Same for V with
 *             v_scale.  This is a decision that floating point takes about an integer, so it
 *             is specified in the precision the kernel uses (fp32) and compared bit for bit.
 *   attend    eq. (3), (4) on the dequantised values, in fp64:
 *                 s_j = scale * k_scale * <q_h, value(kcode_j)> + slope_h * (j - pos)
 *                 out = v_scale * sum_j softmax(s)_j * value(vcode_j)
 *
 * Pins (tests/pins_e4m3.py): decoder against a library's float8 type for all 256 codes; encoder
 * against the same library on every representable value and midpoint, ties and saturation by
 * exact rational arithmetic; attention reduced to the 2-byte oracle on a cache that holds the
 * dequantised values exactly (every E4M3 value is a bf16 and an fp16 value).
 *
 *   scales    one pair (k_scale, v_scale) per tensor, or - the *_heads functions at the end of this
 *             file - one pair per KV head g (arrays of num_kv_heads fp32 values): the same three
 *             clauses with k_scale, v_scale replaced by k_scales[g], v_scales[g], g being the KV head
 *             the element belongs to (store) or the KV head h div G that query head h reads (attend).
 *             Pinned by reduction to the per-tensor clauses, KV head by KV head.
 *
 * Cache layout: [num_blocks][num_kv_heads][block_size][head_dim], 1-byte elements.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { E4M3_F16 = 0, E4M3_BF16 = 1 };

/* exact widening of the 2-byte query / new-token elements (written again here on purpose:
 * this file stands alone) */
static double two_byte_value_formula(uint16_t h, int dtype)
{
    int sign = (h >> 15) & 1;
    double v;
    if (dtype == E4M3_F16) {
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

static double e4m3_value_formula(uint8_t c)
{
    int sign = c >> 7, e = (c >> 3) & 15, m = c & 7;
    double v;
    if (e == 15 && m == 7) v = NAN;
    else if (e == 0) v = ldexp((double)m, -9);
    else v = ldexp(1.0 + (double)m / 8.0, e - 7);
    return sign ? -v : v;
}

/* The two decoders above, tabulated once per process for all 65 536 two-byte patterns of both
 * types and all 256 codes (the attention loops decode every cache element once per query row;
 * nothing is computed differently, each entry is the formula's own result). */
static double *g_two_byte_value_table[2];
static double g_e4m3_value_table[256];

static void two_byte_value_tabulate(void)
{
    for (int c = 0; c < 256; ++c) g_e4m3_value_table[c] = e4m3_value_formula((uint8_t)c);
    for (int dt = 0; dt < 2; ++dt) {
        if (g_two_byte_value_table[dt]) continue;
        double *t = (double *)malloc(sizeof(double) * 65536);
        for (int h = 0; h < 65536; ++h) t[h] = two_byte_value_formula((uint16_t)h, dt);
        g_two_byte_value_table[dt] = t;
    }
}

static double two_byte_value(uint16_t h, int dtype) { return g_two_byte_value_table[dtype][h]; }
static double e4m3_value(uint8_t c) { return g_e4m3_value_table[c]; }

/* nearest code, ties to even, saturating; nearbyint() rounds to nearest-even in the default
 * rounding mode, and every scaling below is by a power of two, hence exact */
static uint8_t e4m3_nearest(float x)
{
    if (x != x) return 0x7f;
    uint8_t sign = signbit(x) ? 0x80 : 0x00;
    double a = fabs((double)x);
    if (a > 448.0) return sign | 0x7e;                  /* saturate (also +-infinity) */
    if (a < ldexp(1.0, -6)) {                           /* below the smallest normal: steps of 2^-9 */
        int q = (int)nearbyint(ldexp(a, 9));            /* 0 .. 8; 8 is the code of 2^-6 itself */
        return sign | (uint8_t)q;
    }
    int e;
    double f = frexp(a, &e);                            /* a = f * 2^e, f in [0.5, 1) */
    int q = (int)nearbyint(ldexp(f, 4)) - 8;            /* mantissa steps: (2f - 1) * 8, in 0 .. 8 */
    e -= 1;                                             /* a = (1 + q/8) * 2^e */
    if (q == 8) { q = 0; e += 1; }
    if (e > 8 || (e == 8 && q > 6)) return sign | 0x7e; /* rounded past 448 */
    return sign | (uint8_t)(((e + 7) << 3) | q);
}

void oracle_e4m3_values(double *out256)
{
    two_byte_value_tabulate();
    for (int c = 0; c < 256; ++c) out256[c] = e4m3_value((uint8_t)c);
}

void oracle_e4m3_nearest(const float *x, int n, uint8_t *codes)
{
    for (int i = 0; i < n; ++i) codes[i] = e4m3_nearest(x[i]);
}

/* ---- cache write with the quantiser in front ------------------------------------------ */
void oracle_reshape_and_cache_e4m3(const uint16_t *k, const uint16_t *v,
                                   uint8_t *k_cache, uint8_t *v_cache, const int64_t *slot_mapping,
                                   int num_tokens, int num_kv_heads, int head_dim, int block_size,
                                   int64_t k_token_stride, int64_t v_token_stride,
                                   float k_scale, float v_scale, int dtype)
{
    two_byte_value_tabulate();
    const float k_inv = 1.0f / k_scale, v_inv = 1.0f / v_scale;
    for (int t = 0; t < num_tokens; ++t) {
        int64_t slot = slot_mapping[t];
        if (slot < 0) continue;
        int64_t block = slot / block_size, row = slot % block_size;
        for (int g = 0; g < num_kv_heads; ++g) {
            int64_t dst = ((block * num_kv_heads + g) * block_size + row) * head_dim;
            for (int d = 0; d < head_dim; ++d) {
                float kf = (float)two_byte_value(k[t * k_token_stride + (int64_t)g * head_dim + d], dtype);
                float vf = (float)two_byte_value(v[t * v_token_stride + (int64_t)g * head_dim + d], dtype);
                volatile float kp = kf * k_inv;          /* one fp32 multiplication, rounded to fp32 */
                volatile float vp = vf * v_inv;
                k_cache[dst + d] = e4m3_nearest(kp);
                v_cache[dst + d] = e4m3_nearest(vp);
            }
        }
    }
}

/* ---- one query row against the first n_keys tokens of a sequence ----------------------- */
static void attend_row_e4m3(double *out_row, const uint16_t *q_row,
                            const uint8_t *k_cache, const uint8_t *v_cache,
                            const int32_t *table_row, int n_keys, int pos_q, int kv_head,
                            double slope, double scale, double k_scale, double v_scale,
                            int num_kv_heads, int head_dim, int block_size, int dtype)
{
    for (int d = 0; d < head_dim; ++d) out_row[d] = 0.0;
    if (n_keys <= 0) return;
    double *s = (double *)malloc(sizeof(double) * (size_t)n_keys);
    double m = -INFINITY;
    for (int j = 0; j < n_keys; ++j) {
        int64_t at = (((int64_t)table_row[j / block_size] * num_kv_heads + kv_head) * block_size
                      + j % block_size) * head_dim;
        double dot = 0.0;
        for (int d = 0; d < head_dim; ++d)
            dot += two_byte_value(q_row[d], dtype) * e4m3_value(k_cache[at + d]);
        s[j] = scale * k_scale * dot + slope * (double)(j - pos_q);
        if (s[j] > m) m = s[j];
    }
    double denom = 0.0;
    for (int j = 0; j < n_keys; ++j) {
        s[j] = exp(s[j] - m);
        denom += s[j];
    }
    for (int j = 0; j < n_keys; ++j) {
        int64_t at = (((int64_t)table_row[j / block_size] * num_kv_heads + kv_head) * block_size
                      + j % block_size) * head_dim;
        double w = s[j] / denom;
        for (int d = 0; d < head_dim; ++d) out_row[d] += w * e4m3_value(v_cache[at + d]);
    }
    for (int d = 0; d < head_dim; ++d) out_row[d] *= v_scale;
    free(s);
}

/* Decode attention for a list of (sequence, head) pairs (row_seq == NULL: all pairs in order,
 * n_rows = num_seqs * num_heads); out is [n_rows, D]. */
void oracle_paged_attention_e4m3(double *out, const int32_t *row_seq, const int32_t *row_head,
                                 int n_rows, const uint16_t *q,
                                 const uint8_t *k_cache, const uint8_t *v_cache,
                                 const int32_t *block_tables, const int32_t *context_lens,
                                 const float *alibi_slopes, float scale, float k_scale, float v_scale,
                                 int num_heads, int num_kv_heads, int head_dim, int block_size,
                                 int max_blocks_per_seq, int dtype)
{
    two_byte_value_tabulate();
    int group = num_heads / num_kv_heads;
#pragma omp parallel for schedule(dynamic, 1)
    for (int r = 0; r < n_rows; ++r) {
        int b = row_seq ? row_seq[r] : r / num_heads;
        int h = row_seq ? row_head[r] : r % num_heads;
        int L = context_lens[b];
        double slope = alibi_slopes ? (double)alibi_slopes[h] : 0.0;
        attend_row_e4m3(out + (int64_t)r * head_dim, q + ((int64_t)b * num_heads + h) * head_dim,
                        k_cache, v_cache, block_tables + (int64_t)b * max_blocks_per_seq, L, L - 1,
                        h / group, slope, (double)scale, (double)k_scale, (double)v_scale,
                        num_kv_heads, head_dim, block_size, dtype);
    }
}

/* Prefill over an E4M3 cache (Alg. 1 prompt branch on dequantised values): query token t of
 * sequence b sits at position pos = context_lens[b] - q_len_b + (t - cu_q_lens[b]), sees keys
 * 0..pos and gets the bias slope * (j - pos).  For a list of (query token, head) pairs
 * (row_token == NULL: all pairs in order, n_rows = total tokens * num_heads); out is [n_rows, D]. */
void oracle_paged_prefill_e4m3(double *out, const int32_t *row_token, const int32_t *row_head,
                               int n_rows, const uint16_t *q,
                               const uint8_t *k_cache, const uint8_t *v_cache,
                               const int32_t *block_tables, const int32_t *context_lens,
                               const int32_t *cu_q_lens, const float *alibi_slopes,
                               float scale, float k_scale, float v_scale, int num_seqs,
                               int num_heads, int num_kv_heads, int head_dim, int block_size,
                               int max_blocks_per_seq, int dtype)
{
    two_byte_value_tabulate();
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
        attend_row_e4m3(out + (int64_t)r * head_dim, q + ((int64_t)t * num_heads + h) * head_dim,
                        k_cache, v_cache, block_tables + (int64_t)b * max_blocks_per_seq, pos + 1, pos,
                        h / group, slope, (double)scale, (double)k_scale, (double)v_scale,
                        num_kv_heads, head_dim, block_size, dtype);
    }
}

/* ---- one scale pair per KV head ---------------------------------------------------------
 * The three clauses above with k_scales[g], v_scales[g] in place of k_scale, v_scale. */
void oracle_reshape_and_cache_e4m3_heads(const uint16_t *k, const uint16_t *v,
                                         uint8_t *k_cache, uint8_t *v_cache, const int64_t *slot_mapping,
                                         int num_tokens, int num_kv_heads, int head_dim, int block_size,
                                         int64_t k_token_stride, int64_t v_token_stride,
                                         const float *k_scales, const float *v_scales, int dtype)
{
    two_byte_value_tabulate();
    for (int t = 0; t < num_tokens; ++t) {
        int64_t slot = slot_mapping[t];
        if (slot < 0) continue;
        int64_t block = slot / block_size, row = slot % block_size;
        for (int g = 0; g < num_kv_heads; ++g) {
            const float k_inv_g = 1.0f / k_scales[g], v_inv_g = 1.0f / v_scales[g];   /* one fp32 division each */
            int64_t dst_g = ((block * num_kv_heads + g) * block_size + row) * head_dim;
            for (int d = 0; d < head_dim; ++d) {
                float kf = (float)two_byte_value(k[t * k_token_stride + (int64_t)g * head_dim + d], dtype);
                float vf = (float)two_byte_value(v[t * v_token_stride + (int64_t)g * head_dim + d], dtype);
                volatile float kq = kf * k_inv_g;
                volatile float vq = vf * v_inv_g;
                k_cache[dst_g + d] = e4m3_nearest(kq);
                v_cache[dst_g + d] = e4m3_nearest(vq);
            }
        }
    }
}

void oracle_paged_attention_e4m3_heads(double *out, const int32_t *row_seq, const int32_t *row_head,
                                       int n_rows, const uint16_t *q,
                                       const uint8_t *k_cache, const uint8_t *v_cache,
                                       const int32_t *block_tables, const int32_t *context_lens,
                                       const float *alibi_slopes, float scale,
                                       const float *k_scales, const float *v_scales,
                                       int num_heads, int num_kv_heads, int head_dim, int block_size,
                                       int max_blocks_per_seq, int dtype)
{
    two_byte_value_tabulate();
    int group = num_heads / num_kv_heads;
#pragma omp parallel for schedule(dynamic, 1)
    for (int r = 0; r < n_rows; ++r) {
        int b = row_seq ? row_seq[r] : r / num_heads;
        int h = row_seq ? row_head[r] : r % num_heads;
        int L = context_lens[b];
        int kv = h / group;                                  /* the KV head this query head reads */
        double slope = alibi_slopes ? (double)alibi_slopes[h] : 0.0;
        attend_row_e4m3(out + (int64_t)r * head_dim, q + ((int64_t)b * num_heads + h) * head_dim,
                        k_cache, v_cache, block_tables + (int64_t)b * max_blocks_per_seq, L, L - 1,
                        kv, slope, (double)scale, (double)k_scales[kv], (double)v_scales[kv],
                        num_kv_heads, head_dim, block_size, dtype);
    }
}

void oracle_paged_prefill_e4m3_heads(double *out, const int32_t *row_token, const int32_t *row_head,
                                     int n_rows, const uint16_t *q,
                                     const uint8_t *k_cache, const uint8_t *v_cache,
                                     const int32_t *block_tables, const int32_t *context_lens,
                                     const int32_t *cu_q_lens, const float *alibi_slopes, float scale,
                                     const float *k_scales, const float *v_scales, int num_seqs,
                                     int num_heads, int num_kv_heads, int head_dim, int block_size,
                                     int max_blocks_per_seq, int dtype)
{
    two_byte_value_tabulate();
    int group = num_heads / num_kv_heads;
#pragma omp parallel for schedule(dynamic, 1)
    for (int r = 0; r < n_rows; ++r) {
        int t = row_token ? row_token[r] : r / num_heads;
        int h = row_token ? row_head[r] : r % num_heads;
        int b = 0;
        while (b + 1 < num_seqs && cu_q_lens[b + 1] <= t) ++b;
        int n_new = cu_q_lens[b + 1] - cu_q_lens[b];          /* new tokens of sequence b */
        int pos = context_lens[b] - n_new + (t - cu_q_lens[b]);
        int kv = h / group;
        double slope = alibi_slopes ? (double)alibi_slopes[h] : 0.0;
        attend_row_e4m3(out + (int64_t)r * head_dim, q + ((int64_t)t * num_heads + h) * head_dim,
                        k_cache, v_cache, block_tables + (int64_t)b * max_blocks_per_seq, pos + 1, pos,
                        kv, slope, (double)scale, (double)k_scales[kv], (double)v_scales[kv],
                        num_kv_heads, head_dim, block_size, dtype);
    }
}
