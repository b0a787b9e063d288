/*
 * optgqa -- paged grouped-query attention with ALiBi biases for AMD MI355X (gfx950).
 *
 * C ABI of the attention hot path of Opt-GQA (Alg. 1, the forward pass, and Alg. 2,
 * its optimised form on the accelerator, of the paper): the forward pass takes (Q, K, V, C_K, C_V, M)
 * and returns the attention output; M.is_prompt selects the prompt branch or the
 * branch that attends over the caches.  Here the two branches are two entry points and
 * the cache store is a third.
 *
 * General rules for every entry point
 *   - Pointers are DEVICE pointers unless the name ends in _host.  The caller owns every
 *     buffer.  The library never allocates, frees or synchronises; all work is enqueued on
 *     `stream` (a hipStream_t passed as void*, NULL = the default stream).
 *   - State the library keeps between calls: the per-thread event pair of
 *     optgqa_set_kernel_events, the static scratch array of optgqa_paged_attention_static, and
 *     three facts about the device that are asked once per process (compute-unit count,
 *     resident workgroups per kernel, address of that array).  Nothing that depends on a
 *     call's inputs survives the call.
 *   - dtype selects the 2-byte element type of q, k, v, the caches and out.
 *   - Return value: OPTGQA_OK or a negative optgqa_status.  Arguments are checked on the host
 *     before anything is launched; on error nothing has been enqueued.  OPTGQA_ERR_LAUNCH
 *     reports the status of the library's own launch only: an error that earlier work of the
 *     caller left pending in the HIP runtime is neither reported here nor cleared.
 *   - `scale` must be finite (else OPTGQA_ERR_SHAPE).  The prefill entry points evaluate
 *     |scale| < 2^-64 (zero included) as +-2^-64, which changes no output bit at the stated
 *     tolerances, and need |alibi_slopes| * 2^64 to stay finite in fp32.
 *   - Contents of device tables (block ids, slots, context lengths) are NOT checked by the
 *     kernels; out-of-range values are undefined behaviour.  optgqa_validate_tables_host
 *     checks host copies.
 *
 * Cache layout (both caches):  [num_blocks][num_kv_heads][block_size][head_dim], dense,
 * head_dim innermost.  Token j of sequence b lives in physical block
 * block_tables[b][j / block_size], row j % block_size.  (Section III-B: key-value vectors are
 * kept in contiguous fixed-size blocks of a pre-allocated pool.)
 *
 * Supported shapes: head_dim in {64, 128}; block_size in {16, 32, 64};
 * num_heads a multiple of num_kv_heads (any group size).
 */
#ifndef OPTGQA_H
#define OPTGQA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Values of every `dtype` argument.  The arguments themselves are plain ints, so that a value
 * outside this list is answered with OPTGQA_ERR_UNSUPPORTED instead of being undefined behaviour. */
typedef enum { OPTGQA_F16 = 0, OPTGQA_BF16 = 1 } optgqa_dtype;

/* partition_size value that asks optgqa_paged_attention for the equal-work split. */
#define OPTGQA_SPLIT_BALANCED (-2)

typedef enum {
    OPTGQA_OK = 0,
    OPTGQA_ERR_NULL = -1,        /* a required pointer is NULL */
    OPTGQA_ERR_SHAPE = -2,       /* inconsistent or non-positive sizes */
    OPTGQA_ERR_UNSUPPORTED = -3, /* head_dim / block_size / dtype / alignment not supported */
    OPTGQA_ERR_WORKSPACE = -4,   /* split-context needs a larger workspace */
    OPTGQA_ERR_LAUNCH = -5,      /* the HIP runtime refused a launch */
    OPTGQA_ERR_TABLE = -6        /* optgqa_validate_tables_host found a bad entry */
} optgqa_status;

/* Library / ABI version, bumped when a signature changes. */
int optgqa_abi_version(void);

/* Static, human-readable text for a status code. */
const char *optgqa_status_string(int status);

/*
 * KV-cache write (Alg. 1, the cache-store step; eq. (2): the cache is the
 * concatenation, along the token axis, of all blocks so far).
 *
 * For each token t with slot = slot_mapping[t] >= 0, the 2-byte patterns of k[t][g][:] and
 * v[t][g][:] are copied to row slot % block_size of physical block slot / block_size, for every
 * KV head g.  Negative slots are padding and are skipped.  Nothing else in the caches changes.
 * Two tokens with the same slot in one call: undefined which one lands.
 *
 *   k, v            [num_tokens][num_kv_heads][head_dim]; token t starts at element
 *                   t * k_token_stride (resp. v_token_stride); strides in elements,
 *                   >= num_kv_heads * head_dim
 *   k_cache,v_cache [num_blocks][num_kv_heads][block_size][head_dim], modified in place
 *   slot_mapping    [num_tokens] int64
 * num_tokens == 0 is allowed and does nothing.
 */
int optgqa_reshape_and_cache(const void *k, const void *v, void *k_cache, void *v_cache,
                             const int64_t *slot_mapping, int num_tokens, int num_kv_heads,
                             int head_dim, int block_size, int64_t k_token_stride,
                             int64_t v_token_stride, int dtype, void *stream);

/*
 * Decode attention over the paged cache (Alg. 2, the non-prompt branch;
 * eq. (3)-(4); Section II query grouping, shared key-value and ALiBi; Section III-A pages
 * and partitions).
 *
 * For sequence b and query head h, with g = h / (num_heads / num_kv_heads) and
 * L = context_lens[b] (the token being decoded included, its K/V already in the cache):
 *     s_j   = scale * <q[b][h], K_g[j]> + alibi_slopes[h] * (j - (L - 1)),   j = 0..L-1
 *     out[b][h] = sum_j softmax(s)_j * V_g[j]
 * accumulated in fp32 and rounded once (nearest-even) to dtype.  L == 0 gives a row of +0.
 * Rows of a partial last block beyond L and unreferenced blocks are never read.
 *
 *   out, q          [num_seqs][num_heads][head_dim]
 *   block_tables    [num_seqs][max_blocks_per_seq] int32; entries past ceil(L/block_size) unused
 *   context_lens    [num_seqs] int32, 0 <= L <= max_blocks_per_seq * block_size
 *   alibi_slopes    [num_heads] fp32, or NULL for no bias
 *   max_context_len an upper bound on context_lens (used for sizing only)
 *   partition_size  0: the library decides whether and how to split the context;
 *                   >0: split the context into partitions of this many tokens (multiple of
 *                       block_size and of 16) whose results are computed separately and then
 *                       combined (the waves of the launch still get equal shares: a share
 *                       boundary may cut a partition into two separately computed pieces);
 *                   OPTGQA_SPLIT_BALANCED: split by equal work - every wave of the launch gets
 *                       the same number of 16-token tiles, whatever the mix of context
 *                       lengths, and the pieces are combined afterwards; this is also what
 *                       0 picks whenever it splits;
 *                   any other negative value: never split.
 *   workspace       fp32 scratch for the split path, at least
 *                   optgqa_paged_attention_workspace_bytes(...) bytes for the same arguments;
 *                   may be NULL when that returns 0.  Contents are undefined afterwards.
 *                   With partition_size == 0 and a NULL / too small workspace the library
 *                   falls back to the unsplit kernel instead of failing.
 */
int optgqa_paged_attention(void *out, const void *q, const void *k_cache, const void *v_cache,
                           const int32_t *block_tables, const int32_t *context_lens,
                           const float *alibi_slopes, float scale, int num_seqs, int num_heads,
                           int num_kv_heads, int head_dim, int block_size,
                           int max_blocks_per_seq, int max_context_len, int partition_size,
                           void *workspace, size_t workspace_bytes, int dtype,
                           void *stream);

/*
 * optgqa_paged_attention for callers that cannot allocate and cannot bring a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same result
 * as optgqa_paged_attention with partition_size 0 and a workspace of the size it asks for; the
 * split-context scratch is a static array of OPTGQA_STATIC_SCRATCH_BYTES bytes in device memory
 * that belongs to the library (one per GPU the library runs on, held until the process ends).
 * The call allocates and frees nothing.
 *
 *   - Shapes whose split would need more than OPTGQA_STATIC_SCRATCH_BYTES return
 *     OPTGQA_ERR_WORKSPACE and launch nothing (the five measured configurations need at most
 *     9.5 MB; optgqa_paged_attention_workspace_bytes(..., 0, NULL) tells for any shape).
 *   - Every call on a GPU shares that GPU's array: calls that overlap in time on one GPU (two
 *     streams, two threads) race.  Nothing needs clearing between calls.
 *   - The array's address is looked up on the calling thread's current device at the first
 *     call on that device (no allocation, but make that first call outside a graph capture).
 * Other arguments, layouts and errors as optgqa_paged_attention.
 */
#define OPTGQA_STATIC_SCRATCH_BYTES (16u << 20)
int optgqa_paged_attention_static(void *out, const void *q, const void *k_cache, const void *v_cache,
                                  const int32_t *block_tables, const int32_t *context_lens,
                                  const float *alibi_slopes, float scale, int num_seqs, int num_heads,
                                  int num_kv_heads, int head_dim, int block_size,
                                  int max_blocks_per_seq, int max_context_len, int dtype,
                                  void *stream);

/*
 * Measurement aid, not part of the method: with two hipEvent_t handles set, every later
 * optgqa_paged_attention / optgqa_decode_step / optgqa_paged_prefill call made by the SAME
 * host thread records `start_event` just before and `stop_event` just after it launches the
 * kernel that streams the KV cache (the partition / equal-work / tiled prefill kernel), on
 * the call's stream - the small combine and cache-write kernels stay outside the pair.  The
 * caller owns the events and reads hipEventElapsedTime after synchronising.  (NULL, NULL)
 * switches the recording off; one NULL and one handle is OPTGQA_ERR_NULL.
 */
int optgqa_set_kernel_events(void *start_event, void *stop_event);

/*
 * One decode step as a single call (Alg. 2: store K_new, V_new into the caches, then compute
 * the context attention with the caches).  Sequence b appends exactly one token: its K/V rows
 * k_new[b], v_new[b] go to logical position context_lens[b] - 1 (context_lens already counts
 * the new token; the physical slot is block_tables[b][pos / block_size] * block_size +
 * pos % block_size), and out[b] is the attention of q[b] over positions 0 .. context_lens[b] - 1.
 * Same result, bit for bit in the caches and to rounding in `out`, as
 * optgqa_reshape_and_cache with that slot mapping followed by optgqa_paged_attention with
 * partition_size 0; sequences with context_lens[b] == 0 write nothing and give a row of +0.
 * Where the equal-work split applies (a context worth splitting, workspace given) the cache write happens
 * inside the attention kernel - one launch less per step; otherwise the library issues the
 * two launches itself.
 *
 *   k_new, v_new    [num_seqs][num_kv_heads][head_dim]; sequence b starts at element
 *                   b * k_token_stride (resp. v_token_stride), strides >= num_kv_heads * head_dim
 *   k_cache,v_cache modified in place (one row per sequence and KV head)
 *   workspace       as for optgqa_paged_attention with partition_size 0 (sized by
 *                   optgqa_paged_attention_workspace_bytes); NULL / too small: unsplit kernels
 * Other arguments and errors as optgqa_paged_attention.
 */
int optgqa_decode_step(void *out, const void *q, const void *k_new, const void *v_new,
                       void *k_cache, void *v_cache, const int32_t *block_tables,
                       const int32_t *context_lens, const float *alibi_slopes, float scale,
                       int num_seqs, int num_heads, int num_kv_heads, int head_dim, int block_size,
                       int max_blocks_per_seq, int max_context_len, int64_t k_token_stride,
                       int64_t v_token_stride, void *workspace, size_t workspace_bytes,
                       int dtype, void *stream);

/*
 * 8-bit KV cache (the paper's title and Section I pair quantisation with grouped-query attention
 * as the levers on KV-cache traffic; it fixes no format - this is the variant built here).
 * The caches hold 1-byte E4M3 codes (1 sign, 4 exponent bits with bias 7, 3 mantissa bits; no
 * infinities, largest finite value 448, codes 0x7f / 0xff are NaN) in the same
 * [num_blocks][num_kv_heads][block_size][head_dim] layout, with one scale per tensor (these four
 * calls) or one per KV head (the *_heads calls after them).
 *
 * optgqa_reshape_and_cache_fp8: as optgqa_reshape_and_cache, with a quantiser in front:
 *     code = nearest_e4m3( fp32(x) * fp32(1 / scale) )
 * - one fp32 division on the host, one fp32 multiplication per element, round to nearest with
 * ties to the even code, magnitudes above 448 (infinities included) saturate to +-448, NaN
 * becomes 0x7f.  k and v are 2-byte elements of `dtype`; they must be 16-byte aligned with
 * token strides that are multiples of 8 elements, the caches 8-byte aligned
 * (else OPTGQA_ERR_UNSUPPORTED).  k_scale, v_scale: finite and > 0 (else OPTGQA_ERR_SHAPE).
 *
 * optgqa_paged_attention_fp8: as optgqa_paged_attention over such caches (dequantise, then attend):
 *     s_j = scale * k_scale * <q[b][h], value(kcode_j)> + alibi_slopes[h] * (j - (L - 1))
 *     out[b][h] = v_scale * sum_j softmax(s)_j * value(vcode_j)
 * q and out are 2-byte elements of `dtype`.  Always the equal-work split, so
 * the workspace of optgqa_paged_attention_workspace_bytes(..., OPTGQA_SPLIT_BALANCED, ...) is
 * required (OPTGQA_ERR_WORKSPACE without it).
 *
 * optgqa_decode_step_fp8: optgqa_decode_step over such caches - the new token's K / V rows
 * (2-byte, k_new / v_new) are quantised as optgqa_reshape_and_cache_fp8 quantises them and
 * stored at position context_lens[b] - 1, and the attention runs over the codes, the new
 * token's included: same cache bytes and same output (to rounding) as the two calls.  Two
 * launches instead of three: the attention kernel streams the tokens already cached, the
 * combine kernel adds the new token's term and stores its codes.  k_new, v_new 16-byte
 * aligned, strides multiples of 8 (OPTGQA_ERR_UNSUPPORTED otherwise); workspace required.
 *
 * optgqa_paged_prefill_fp8: as optgqa_paged_prefill over such caches, same formulas with the
 * causal bound (query i of sequence b sees keys 0 .. pos_i).  No workspace.
 */
int optgqa_reshape_and_cache_fp8(const void *k, const void *v, void *k_cache, void *v_cache,
                                 const int64_t *slot_mapping, int num_tokens, int num_kv_heads,
                                 int head_dim, int block_size, int64_t k_token_stride,
                                 int64_t v_token_stride, float k_scale, float v_scale,
                                 int dtype, void *stream);

int optgqa_paged_attention_fp8(void *out, const void *q, const void *k_cache, const void *v_cache,
                               const int32_t *block_tables, const int32_t *context_lens,
                               const float *alibi_slopes, float scale, float k_scale, float v_scale,
                               int num_seqs, int num_heads, int num_kv_heads, int head_dim,
                               int block_size, int max_blocks_per_seq, int max_context_len,
                               void *workspace, size_t workspace_bytes, int dtype,
                               void *stream);

int optgqa_decode_step_fp8(void *out, const void *q, const void *k_new, const void *v_new,
                           void *k_cache, void *v_cache, const int32_t *block_tables,
                           const int32_t *context_lens, const float *alibi_slopes, float scale,
                           float k_scale, float v_scale, int num_seqs, int num_heads,
                           int num_kv_heads, int head_dim, int block_size, int max_blocks_per_seq,
                           int max_context_len, int64_t k_token_stride, int64_t v_token_stride,
                           void *workspace, size_t workspace_bytes, int dtype, void *stream);

int optgqa_paged_prefill_fp8(void *out, const void *q, const void *k_cache, const void *v_cache,
                             const int32_t *block_tables, const int32_t *context_lens,
                             const int32_t *cu_q_lens, const float *alibi_slopes, float scale,
                             float k_scale, float v_scale, int num_seqs, int num_heads,
                             int num_kv_heads, int head_dim, int block_size,
                             int max_blocks_per_seq, int max_q_len, int dtype,
                             void *stream);

/*
 * The same four calls with ONE SCALE PAIR PER KV HEAD (k_scales, v_scales: DEVICE arrays of
 * num_kv_heads fp32 values, finite and > 0 - contents are not checked): every formula above with
 * k_scale, v_scale replaced by k_scales[g], v_scales[g], g being the KV head an element belongs
 * to (store: code = nearest_e4m3(fp32(x) * fp32(1 / k_scales[g])), the division done once per use
 * in fp32 on the device, correctly rounded) or the KV head h / (num_heads / num_kv_heads) that query
 * head h reads (attend).  Key and value magnitudes differ from head to head far more than inside
 * one; a scale per head keeps each head's codes in the format's best range.  Shapes, alignment,
 * workspace and errors as for the per-tensor calls; a NULL scale array is OPTGQA_ERR_NULL.
 */
int optgqa_reshape_and_cache_fp8_heads(const void *k, const void *v, void *k_cache, void *v_cache,
                                       const int64_t *slot_mapping, int num_tokens, int num_kv_heads,
                                       int head_dim, int block_size, int64_t k_token_stride,
                                       int64_t v_token_stride, const float *k_scales,
                                       const float *v_scales, int dtype, void *stream);

int optgqa_paged_attention_fp8_heads(void *out, const void *q, const void *k_cache, const void *v_cache,
                                     const int32_t *block_tables, const int32_t *context_lens,
                                     const float *alibi_slopes, float scale, const float *k_scales,
                                     const float *v_scales, int num_seqs, int num_heads,
                                     int num_kv_heads, int head_dim, int block_size,
                                     int max_blocks_per_seq, int max_context_len, void *workspace,
                                     size_t workspace_bytes, int dtype, void *stream);

int optgqa_decode_step_fp8_heads(void *out, const void *q, const void *k_new, const void *v_new,
                                 void *k_cache, void *v_cache, const int32_t *block_tables,
                                 const int32_t *context_lens, const float *alibi_slopes, float scale,
                                 const float *k_scales, const float *v_scales, int num_seqs,
                                 int num_heads, int num_kv_heads, int head_dim, int block_size,
                                 int max_blocks_per_seq, int max_context_len, int64_t k_token_stride,
                                 int64_t v_token_stride, void *workspace, size_t workspace_bytes,
                                 int dtype, void *stream);

int optgqa_paged_prefill_fp8_heads(void *out, const void *q, const void *k_cache, const void *v_cache,
                                   const int32_t *block_tables, const int32_t *context_lens,
                                   const int32_t *cu_q_lens, const float *alibi_slopes, float scale,
                                   const float *k_scales, const float *v_scales, int num_seqs,
                                   int num_heads, int num_kv_heads, int head_dim, int block_size,
                                   int max_blocks_per_seq, int max_q_len, int dtype, void *stream);

/* Bytes of workspace optgqa_paged_attention wants for these arguments (0 = none needed).
 * Also reports, when chosen_partition_size is not NULL, the partition size the library would
 * use (0 = unsplit, OPTGQA_SPLIT_BALANCED = the equal-work split). */
size_t optgqa_paged_attention_workspace_bytes(int num_seqs, int num_heads, int num_kv_heads,
                                              int head_dim, int block_size, int max_context_len,
                                              int partition_size, int *chosen_partition_size);

/*
 * Prefill over the paged cache (Alg. 1 prompt branch: scores, bias, softmax, weighted sum,
 * with a causal mask and the ALiBi bias together).  Sequence b contributes
 * n_b = cu_q_lens[b+1] - cu_q_lens[b] new query tokens whose K/V are already in the cache;
 * query i sits at position pos = context_lens[b] - n_b + i, sees keys 0..pos, and gets the
 * bias alibi_slopes[h] * (j - pos).  QK^T and PV run as bf16/fp16 MFMA contractions with
 * fp32 accumulation; the softmax weights enter the PV product as 2-byte values (fp16: one
 * rounding, the row sum taken over the rounded weights; bf16: a bf16 head plus a bf16 tail, two
 * contractions, so that the weights keep 16 significant bits).  Keys are
 * visited from the query's own position backwards; a 32-key tile in which every weight, for
 * every query row a wave holds, is below 2^-24 of that row's sum so far is dropped (less than
 * half an ulp of the fp32 sum per tile: with ALiBi slopes the far keys of steep heads).
 *
 *   out, q          [total_q_tokens][num_heads][head_dim], total_q_tokens = cu_q_lens[num_seqs]
 *   cu_q_lens       [num_seqs + 1] int32, non-decreasing prefix sums of the n_b, cu_q_lens[0] = 0
 *   context_lens    [num_seqs] int32, total length AFTER the new tokens were cached (>= n_b)
 *   max_q_len       an upper bound on the n_b (sizes the launch; rows beyond n_b do not exist)
 * Sequences with n_b == 0 produce nothing.
 */
int optgqa_paged_prefill(void *out, const void *q, const void *k_cache, const void *v_cache,
                         const int32_t *block_tables, const int32_t *context_lens,
                         const int32_t *cu_q_lens, const float *alibi_slopes, float scale,
                         int num_seqs, int num_heads, int num_kv_heads, int head_dim,
                         int block_size, int max_blocks_per_seq, int max_q_len,
                         int dtype, void *stream);

/*
 * Local attention (Alg. 1: when no ALiBi slopes are given the bias is built from a causal and a
 * local mask; eq. (4) adds the mask inside the softmax).  The paper fixes no window size and
 * no boundary convention; here `window` = W > 0 means that the query at position pos sees
 * exactly the keys pos - W < j <= pos (all of them while pos + 1 <= W).  The mask composes
 * with the ALiBi term, which stays relative to the query's position: pass alibi_slopes or NULL.
 * Blocks that lie wholly before the window are never read.
 *
 *   optgqa_paged_attention_window   optgqa_paged_attention restricted to the last W tokens
 *   optgqa_decode_step_window       optgqa_decode_step (cache write + attention) likewise
 *   optgqa_paged_prefill_window     optgqa_paged_prefill, every new token with its own window
 *
 * window <= 0 is OPTGQA_ERR_SHAPE (call the plain entry points for full attention).  The two
 * decode calls always use the equal-work split: a workspace of
 * optgqa_paged_attention_workspace_bytes(..., OPTGQA_SPLIT_BALANCED) bytes is required
 * (OPTGQA_ERR_WORKSPACE without it).  Other arguments, layouts,
 * ownership and errors as for the calls they extend.
 */
int optgqa_paged_attention_window(void *out, const void *q, const void *k_cache,
                                  const void *v_cache, const int32_t *block_tables,
                                  const int32_t *context_lens, const float *alibi_slopes,
                                  float scale, int window, int num_seqs, int num_heads,
                                  int num_kv_heads, int head_dim, int block_size,
                                  int max_blocks_per_seq, int max_context_len, void *workspace,
                                  size_t workspace_bytes, int dtype, void *stream);

int optgqa_decode_step_window(void *out, const void *q, const void *k_new, const void *v_new,
                              void *k_cache, void *v_cache, const int32_t *block_tables,
                              const int32_t *context_lens, const float *alibi_slopes, float scale,
                              int window, int num_seqs, int num_heads, int num_kv_heads,
                              int head_dim, int block_size, int max_blocks_per_seq,
                              int max_context_len, int64_t k_token_stride, int64_t v_token_stride,
                              void *workspace, size_t workspace_bytes, int dtype,
                              void *stream);

int optgqa_paged_prefill_window(void *out, const void *q, const void *k_cache, const void *v_cache,
                                const int32_t *block_tables, const int32_t *context_lens,
                                const int32_t *cu_q_lens, const float *alibi_slopes, float scale,
                                int window, int num_seqs, int num_heads, int num_kv_heads,
                                int head_dim, int block_size, int max_blocks_per_seq,
                                int max_q_len, int dtype, void *stream);

/*
 * Shared prefixes (Section III-B: cached key-value blocks are shared and reused across requests;
 * the paper gives no interface - this is the one built here).  Sequences that start with the same
 * prompt carry the same physical block ids in the leading entries of their block tables.  The
 * plain entry points already accept such tables (they read the shared blocks once per sequence);
 * these two read them once per BUNDLE of sequences, batching the bundle's queries against each
 * shared K/V tile - the score matrix instruction has 16 query-head columns, a KV head's group
 * fills num_heads / num_kv_heads of them (or the largest divisor <= 16), and the other columns
 * carry the other members' heads at no extra matrix or vector work.
 *
 *   bundle        = optgqa_shared_prefix_bundle(...): sequences per bundle (16 / heads per pass:
 *                   2 for a group of 8, 4 for a group of 4, 16 for multi-head attention).
 *                   Bundles are aligned runs of consecutive sequences: the bundle of sequence b is
 *                   led by sequence b0 = b - b % bundle.  The caller (its scheduler) orders the
 *                   batch so that sequences with a common prefix are neighbours.
 *   shared_blocks   [num_seqs] int32, device.  shared_blocks[b] = n > 0: the first n block-table
 *                   entries of sequence b equal the leader's, every one of those blocks is full
 *                   and already cached for both (never the block that receives a new token);
 *                   0: b shares nothing (always 0 for a leader).  Per bundle the kernel reads
 *                   min over its sharing members of those prefixes once, for all of them, and the
 *                   rest of every sequence as the plain entry points do.  Contents that break
 *                   these rules are undefined behaviour, as for the other device tables;
 *                   optgqa_validate_shared_prefix_host checks host copies (new_tokens = 1 before a
 *                   decode step whose token is counted in context_lens but not yet cached, else 0).
 *   workspace       required: optgqa_shared_prefix_workspace_bytes(...) bytes (always the
 *                   equal-work split; OPTGQA_ERR_WORKSPACE without it).
 * 2-byte caches, no window (there are no entry points for the combinations).  Results: what
 * optgqa_paged_attention / optgqa_decode_step give on the same tables, to rounding (the
 * definition does not know about sharing: eq. (3), (4) over the tokens the tables name).
 */
int optgqa_shared_prefix_bundle(int num_heads, int num_kv_heads, int head_dim);

size_t optgqa_shared_prefix_workspace_bytes(int num_seqs, int num_heads, int num_kv_heads, int head_dim,
                                            int block_size, int max_context_len);

int optgqa_paged_attention_shared(void *out, const void *q, const void *k_cache, const void *v_cache,
                                  const int32_t *block_tables, const int32_t *context_lens,
                                  const int32_t *shared_blocks, const float *alibi_slopes, float scale,
                                  int num_seqs, int num_heads, int num_kv_heads, int head_dim,
                                  int block_size, int max_blocks_per_seq, int max_context_len,
                                  void *workspace, size_t workspace_bytes, int dtype,
                                  void *stream);

int optgqa_decode_step_shared(void *out, const void *q, const void *k_new, const void *v_new,
                              void *k_cache, void *v_cache, const int32_t *block_tables,
                              const int32_t *context_lens, const int32_t *shared_blocks,
                              const float *alibi_slopes, float scale, int num_seqs, int num_heads,
                              int num_kv_heads, int head_dim, int block_size, int max_blocks_per_seq,
                              int max_context_len, int64_t k_token_stride, int64_t v_token_stride,
                              void *workspace, size_t workspace_bytes, int dtype,
                              void *stream);

int optgqa_validate_shared_prefix_host(const int32_t *block_tables_host,
                                       const int32_t *context_lens_host,
                                       const int32_t *shared_blocks_host, int num_seqs,
                                       int max_blocks_per_seq, int block_size, int bundle,
                                       int new_tokens);

/*
 * Whole-prompt attention with empty caches (Alg. 1, prompt branch: the cache-store step,
 * then causal / ALiBi attention computed on the inputs themselves).  Sequence b owns
 * tokens cu_seq_lens[b] .. cu_seq_lens[b+1] - 1 of q, k, v; token i of a sequence attends to
 * tokens 0 .. i of the same sequence with bias slope_h * (j - i).  K / V are read from the
 * contiguous inputs, never from the cache.  With k_cache and v_cache given, the same launch
 * also stores token i's K / V rows at slot block_tables[b][i / block_size] * block_size +
 * i % block_size - bit for bit what optgqa_reshape_and_cache does with that slot mapping -
 * so that later decode steps find them; with both NULL nothing is stored and block_tables,
 * block_size, max_blocks_per_seq are ignored.
 *
 *   out, q          [T][num_heads][head_dim], dense
 *   k, v            [T][num_kv_heads][head_dim]; token t starts at element t * k_token_stride
 *                   (resp. v_token_stride): strides >= num_kv_heads * head_dim, multiples of 8,
 *                   at most 2^30
 *   cu_seq_lens     [num_seqs + 1] int32, cu_seq_lens[0] = 0, T = cu_seq_lens[num_seqs]
 *   max_seq_len     an upper bound on the sequences' lengths (<= max_blocks_per_seq * block_size
 *                   when the caches are given)
 * All pointers device memory, 16-byte aligned; errors as for optgqa_paged_prefill.
 */
int optgqa_prompt_prefill(void *out, const void *q, const void *k, const void *v, void *k_cache,
                          void *v_cache, const int32_t *block_tables, const int32_t *cu_seq_lens,
                          const float *alibi_slopes, float scale, int num_seqs, int num_heads,
                          int num_kv_heads, int head_dim, int block_size, int max_blocks_per_seq,
                          int max_seq_len, int64_t k_token_stride, int64_t v_token_stride,
                          int dtype, void *stream);

/*
 * One prefill step as a single call (Alg. 1: store K, V into the caches, then the attention over the
 * caches - what optgqa_decode_step is for decoding, for any number of new tokens per sequence).
 * Sequence b appends n_b = cu_q_lens[b+1] - cu_q_lens[b] tokens after the
 * context_lens[b] - n_b it already has in the cache (context_lens counts the new tokens): their
 * K / V rows k_new[cu_q_lens[b] + i], v_new[...] go to positions context_lens[b] - n_b + i (slot
 * block_tables[b][pos / block_size] * block_size + pos % block_size), and out is what
 * optgqa_paged_prefill gives afterwards.  Same result, bit for bit in the caches AND in `out`, as
 * optgqa_reshape_and_cache with that slot mapping followed by optgqa_paged_prefill - in one launch:
 * keys before a sequence's first new position are read through the block table, the new ones
 * from k_new / v_new, and the workgroups store the new rows on the side.  No row this call writes is
 * read by it; rows of earlier tokens must be in the cache already.
 *
 *   k_new, v_new    [total_q_tokens][num_kv_heads][head_dim]; token t starts at element
 *                   t * k_token_stride (resp. v_token_stride): strides >= num_kv_heads * head_dim,
 *                   multiples of 8, at most 2^30
 *   k_cache,v_cache modified in place (2-byte caches; n_b rows per sequence and KV head)
 * All pointers device memory, 16-byte aligned.  Other arguments, the dropped key tiles, and errors
 * as optgqa_paged_prefill.
 */
int optgqa_prefill_step(void *out, const void *q, const void *k_new, const void *v_new, void *k_cache,
                        void *v_cache, const int32_t *block_tables, const int32_t *context_lens,
                        const int32_t *cu_q_lens, const float *alibi_slopes, float scale, int num_seqs,
                        int num_heads, int num_kv_heads, int head_dim, int block_size,
                        int max_blocks_per_seq, int max_q_len, int64_t k_token_stride,
                        int64_t v_token_stride, int dtype, void *stream);

/*
 * Diagnostic: un-page the cache (Section III-A: pages are only a re-arrangement of the
 * sequence).  k_out / v_out are [num_seqs][max_context_len][num_kv_heads][head_dim]; token j of
 * sequence b is copied bit for bit for j < context_lens[b]; other rows are left untouched.
 */
int optgqa_gather_kv(void *k_out, void *v_out, const void *k_cache, const void *v_cache,
                     const int32_t *block_tables, const int32_t *context_lens, int num_seqs,
                     int num_kv_heads, int head_dim, int block_size, int max_blocks_per_seq,
                     int max_context_len, int dtype, void *stream);

/*
 * Measurement aid, not part of the method: the decode kernels' memory access pattern with no
 * arithmetic behind it, for pricing them against what the memory system actually delivers.
 * num_workgroups x 4 waves each stream tiles_per_wave "tiles"; tile t of wave w is the 4 KiB
 * piece number tile_list[w * tiles_per_wave + t] of k_pool AND of v_pool (4 KiB = 16 token rows
 * of 256 bytes), read with the K-operand load pattern and the V load pattern of the decode
 * kernels, one tile ahead of a consumer that only XORs the registers together.  Nothing is
 * written (`sink`, 16 bytes, exists so that the loads cannot be optimised away).
 *
 *   k_pool, v_pool  device buffers of pool_bytes each (16-byte aligned)
 *   tile_list       device copy of the list; tile_list_host the SAME list in host memory: every
 *                   entry is checked against pool_bytes / 4096 on the host before the launch
 *                   (OPTGQA_ERR_TABLE if out of range)
 * Bytes read per launch: num_workgroups * 4 * tiles_per_wave * 8192.
 */
int optgqa_stream_probe(const void *k_pool, const void *v_pool, size_t pool_bytes,
                        const int32_t *tile_list, const int32_t *tile_list_host,
                        int num_workgroups, int tiles_per_wave, void *sink, void *stream);

/*
 * Host-side check of host copies of the tables: every block id a sequence references is in
 * [0, num_blocks), every context length fits its table row.  Returns OPTGQA_OK or
 * OPTGQA_ERR_TABLE / OPTGQA_ERR_NULL / OPTGQA_ERR_SHAPE.  Touches no GPU.
 */
int optgqa_validate_tables_host(const int32_t *block_tables_host, const int32_t *context_lens_host,
                                int num_seqs, int max_blocks_per_seq, int block_size,
                                int num_blocks);

#ifdef __cplusplus
}
#endif
#endif /* OPTGQA_H */
