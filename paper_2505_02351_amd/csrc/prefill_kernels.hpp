// Prefill over the paged cache: several new query tokens per sequence, causal mask + ALiBi
// (Alg. 1, prompt branch: scores, bias, softmax, weighted sum), as tiled matrix-core contractions.
//
// Workgroup (4 or 8 waves, see WAVES below) = 32 (query token, head) rows per wave of one
// (sequence, KV head [x chunk of the group]) against the whole visible context, in 32-key tiles
// staged through LDS and shared by the waves.  Heads vary fastest inside the rows, so all heads of the group consume the same K/V
// tile (Section II: a group shares one key-value pair).
//
// A wave owns 32 rows.  Both contractions are computed transposed, with v_mfma_f32_32x32x16, so that
// no operand has to be transposed in registers:
//   S^T[key][row] = K Q^T      A = K rows from LDS (natural layout: lane (key L % 32, slab L / 32)
//                              needs 8 consecutive dims of its key), B = the lane's query row held in
//                              VGPRs.  The accumulator starts from the tile-invariant part of the
//                              ALiBi term, so one FMA per score finishes eq. (3).  A lane then holds,
//                              for ONE query row, 16 of the tile's 32 scores (keys 8i + 4 * slab + j in
//                              element 4i + j), which after the softmax pack straight into ...
//   O^T[dim][row] += V^T P^T   ... the B operands of the two output MFMAs of a 32-dim block, whose
//                              contraction index runs over the tile's keys in exactly that
//                              (permuted) order.  A = V^T: V lies in LDS in its natural [key][dim]
//                              layout and is read with the LDS transpose load (ds_read_b64_tr_b16:
//                              inside each group of 16 lanes, lane i receives element i % 4 of the
//                              8-byte chunks addressed by lanes i/4, 4 + i/4, 8 + i/4, 12 + i/4),
//                              so that a lane ends up with four consecutive keys of its dim from
//                              one instruction.
// (32x32x16 rather than 16x16x32 MFMAs: same flops per cycle, half as many matrix and LDS
// instructions per tile, and a row's scores live in 2 lanes instead of 4.  Measured on this chip, a
// SIMD does not overlap 16x16x32 MFMAs of one wave with vector instructions of another at all, and
// 32x32x16 ones only partly, and a wave issues at most one instruction every ~4.4 cycles: the
// loop's cost is close to MFMA cycles plus 4.4 cycles per other instruction, so instruction
// count per tile is what this kernel is tuned for.)
// Scores, sums and the output accumulate in fp32.  For the second contraction the softmax
// weights must become 2-byte values:
//   fp16: one rounding (11 significant bits); the lazily moved reference of the exponentials (see
//         decode_mma_kernels.hpp) is kept tight enough (threshold 2^14, headroom 2^2) that weights
//         stay inside fp16's range;
//   bf16: 8 significant bits are not enough for the 1e-2 output budget once the output itself is
//         rounded to bf16 (measured: 1.003e-2), so each weight is split into a bf16 head and a
//         bf16 tail and the contraction runs twice; bf16's range allows the wide lazy reference.
//
// Key order.  Without a window the tiles are walked from the diagonal BACKWARDS (newest keys
// first).  With ALiBi the bias falls as the walk goes on, so the softmax reference that the first
// tiles set stays valid (walking forwards, steep heads push it up every other tile and the
// accumulators are rescaled each time), and a tile can be judged against what has already been
// summed: when, for every row of the wave, the largest weight of the tile is below 2^-24 of the
// row's sum so far - half an ulp of that fp32 sum, a fact read off the scores, not assumed from
// the slopes - the tile's exponentials, weight packing and output MFMAs are skipped.  Each dropped
// weight is one that an fp32 "sum += w" would have rounded away by itself; a tile drops at most
// 32 of them per row (2^-19 of the row sum), and since skipping only sets in where the weights
// keep falling, the total stays within a few 2^-19 - three orders of magnitude below the compute
// budget of the stated tolerance.  (The definition, eq. (3)-(4), still sums every key; heads with a
// steep slope simply give most keys a weight that no fp32 sum can see.)
#pragma once
#include <type_traits>

#include "decode_mma_kernels.hpp"

namespace optgqa {

// log2 of the fraction of a row's running sum below which a whole tile's weights are dropped
// (half an ulp of an fp32 sum)
#ifndef OPTGQA_PF_SKIP_LOG2
#define OPTGQA_PF_SKIP_LOG2 (-24.f)
#endif
constexpr float kPfSkipLog2 = OPTGQA_PF_SKIP_LOG2;

struct PrefillParams {
    void* out;                  // [T][Hq][D] dtype
    const void* q;              // [T][Hq][D]
    const void* k_cache;        // [NB][Hkv][bs][D]
    const void* v_cache;
    const int32_t* block_tables;
    const int32_t* context_lens;
    const int32_t* cu_q_lens;   // [B + 1]
    const float* slopes;        // [Hq] or nullptr
    float scale2;               // scale * log2(e) (times k_scale for E4M3 caches)
    float out_scale;            // multiplies the output (v_scale of an E4M3 cache, else 1)
    const float* k_scales;      // E4M3 caches with one scale pair per KV head: device arrays [num_kv_heads]
    const float* v_scales;      // (then scale2 holds no k_scale and out_scale is 1), else nullptr
    int num_heads, num_kv_heads, block_size, max_blocks_per_seq;
    int num_seqs;
    int heads_per_wg;           // GH: query heads per workgroup (divides the group size, <= 16)
    int heads_pow2_shift;       // log2 of GH rounded up to a power of two (row = token * 2^shift + head)
    int q_tiles;                // ceil(max_q_len / tokens per workgroup)
    int units;                  // num_seqs * num_kv_heads * (group / GH)
    int window;                 // > 0: the query at position pos sees keys pos - window < j <= pos only
    // whole-prompt variant (CONTIG): K/V come from the step's contiguous inputs, not from the cache
    const void* k_in;           // [T][Hkv][D] with token strides (elements)
    const void* v_in;
    int64_t k_in_stride, v_in_stride;
    void* k_cache_w;            // caches to store the prompt's K/V into (both or neither), else nullptr
    void* v_cache_w;
};

// Waves per workgroup (a template parameter, 32 rows per wave): 8 - 256 rows against one K/V tile,
// half the loader work and LDS stores per row, measured 4 % on the causal kernel - when that still
// gives every CU two rounds of workgroups; else 4, and always 4 with a sliding window, where a
// workgroup's rows should span few keys because every tile that some row's window start or causal
// end cuts needs the masked path (measured: 8 waves 9 % slower there).
constexpr int kPfKeys = 32;                              // keys per tile
// LDS rows, elements: K rows padded by 8 (16-byte reads of 16 keys then cover all 64 banks), V rows
// by 16 (so do the rows a transposing load touches) - head_dim 128: 272 / 288 bytes, 64: 144 / 160
template <int D> struct PfTile {
    static constexpr int kKRow = D + 8, kVRow = D + 16;
    static constexpr int kLdsBytes = 2 * kPfKeys * (kKRow + kVRow) * 2;   // two buffers of one K and one V tile
};

template <int DT> __device__ __forceinline__ uint32_t pack2(float lo, float hi) { return narrow2<DT>(lo, hi); }

typedef float f32x16 __attribute__((ext_vector_type(16)));
// v_mfma_f32_32x32x16: A lane (row L % 32, k-slab L / 32) holds k = 8 * slab .. + 7, B likewise
// for its column; C / D lane (column L % 32, half L / 32) holds rows 8i + 4 * half + j in
// element 4i + j (i, j = 0..3).
template <int DT> __device__ __forceinline__ f32x16 mfma32(uint4 a, uint4 b, f32x16 c);
template <> __device__ __forceinline__ f32x16 mfma32<kF16>(uint4 a, uint4 b, f32x16 c)
{
    typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}
template <> __device__ __forceinline__ f32x16 mfma32<kBF16>(uint4 a, uint4 b, f32x16 c)
{
    typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

template <int DT> struct PfSoftmax;
template <> struct PfSoftmax<kF16> {
    static constexpr float kThreshold = 14.f, kHeadroom = 2.f;
    static constexpr bool kSplitWeights = false;
};
template <> struct PfSoftmax<kBF16> {
    static constexpr float kThreshold = kRescaleThreshold, kHeadroom = kRescaleHeadroom;
    static constexpr bool kSplitWeights = true;
};

#ifndef OPTGQA_PF_WAVES_PER_SIMD
#define OPTGQA_PF_WAVES_PER_SIMD 2
#endif
// KV8: the caches hold 1-byte E4M3 codes with per-tensor scales (k_scale folded into scale2,
// v_scale into out_scale on the host); the loader threads widen them to DT - exactly - on the
// way into LDS, everything after that is unchanged.
//
// CONTIG: the whole prompt is new and nothing of it is in the cache yet (Alg. 1, prompt branch with
// empty caches): the context of sequence b is its own cu_q_lens[b+1] - cu_q_lens[b] tokens, and
// K / V tiles are fetched from the contiguous inputs k_in / v_in (token strides) instead of
// through the block table.  With k_cache_w / v_cache_w set, the workgroups of a KV head's first
// head chunk also store their own tokens' K / V rows into the paged caches (Alg. 1, the
// cache-store step), so the step needs no separate cache-write launch.
//
// STEP: one prefill step over a cache that already holds the earlier tokens (Alg. 1: the cache-store
// step, then the attention): the n_b new tokens of sequence b have their K / V rows in k_in / v_in
// (token cu_q_lens[b] + i = position context_lens[b] - n_b + i) and NOT yet in the cache.  A key
// below the first new position is fetched through the block table, a key at or above it from the
// inputs - chosen per key, both addresses are always valid - and, as with CONTIG, the workgroups of
// a KV head's first head chunk store their own tokens' rows into the caches.  No workgroup reads
// a cache row that this launch writes.
template <int DT, bool KV8, bool WIN, bool CONTIG, int D, int WAVES, bool STEP>
__device__ __forceinline__ void prefill_body(const PrefillParams& p)
{
    static_assert(WAVES == 4 || (WAVES == 8 && !WIN), "4 waves, or 8 without a window");
    constexpr int kPfWaves = WAVES, kPfRows = WAVES * 32;
    static_assert(!(CONTIG && (KV8 || WIN)), "the whole-prompt variant reads 2-byte inputs, full causal mask");
    static_assert(!(STEP && (KV8 || WIN || CONTIG)), "the one-call step runs over 2-byte caches, full causal mask");
    static_assert(D == 128 || D == 64, "head_dim 64 or 128");
    constexpr int kPfKRow = PfTile<D>::kKRow, kPfVRow = PfTile<D>::kVRow;
    constexpr int kQ = D / 16;                          // score MFMAs per tile (16 dims each)
    constexpr int kDB = D / 32;                         // 32-dim blocks of the output
    constexpr int kCPR = D / 8;                         // 16-byte (8-element) column pieces per row
    constexpr int kKPT = kPfKeys * (D / 8) / (kPfWaves * 32);   // consecutive keys a loader thread moves per tile (half the threads per tensor)
    constexpr int ES = KV8 ? 1 : 2;                     // bytes per cache element
    // two tile buffers, each a K tile [32][kPfKRow] followed by a V tile [32][kPfVRow]
    constexpr int kKTile = kPfKeys * kPfKRow, kBuf = kKTile + kPfKeys * kPfVRow;
    extern __shared__ __attribute__((aligned(16))) uint16_t tile_lds[];          // PfTile<D>::kLdsBytes

    // ---- which rows -----------------------------------------------------------------------
    // XCD-aware order: workgroups go to XCD (flat id % 8); all query tiles of one (sequence, KV
    // head) unit are given the same residue so that its K/V stay in one XCD's L2.
    // Longest first: the hardware hands workgroups to free slots in id order, so the workgroups that
    // will run longest should have the lowest ids and the short ones fill the tail of the launch.
    // A later query tile sees more keys; and, walking backwards from the diagonal, a head with a
    // steep ALiBi slope skips most of its tiles while one with a shallow slope skips none - slopes
    // fall with the head number in every usual recipe, so the units are taken from the last KV head
    // down (a wrong guess costs nothing but the order).  Consecutive units, which then share a KV
    // head, are dealt to different XCDs (rotation by the row of eight).
    const int xcd = blockIdx.x & 7, w = blockIdx.x >> 3;
    const int Hq = p.num_heads, Hkv = p.num_kv_heads, bs = p.block_size;
    const int bs_shift = __builtin_ctz(bs);
    const int GH = p.heads_per_wg, gshift = p.heads_pow2_shift;
    const int G = Hq / Hkv, chunks = G / GH;
    const int units_per_seq = Hkv * chunks;
    // (without slopes nothing is skipped and only the query tile decides the length: query tiles first)
    const bool by_head = p.slopes != nullptr;
    const int units8 = (p.units + 7) >> 3;
    const int urow = by_head ? w / p.q_tiles : w % units8;
    const int qt = p.q_tiles - 1 - (by_head ? w % p.q_tiles : w / units8);
    const int ui = urow * 8 + ((xcd - urow) & 7);
    if (ui >= p.units) return;
    const int b = by_head ? ui % p.num_seqs : ui / units_per_seq;
    const int gu = by_head ? units_per_seq - 1 - ui / p.num_seqs : ui - b * units_per_seq;
    const int g = gu / chunks;
    const int h0 = g * G + (gu - g * chunks) * GH;
    const int tokens_per_wg = kPfRows >> gshift;

    const int cu0 = p.cu_q_lens[b];
    const int n_b = p.cu_q_lens[b + 1] - cu0;
    const int tq0 = qt * tokens_per_wg;
    if (tq0 >= n_b) return;
    const int L = CONTIG ? n_b : p.context_lens[b];
    const int pos0 = L - n_b;                                   // position of the sequence's first new token
    const int kmax = pos0 + min(tq0 + tokens_per_wg, n_b);      // keys 0 .. kmax-1 are visible to some row
    const int ntiles = (kmax + kPfKeys - 1) / kPfKeys;
    // Sliding window (Alg. 1, local mask): the workgroup's first row sits at pos0 + tq0 and sees no
    // key before kmin, later rows see even fewer of the early keys, so the tiles before kmin's are
    // never read.
    // (WIN is a compile-time switch so that the plain causal kernel carries none of this)
    const int W = WIN ? p.window : 0;
    const int kmin = W > 0 ? max(pos0 + tq0 - W + 1, 0) : 0;
    const int kt0 = kmin / kPfKeys;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n32 = lane & 31, h2 = lane >> 5;

    const uint16_t* __restrict__ qp = static_cast<const uint16_t*>(p.q);
    // paged: the KV head's offset inside a block; CONTIG: the sequence's token 0, KV head g
    const unsigned char* __restrict__ kc = CONTIG
        ? static_cast<const unsigned char*>(p.k_in) + (cu0 * p.k_in_stride + (int64_t)g * D) * 2
        : static_cast<const unsigned char*>(p.k_cache) + (int64_t)g * bs * D * ES;
    const unsigned char* __restrict__ vc = CONTIG
        ? static_cast<const unsigned char*>(p.v_in) + (cu0 * p.v_in_stride + (int64_t)g * D) * 2
        : static_cast<const unsigned char*>(p.v_cache) + (int64_t)g * bs * D * ES;
    const int32_t* __restrict__ table = p.block_tables + (int64_t)b * p.max_blocks_per_seq;
    const int64_t block_stride = (int64_t)Hkv * bs * D;

    // STEP: the sequence's first new token, KV head g, in the inputs
    const unsigned char* __restrict__ kin = !STEP ? kc
        : static_cast<const unsigned char*>(p.k_in) + (cu0 * p.k_in_stride + (int64_t)g * D) * 2;
    const unsigned char* __restrict__ vin = !STEP ? vc
        : static_cast<const unsigned char*>(p.v_in) + (cu0 * p.v_in_stride + (int64_t)g * D) * 2;

    // CONTIG / STEP: this workgroup's own tokens' K / V rows of head g go into the caches, as 16-byte
    // pieces (kCPR per row and tensor; piece idx = ((token * 2 + is_v) * kCPR + column piece)).  The
    // first kOwnBatch pieces of every thread are loaded here, in front of the first tile fetch, and
    // stored once that tile has landed - one memory latency shared with the fetch instead of a
    // load-then-store loop of its own in front of or behind the walk (each workgroup has the CU to
    // itself, so such a loop is not overlapped by anything: measured 2 us per workgroup round);
    // whatever is left (more than 64 tokens per workgroup) goes out behind the output.
    constexpr int kOwnBatch = 4;
    typedef uint32_t own_u32x4 __attribute__((ext_vector_type(4)));
    const int n_own = ((CONTIG || STEP) && p.k_cache_w && gu == g * chunks) ? min(tokens_per_wg, n_b - tq0) * 2 * kCPR : 0;
    auto own_src = [&](int idx) __attribute__((always_inline)) {
        const int ti = tq0 + idx / (2 * kCPR), is_v = (idx / kCPR) & 1, piece = idx % kCPR;
        return (is_v ? vin + (int64_t)ti * p.v_in_stride * 2 : kin + (int64_t)ti * p.k_in_stride * 2) + 16 * piece;
    };
    auto own_blk_of = [&](int idx) __attribute__((always_inline)) {
        return table[(pos0 + tq0 + idx / (2 * kCPR)) >> bs_shift];   // position in the sequence (CONTIG: pos0 == 0)
    };
    auto own_dst = [&](int idx, int blk) __attribute__((always_inline)) {
        const int tok = pos0 + tq0 + idx / (2 * kCPR), is_v = (idx / kCPR) & 1, piece = idx % kCPR;
        const int64_t dst = blk * block_stride + (int64_t)g * bs * D + (int64_t)(tok & (bs - 1)) * D + 8 * piece;
        return reinterpret_cast<own_u32x4*>((is_v ? static_cast<uint16_t*>(p.v_cache_w) : static_cast<uint16_t*>(p.k_cache_w)) + dst);
    };
    own_u32x4 own[kOwnBatch];
    int own_blk[kOwnBatch];
    if (n_own > 0) {                                             // workgroup-uniform
#pragma unroll
        for (int c = 0; c < kOwnBatch; ++c) {
            const int ic = min((int)threadIdx.x + c * kPfWaves * 64, n_own - 1);
            own[c] = *reinterpret_cast<const own_u32x4*>(own_src(ic));
            own_blk[c] = own_blk_of(ic);
        }
    }

    // This lane's query row (row n32 of the wave's 32): B operand of the score MFMAs (dims
    // 16m + 8h2 .. +7, m = 0..7), its position, slope and validity.
    uint4 qb[kQ];
    float posf, lof, slope2, m_ref, lsum;
    bool row_ok, started;
    int64_t out_off;
    {
        const int row = 32 * wave + n32;
        const int ti = tq0 + (row >> gshift), head = row & ((1 << gshift) - 1);
        row_ok = ti < n_b && head < GH;
        const int tc = min(ti, n_b - 1), hc = min(head, GH - 1);
        const int64_t qrow = ((int64_t)(cu0 + tc) * Hq + h0 + hc) * D;
        out_off = qrow;
        const int pos = pos0 + tc;
        posf = (float)pos;
        lof = W > 0 ? (float)(pos - W) : -1.f;                   // keys above this one are inside the window
        slope2 = p.slopes ? p.slopes[h0 + hc] * kLog2e : 0.f;
        m_ref = 0.f;                                             // set by the first tile in which the row sees a key
        started = false;
        lsum = 0.f;
        const uint32_t keep = row_ok ? 0xffffffffu : 0u;
#pragma unroll
        for (int m = 0; m < kQ; ++m) {
            const uint4 x = *reinterpret_cast<const uint4*>(qp + qrow + 16 * m + 8 * h2);
            qb[m] = make_uint4(x.x & keep, x.y & keep, x.z & keep, x.w & keep);
        }
    }
    // score scale (base 2) and output scale of this workgroup's KV head
    const float scale2 = KV8 && p.k_scales ? p.scale2 * p.k_scales[g] : p.scale2;
    const float out_scale = KV8 && p.v_scales ? p.v_scales[g] : p.out_scale;
    // slope * (offset of the lane's e-th key from its first key in a tile) / score scale: the part of
    // the ALiBi term that does not change from tile to tile, as the score MFMAs' starting value
    f32x16 key_bias;
    {
        const float per_key = slope2 / scale2;
#pragma unroll
        for (int e = 0; e < 16; ++e) key_bias[e] = per_key * (float)(8 * (e >> 2) + (e & 3));
    }
    f32x16 acc[kDB];                                             // O^T: dims 32db + 8i + 4h2 + j of row n32 in element 4i + j
#pragma unroll
    for (int db = 0; db < kDB; ++db)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[db][e] = 0.f;

    // ---- tile staging: threads 0..127 fetch K, 128..255 fetch V; either way a thread moves the
    // same 16-byte column piece of kKPT consecutive keys (kCPR lanes cover one row) ----------------
    const bool k_loader = wave < kPfWaves / 2;                   // wave-uniform (first half of the waves: K; second: V)
    const int l_ahead = k_loader ? 1 : 0;                        // K tiles run one tile ahead of V tiles (below)
    const int ld = k_loader ? tid : tid - kPfWaves * 32;
    const int l_group = ld / kCPR, l_chunk = ld % kCPR;          // keys kKPT*group .. , dims 8*chunk ..
    const unsigned char* __restrict__ l_src = k_loader ? kc : vc;
    const int64_t l_row = CONTIG ? (k_loader ? p.k_in_stride : p.v_in_stride) * 2 : D * ES;   // bytes from key to key
    // STEP: this lane's column piece of the first new token, and the inputs' bytes from token to token
    const unsigned char* const l_in = (k_loader ? kin : vin) + 8 * l_chunk * 2;
    const uint32_t l_in_row = STEP ? (uint32_t)((k_loader ? p.k_in_stride : p.v_in_stride) * 2) : 0u;
    const int l_pitch = k_loader ? kPfKRow : kPfVRow;
    const int l_dst = kKPT * l_group * l_pitch + 8 * l_chunk;
    // One register stage: while tile t is computed, the loader's next tile sits in the other LDS
    // buffer and the one after it is on its way to registers; the block id of the next tile to
    // fetch is read one fetch earlier, so a fetch never waits for the table.  Fetches past the last
    // tile re-read it (cache hits): no branches around loads, which keeps the compiler's load
    // counting exact.
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // native vectors: plain loads and stores
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    typedef typename std::conditional<KV8, u32x2, u32x4>::type StageT;   // 8 elements of one key
    StageT stage[kKPT];
    const int last_tile = ntiles - 1;                             // >= kt0
    const int nt = ntiles - kt0;                                  // tiles this workgroup walks
    // the i-th tile of the walk (i past the end: the last one again)
    auto tile_of = [&](int i) __attribute__((always_inline)) {
        const int ic = min(i, nt - 1);
        return last_tile - ic;                                    // from the diagonal backwards
    };
    auto load_blk = [&](int i) __attribute__((always_inline)) {
        // the keys of a group share a block (groups are aligned, clamping keeps the block)
        if (CONTIG) return 0;
        const int key = min(tile_of(i) * kPfKeys + kKPT * l_group, kmax - 1);
        return table[key >> bs_shift];
    };
    int blk_next = load_blk(0);

    // (address arithmetic kept short on purpose - this loop pays for every instruction: one 64-bit
    // multiply-add for the block, one shift-add for the first row, then per key a clamp and a shift-add;
    // rows past the sequence's last key re-read that key, which lies in the same block)
    const unsigned char* const l_lane = l_src + 8 * l_chunk * ES;                 // this lane's column piece
    const uint32_t l_blk_bytes = (uint32_t)(block_stride * ES);                   // < 2^32: one block of all KV heads
    auto fetch_tile = [&](StageT (&stage)[kKPT], int i) __attribute__((always_inline)) {
        const int key0 = min(tile_of(i) * kPfKeys + kKPT * l_group, kmax - 1);
        const int rmax = kmax - 1 - key0;                         // >= 0; < kKPT - 1 only at the sequence's end
        const unsigned char* base;
        if (CONTIG) base = l_lane + (uint64_t)(uint32_t)key0 * (uint32_t)l_row;
        else base = l_lane + (uint64_t)(uint32_t)blk_next * l_blk_bytes + (uint32_t)((key0 & (bs - 1)) * (D * ES));
        // STEP: a tile that ends below the first new position is all cache (the plain path: most
        // tiles); otherwise the keys from that position on come from the inputs, chosen per key (the
        // clamped key, so that rows past the last visible key re-read it from wherever it lives)
        if (STEP && tile_of(i) * kPfKeys + kPfKeys > pos0) {     // workgroup-uniform
#pragma unroll
            for (int j = 0; j < kKPT; ++j) {
                const unsigned char* a = base + (uint32_t)(min(j, rmax) * (D * ES));
                const int nk = key0 + min(j, rmax) - pos0;
                if (nk >= 0) a = l_in + (uint64_t)(uint32_t)nk * l_in_row;
                stage[j] = *reinterpret_cast<const StageT*>(a);
            }
        } else {
#pragma unroll
            for (int j = 0; j < kKPT; ++j)
                stage[j] = *reinterpret_cast<const StageT*>(base + (uint32_t)(min(j, rmax) * (CONTIG ? (int)l_row : D * ES)));
        }
        blk_next = load_blk(i + 1);
    };
    // A tile's place in LDS: the j-th tile of the walk sits in buffer j % 2.
    auto tile_base = [&](int j) __attribute__((always_inline)) { return (j & 1) * kBuf; };
    auto tile_base_v = [&](int j) __attribute__((always_inline)) { return (j & 1) * kBuf + kKTile; };
    auto store_tile = [&](const StageT (&stage)[kKPT], int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < kKPT; ++j) {
            u32x4 w;
            if constexpr (KV8) {
                const uint4 x = widen8_e4m3<DT>(stage[j][0], stage[j][1]);
                w = u32x4{x.x, x.y, x.z, x.w};
            } else {
                w = stage[j];
            }
            *reinterpret_cast<u32x4*>(&tile_lds[(k_loader ? tile_base(buf) : tile_base_v(buf)) + l_dst + j * l_pitch]) = w;
        }
    };

    // ---- S^T = K Q^T : element 4i + j = score of key 32kt + 8i + 4h2 + j against row n32
    // (the accumulator starts from the tile-invariant part of the ALiBi term, already divided by the
    // score scale, so that one FMA per score finishes eq. (3))
    auto scores = [&](int buf) __attribute__((always_inline)) {
        f32x16 st = key_bias;
#pragma unroll
        for (int m = 0; m < kQ; ++m) {
            const uint4 ka = *reinterpret_cast<const uint4*>(&tile_lds[tile_base(buf) + n32 * kPfKRow + 16 * m + 8 * h2]);
            st = mfma32<DT>(ka, qb[m], st);
        }
        return st;
    };
    // kt: the tile's number along the context; buf: its number in the walk (LDS buffer buf % 2)
    auto softmax_pv = [&](int kt, int buf, f32x16 st, auto masked) __attribute__((always_inline)) {
        constexpr bool MASKED = decltype(masked)::value;
        // ---- bias, causal mask, lazily referenced exponentials (eq. (3), (4)) --------------------
        // x = score - reference, formed directly: st*scale2 + slope2*key + (-slope2*pos - m_ref)
        const float k0 = (float)(kt * kPfKeys + 4 * h2);
        const float cm = -fmaf(slope2, posf, m_ref);
        const float b0 = fmaf(slope2, k0, cm);                   // bias - reference of this lane's first key
        float x[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            x[e] = fmaf(st[e], scale2, b0);
            if (MASKED) {
                const float keyf = k0 + (float)(8 * (e >> 2) + (e & 3));
                const bool visible = WIN ? (keyf <= posf && keyf > lof) : keyf <= posf;
                x[e] = visible ? x[e] : -INFINITY;
            }
        }
        float mx = x[0];
#pragma unroll
        for (int e = 1; e < 16; ++e) mx = fmaxf(mx, x[e]);
        {
            // Walking backwards, the weights of a tile can be judged against what is already summed:
            // below 2^kPfSkipLog2 of the row's sum (this lane's half of it, which is no more) for
            // every row of the wave, the tile changes no bit that the accumulators keep.
            const float room = __builtin_amdgcn_logf(lsum) + kPfSkipLog2;        // log2; -inf before the row's first key
            if (__builtin_amdgcn_ballot_w64(mx > room) == 0) return;
        }
        // Has the row seen a key yet?  Walking backwards from the diagonal, a row's first visible key
        // may lie in a later tile of the walk than another row's.
        const bool first = !started;
        if (__builtin_amdgcn_ballot_w64(first || mx > PfSoftmax<DT>::kThreshold) != 0) {
            mx = fmaxf(mx, __shfl_xor(mx, 32));                  // the row's keys live in 2 lanes (h2)
            // The first keys a row sees put its reference kHeadroom above their maximum, wherever
            // that is (nothing has been accumulated yet); afterwards the reference only moves up
            // (rows with no visible key in the tile, or with lower scores, keep theirs).
            const bool sees = mx > -INFINITY;
            const float delta = first ? (sees ? mx + PfSoftmax<DT>::kHeadroom : 0.f)
                                      : fmaxf(mx + PfSoftmax<DT>::kHeadroom, 0.f);
            const float alpha = first ? 1.f : fast_exp2(-delta);
            started = started || sees;
            m_ref += delta;
            lsum *= alpha;
#pragma unroll
            for (int e = 0; e < 16; ++e) x[e] -= delta;
#pragma unroll
            for (int db = 0; db < kDB; ++db)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[db][e] *= alpha;
        }
        // weights as 2-byte pairs: pk[m] = B operand of the output MFMA over keys 16m .. 16m + 15
        // (its contraction slot (h2, e) is key 16m + 8(e / 4) + 4h2 + e % 4, elements 8m + e of x)
        uint32_t pk[2][4], pk_lo[2][4];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float w0 = fast_exp2(x[2 * e]), w1 = fast_exp2(x[2 * e + 1]);
            if (PfSoftmax<DT>::kSplitWeights) {
                split_bf16(w0, w1, pk[e >> 2][e & 3], pk_lo[e >> 2][e & 3]);
                lsum += w0 + w1;
            } else {
                // single rounding: normalise by the weights as rounded, so that the output stays
                // an exact convex combination of V rows
                const uint32_t hi = pack2<DT>(w0, w1);
                pk[e >> 2][e & 3] = hi;
                pk_lo[e >> 2][e & 3] = 0u;
                lsum += widen_lo<DT>(hi) + widen_hi<DT>(hi);
            }
        }

        // ---- O^T += V^T P^T ---------------------------------------------------------------------
        // A = V^T for dims 32db .. +31: this lane is dim 32db + n32 and needs keys 16m + 4h2 + (0..3)
        // and 16m + 8 + 4h2 + (0..3).  One transposing load hands each group of 16 lanes 4 keys x
        // 16 dims: lane s of a group addresses key (s / 4) of the four, dims 4 (s % 4) .. + 3.
        typedef short i16x4 __attribute__((ext_vector_type(4)));
        typedef __attribute__((address_space(3))) i16x4* lds_i16x4_ptr;
        const int s16 = lane & 15, dhalf = (lane >> 4) & 1;
        const uint16_t* vrow = &tile_lds[tile_base_v(buf) + (4 * h2 + (s16 >> 2)) * kPfVRow + 16 * dhalf + 4 * (s16 & 3)];
#pragma unroll
        for (int db = 0; db < kDB; ++db)
#pragma unroll
            for (int m = 0; m < 2; ++m) {
                const i16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4_ptr)(vrow + 16 * m * kPfVRow + 32 * db));
                const i16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4_ptr)(vrow + (16 * m + 8) * kPfVRow + 32 * db));
                const uint2 lo2 = __builtin_bit_cast(uint2, lo), hi2 = __builtin_bit_cast(uint2, hi);
                const uint4 va = make_uint4(lo2.x, lo2.y, hi2.x, hi2.y);
                acc[db] = mfma32<DT>(va, make_uint4(pk[m][0], pk[m][1], pk[m][2], pk[m][3]), acc[db]);
                if (PfSoftmax<DT>::kSplitWeights)
                    acc[db] = mfma32<DT>(va, make_uint4(pk_lo[m][0], pk_lo[m][1], pk_lo[m][2], pk_lo[m][3]), acc[db]);
            }
    };

    const int pos_min = pos0 + tq0;                             // tiles ending at or below it need no causal mask

    // Software pipeline: the score MFMAs of the walk's next tile are issued before the softmax of the
    // current one, so that the matrix pipe has work while the vector ALU does the exponentials
    // (measured: 3 % on the kernel).  For that the K tiles run one tile ahead of the V tiles: at the
    // start of step j, K tiles j and j + 1 and V tile j are in LDS, K tile j + 2 and V tile j + 1 are
    // on their way to registers.  Prologue:
    fetch_tile(stage, 0);
    store_tile(stage, 0);
    if (n_own > 0) {                                             // the rows loaded at the top have landed with tile 0
#pragma unroll
        for (int c = 0; c < kOwnBatch; ++c) {
            const int idx = (int)threadIdx.x + c * kPfWaves * 64;
            if (idx < n_own) *own_dst(idx, own_blk[c]) = own[c];
        }
    }
    if (k_loader) {                                              // wave-uniform
        fetch_tile(stage, 1);
        store_tile(stage, 1);
    }
    fetch_tile(stage, 1 + l_ahead);
    __syncthreads();
    f32x16 st_next = scores(0);
    __syncthreads();                                             // buffer 0's K tile is overwritten during step 0
    // Tiles wholly inside every row's visible range need no mask: those that end at or below the
    // first row's position (causal side) and start at or above the last row's window start.
    const int n_unmasked = min(ntiles, max(0, (pos_min + 1) / kPfKeys));
    const int n_window_cut = W > 0 ? (max(kmax - W, 0) + kPfKeys - 1) / kPfKeys : 0;
    // (plain loops rather than one with a branch in it, and no branch around the stores: the
    // compiler schedules a loop whose body is one straight line far better)
    // While step j is computed, K tile j + 2 / V tile j + 1 (fetched one step earlier) go into the
    // buffers that step j - 1 used and the next ones are fetched; the waves meet after every step.
    // The last step's look-ahead scores read a stale K buffer and are never used; stores past the
    // last tile put the clamped re-read of it into a buffer nobody reads again.
    // (two steps per trip with the two score registers swapping roles, so that no trip copies the
    // look-ahead scores into place)
    f32x16 st_other;
    auto one_tile = [&](int j, const f32x16& st_cur, f32x16& st_ahead, auto masked) __attribute__((always_inline)) {
        st_ahead = scores(j + 1);
        softmax_pv(last_tile - j, j, st_cur, masked);
        store_tile(stage, j + 1 + l_ahead);
        fetch_tile(stage, j + 2 + l_ahead);
        __syncthreads();
    };
    // steps [from, to) of the walk
    auto run_tiles = [&](int from, int to, auto masked) __attribute__((always_inline)) {
        int j = from;
        for (; j + 1 < to; j += 2) {
            one_tile(j, st_next, st_other, masked);
            one_tile(j + 1, st_other, st_next, masked);
        }
        if (j < to) {
            one_tile(j, st_next, st_other, masked);
            st_next = st_other;
        }
    };
    const int cut_end = max(kt0, min(n_window_cut, n_unmasked));   // tiles cut by some row's window start
    const int plain_end = max(cut_end, n_unmasked);                // tiles no mask touches
    // from the diagonal backwards: the tiles the causal mask cuts come first, those that some
    // row's window start cuts (if there is a window) last
    run_tiles(0, ntiles - plain_end, std::true_type{});
    run_tiles(ntiles - plain_end, ntiles - cut_end, std::false_type{});
    run_tiles(ntiles - cut_end, nt, std::true_type{});

    // ---- normalise and write: this lane holds dims 32db + 8i + 4h2 + (0..3) of its row -----------
    uint16_t* __restrict__ op = static_cast<uint16_t*>(p.out);
    float lt = lsum;
    lt += __shfl_xor(lt, 32);
    if (row_ok) {
        const float inv = out_scale / lt;
#pragma unroll
        for (int db = 0; db < kDB; ++db)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                u32x2 packed;
                packed.x = narrow2<DT>(acc[db][4 * i] * inv, acc[db][4 * i + 1] * inv);
                packed.y = narrow2<DT>(acc[db][4 * i + 2] * inv, acc[db][4 * i + 3] * inv);
                *reinterpret_cast<u32x2*>(op + out_off + 32 * db + 8 * i + 4 * h2) = packed;
            }
    }
    // own rows beyond the first batch (stores inside the walk would delay the tile loads behind
    // them - loads and stores complete in issue order; measured twice as costly as this)
    for (int idx = threadIdx.x + kOwnBatch * kPfWaves * 64; idx < n_own; idx += kPfWaves * 64)
        *own_dst(idx, own_blk_of(idx)) = *reinterpret_cast<const own_u32x4*>(own_src(idx));
}

template <int DT, bool KV8 = false, bool WIN = false, bool CONTIG = false, int D = 128, int WAVES = 4>
__global__ __launch_bounds__(WAVES * 64, OPTGQA_PF_WAVES_PER_SIMD) void paged_prefill_mma_kernel(const PrefillParams p)
{
    prefill_body<DT, KV8, WIN, CONTIG, D, WAVES, false>(p);
}

// cache write + prefill over the cached context in one launch (see STEP above)
template <int DT, int D = 128, int WAVES = 4>
__global__ __launch_bounds__(WAVES * 64, OPTGQA_PF_WAVES_PER_SIMD) void paged_prefill_step_kernel(const PrefillParams p)
{
    prefill_body<DT, false, false, false, D, WAVES, true>(p);
}

}  // namespace optgqa
