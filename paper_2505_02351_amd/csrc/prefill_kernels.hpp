// Prefill over the paged cache: several new query tokens per sequence, causal mask + ALiBi
// (Alg. 1, prompt branch: scores, bias, softmax, weighted sum), as tiled matrix-core contractions.
//
// Workgroup (4 waves) = kPfRows (query token, head) rows of one (sequence, KV head [x chunk of the
// group]) against the whole visible context, in 32-key tiles staged through LDS and shared by the
// four waves.  Heads vary fastest inside the rows, so all heads of the group consume the same K/V
// tile (Section II, "Shared Key-Value").
//
// Both contractions are computed transposed so that no operand has to be transposed in registers:
//   S^T[key][row] = K Q^T      v_mfma_f32_16x16x32: A = K rows from LDS (natural layout: a lane
//                              needs 8 consecutive dims of one key), B = query rows held in VGPRs.
//                              A lane then holds, for ONE query row, keys 4hg+v of both 16-key
//                              halves of the tile: 8 weights that pack straight into ...
//   O^T[dim][row] += V^T P^T   ... the B operand of the second v_mfma_f32_16x16x32, whose
//                              contraction index runs over the tile's keys in exactly that
//                              (permuted) order.  A = V^T: V lies in LDS in its natural [key][dim]
//                              layout and is read with the LDS transpose load (ds_read_b64_tr_b16:
//                              inside each group of 16 lanes, lane i receives element i % 4 of the
//                              8-byte chunks addressed by lanes i/4, 4 + i/4, 8 + i/4, 12 + i/4),
//                              so that lane (dim i, slab q) ends up with keys 4q .. 4q+3 of dim i
//                              from one instruction and keys 16 + 4q .. from a second one.
// Scores, sums and the output accumulate in fp32.  For the second contraction the softmax
// weights must become 2-byte values:
//   fp16: one rounding (11 significant bits); the lazily moved reference of the exponentials (see
//         decode_mma_kernels.hpp) is kept tight enough (threshold 2^14, headroom 2^2) that weights
//         stay inside fp16's range;
//   bf16: 8 significant bits are not enough for the 1e-2 output budget once the output itself is
//         rounded to bf16 (measured: 1.003e-2), so each weight is split into a bf16 head and a
//         bf16 tail and the contraction runs twice; bf16's range allows the wide lazy reference.
#pragma once
#include <type_traits>

#include "decode_mma_kernels.hpp"

namespace optgqa {

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

constexpr int kPfWaves = 4;
constexpr int kPfRowBlocks = 2;                          // 16-row blocks per wave
constexpr int kPfRows = kPfWaves * kPfRowBlocks * 16;    // (token, head) rows per workgroup
constexpr int kPfKeys = 32;                              // keys per tile
constexpr int kPfKRow = 128 + 8;                         // LDS K row, elements (padding spreads banks)
constexpr int kPfVRow = 128 + 16;                        // LDS V row, elements: 288 bytes, so that the 8 rows a
                                                         // transpose load touches per pass cover all 64 banks

template <int DT> __device__ __forceinline__ uint32_t pack2(float lo, float hi) { return narrow2<DT>(lo, hi); }

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
// head chunk also store their own tokens' K / V rows into the paged caches (Alg. 1 "reshape
// and store K, V"), so the step needs no separate cache-write launch.
template <int DT, bool KV8 = false, bool WIN = false, bool CONTIG = false>
__global__ __launch_bounds__(kPfWaves * 64, OPTGQA_PF_WAVES_PER_SIMD) void paged_prefill_mma_kernel(const PrefillParams p)
{
    static_assert(!(CONTIG && (KV8 || WIN)), "the whole-prompt variant reads 2-byte inputs, full causal mask");
    constexpr int D = 128;
    constexpr int ES = KV8 ? 1 : 2;                     // bytes per cache element
    constexpr int RB = kPfRowBlocks;
    // two tile buffers, each a K tile [32][kPfKRow] followed by a V tile [32][kPfVRow]
    constexpr int kKTile = kPfKeys * kPfKRow, kBuf = kKTile + kPfKeys * kPfVRow;
    __shared__ __attribute__((aligned(16))) uint16_t tile_lds[2 * kBuf];

    // ---- which rows -----------------------------------------------------------------------
    // XCD-aware order: workgroups go to XCD (flat id % 8); all query tiles of one (sequence, KV
    // head) unit are given the same residue so that its K/V stay in one XCD's L2.
    const int xcd = blockIdx.x & 7, w = blockIdx.x >> 3;
    const int qt = w % p.q_tiles;
    const int unit = (w / p.q_tiles) * 8 + xcd;
    if (unit >= p.units) return;
    const int Hq = p.num_heads, Hkv = p.num_kv_heads, bs = p.block_size;
    const int bs_shift = __builtin_ctz(bs);
    const int GH = p.heads_per_wg, gshift = p.heads_pow2_shift;
    const int G = Hq / Hkv, chunks = G / GH;
    const int units_per_seq = Hkv * chunks;
    const int b = unit / units_per_seq;
    const int gu = unit - b * units_per_seq;
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
    const int n16 = lane & 15, hg = lane >> 4;

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

    if (CONTIG && p.k_cache_w && gu == g * chunks) {
        // store this workgroup's own tokens' K / V rows of head g (16-byte pieces: 16 per row and tensor)
        const int ntok = min(tokens_per_wg, n_b - tq0);
        for (int idx = threadIdx.x; idx < ntok * 32; idx += kPfWaves * 64) {
            const int tok = tq0 + (idx >> 5), is_v = (idx >> 4) & 1, piece = idx & 15;
            const int blk = table[tok >> bs_shift];
            const int64_t dst = blk * block_stride + (int64_t)g * bs * D + (int64_t)(tok & (bs - 1)) * D + 8 * piece;
            const unsigned char* src = (is_v ? vc + (int64_t)tok * p.v_in_stride * 2 : kc + (int64_t)tok * p.k_in_stride * 2) + 16 * piece;
            uint16_t* dstp = (is_v ? static_cast<uint16_t*>(p.v_cache_w) : static_cast<uint16_t*>(p.k_cache_w)) + dst;
            *reinterpret_cast<uint4*>(dstp) = *reinterpret_cast<const uint4*>(src);
        }
    }

    // This lane's query row in each of the wave's row blocks: B operand of the score MFMAs
    // (row n16, dims 32i + 8hg .. +7), its position, slope and validity.
    uint4 qb[RB][4];
    float posf[RB], lof[RB], slope2[RB], m_ref[RB], lsum[RB];
    int pos[RB];
    bool row_ok[RB], started[RB];
    int64_t out_off[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        const int row = 16 * (wave * RB + rb) + n16;
        const int ti = tq0 + (row >> gshift), head = row & ((1 << gshift) - 1);
        row_ok[rb] = ti < n_b && head < GH;
        const int tc = min(ti, n_b - 1), hc = min(head, GH - 1);
        const int64_t qrow = ((int64_t)(cu0 + tc) * Hq + h0 + hc) * D;
        out_off[rb] = qrow;
        pos[rb] = pos0 + tc;
        posf[rb] = (float)pos[rb];
        lof[rb] = W > 0 ? (float)(pos[rb] - W) : -1.f;           // keys above this one are inside the window
        slope2[rb] = p.slopes ? p.slopes[h0 + hc] * kLog2e : 0.f;
        m_ref[rb] = 0.f;                                         // set by the first tile in which the row sees a key
        started[rb] = false;
        lsum[rb] = 0.f;
        const uint32_t keep = row_ok[rb] ? 0xffffffffu : 0u;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint4 x = *reinterpret_cast<const uint4*>(qp + qrow + 32 * i + 8 * hg);
            qb[rb][i] = make_uint4(x.x & keep, x.y & keep, x.z & keep, x.w & keep);
        }
    }
    f32x4 acc[RB][8];                                            // O^T: dims 16dt + 4hg + v of row n16
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) acc[rb][dt] = f32x4{0.f, 0.f, 0.f, 0.f};

    // ---- tile staging: threads 0..127 fetch K, 128..255 fetch V; either way a thread moves the
    // same 16-byte column piece of 4 consecutive keys (16 lanes cover one 256-byte row) ------------
    const bool k_loader = tid < 128;
    const int ld = k_loader ? tid : tid - 128;
    const int l_group = ld >> 4, l_chunk = ld & 15;              // keys 4*group .. +3, dims 8*chunk ..
    const unsigned char* __restrict__ l_src = k_loader ? kc : vc;
    const int64_t l_row = CONTIG ? (k_loader ? p.k_in_stride : p.v_in_stride) * 2 : D * ES;   // bytes from key to key
    const int l_pitch = k_loader ? kPfKRow : kPfVRow;
    const int l_dst = (k_loader ? 0 : kKTile) + 4 * l_group * l_pitch + 8 * l_chunk;
    // One register stage: while tile t is computed, tile t + 1 sits in the other LDS buffer and
    // tile t + 2 is on its way to registers; the block id of the next tile to fetch is read one
    // fetch earlier, so a fetch never waits for the table.  Fetches past the last tile re-read it (cache hits, never stored):
    // no branches around loads, which keeps the compiler's load counting exact.
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // native vectors: plain loads and stores
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    typedef typename std::conditional<KV8, u32x2, u32x4>::type StageT;   // 8 elements of one key
    StageT stage[4];
    const int last_tile = ntiles - 1;                             // >= kt0
    auto load_blk = [&](int t) __attribute__((always_inline)) {
        // the four keys of a group share a block (groups are 4-aligned, clamping keeps the block)
        if (CONTIG) return 0;
        const int key = min(min(t, last_tile) * kPfKeys + 4 * l_group, kmax - 1);
        return table[key >> bs_shift];
    };
    int blk_next = load_blk(kt0);

    auto fetch_tile = [&](StageT (&stage)[4], int t) __attribute__((always_inline)) {
        const int key0 = min(t, last_tile) * kPfKeys + 4 * l_group;
        const unsigned char* src = l_src + (blk_next * block_stride + 8 * l_chunk) * ES;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int key = min(key0 + j, kmax - 1);
            stage[j] = *reinterpret_cast<const StageT*>(src + (int64_t)(CONTIG ? key : key & (bs - 1)) * l_row);
        }
        blk_next = load_blk(t + 1);
    };
    auto store_tile = [&](const StageT (&stage)[4], int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            u32x4 w;
            if constexpr (KV8) {
                const uint4 x = widen8_e4m3<DT>(stage[j][0], stage[j][1]);
                w = u32x4{x.x, x.y, x.z, x.w};
            } else {
                w = stage[j];
            }
            *reinterpret_cast<u32x4*>(&tile_lds[buf * kBuf + l_dst + j * l_pitch]) = w;
        }
    };

    const float scale2 = p.scale2;
    auto compute_tile = [&](int kt, int buf, auto masked) __attribute__((always_inline)) {
        constexpr bool MASKED = decltype(masked)::value;
        // ---- S^T = K Q^T : st[rb][half][v] = score of key 32kt + 16half + 4hg + v against row n16
        f32x4 st[RB][2];
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) st[rb][0] = st[rb][1] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int half = 0; half < 2; ++half)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint4 ka = *reinterpret_cast<const uint4*>(
                    &tile_lds[buf * kBuf + (16 * half + n16) * kPfKRow + 32 * i + 8 * hg]);
#pragma unroll
                for (int rb = 0; rb < RB; ++rb) st[rb][half] = mfma_qk<DT>(ka, qb[rb][i], st[rb][half]);
            }

        // ---- bias, causal mask, lazily referenced exponentials (eq. (3), (4)) --------------------
        // x = score - reference, formed directly: st*scale2 + slope2*key + (-slope2*pos - m_ref)
        float keyf[8];
        {
            const float k0 = (float)(kt * kPfKeys + 4 * hg);
#pragma unroll
            for (int e = 0; e < 8; ++e) keyf[e] = k0 + (float)(16 * (e >> 2) + (e & 3));
        }
        uint32_t pk[RB][4], pk_lo[RB][4];
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            const float cm = -fmaf(slope2[rb], posf[rb], m_ref[rb]);
            float x[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                x[e] = fmaf(st[rb][e >> 2][e & 3], scale2, fmaf(slope2[rb], keyf[e], cm));
                if (MASKED) {
                    const bool visible = WIN ? (keyf[e] <= posf[rb] && keyf[e] > lof[rb]) : keyf[e] <= posf[rb];
                    x[e] = visible ? x[e] : -INFINITY;
                }
            }
            float mx = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])), fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
            // Has the row seen a key yet?  Plain causal rows all see key 0 in tile 0, so there the
            // answer is wave-uniform; with a window a row's first visible key may lie in a later tile.
            const bool first = WIN ? !started[rb] : kt == 0;
            if (__builtin_amdgcn_ballot_w64(first || mx > PfSoftmax<DT>::kThreshold) != 0) {
                mx = fmaxf(mx, __shfl_xor(mx, 16));              // the row's keys live in 4 lanes (hg)
                mx = fmaxf(mx, __shfl_xor(mx, 32));
                // The first keys a row sees put its reference kHeadroom above their maximum, wherever
                // that is (nothing has been accumulated yet); afterwards the reference only moves up
                // (rows with no visible key in the tile, or with lower scores, keep theirs).
                const bool sees = mx > -INFINITY;
                const float delta = first ? (sees ? mx + PfSoftmax<DT>::kHeadroom : 0.f)
                                          : fmaxf(mx + PfSoftmax<DT>::kHeadroom, 0.f);
                const float alpha = first ? 1.f : fast_exp2(-delta);
                if (WIN) started[rb] = started[rb] || sees;
                m_ref[rb] += delta;
                lsum[rb] *= alpha;
#pragma unroll
                for (int e = 0; e < 8; ++e) x[e] -= delta;
#pragma unroll
                for (int dt = 0; dt < 8; ++dt)
#pragma unroll
                    for (int v = 0; v < 4; ++v) acc[rb][dt][v] *= alpha;
            }
            float pw[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) pw[e] = fast_exp2(x[e]);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                pk[rb][e] = pack2<DT>(pw[2 * e], pw[2 * e + 1]);
                pk_lo[rb][e] = 0u;
                if (PfSoftmax<DT>::kSplitWeights) {
                    pk_lo[rb][e] = pack2<DT>(pw[2 * e] - widen_lo<DT>(pk[rb][e]), pw[2 * e + 1] - widen_hi<DT>(pk[rb][e]));
                    lsum[rb] += pw[2 * e] + pw[2 * e + 1];
                } else {
                    // single rounding: normalise by the weights as rounded, so that the output stays
                    // an exact convex combination of V rows
                    lsum[rb] += widen_lo<DT>(pk[rb][e]) + widen_hi<DT>(pk[rb][e]);
                }
            }
        }

        // ---- O^T += V^T P^T ---------------------------------------------------------------------
        typedef short i16x4 __attribute__((ext_vector_type(4)));
        typedef __attribute__((address_space(3))) i16x4* lds_i16x4_ptr;
        const uint16_t* vrow = &tile_lds[buf * kBuf + kKTile + (4 * hg + (n16 >> 2)) * kPfVRow + 4 * (n16 & 3)];
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) {
            const i16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4_ptr)(vrow + 16 * dt));
            const i16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4_ptr)(vrow + 16 * kPfVRow + 16 * dt));
            const uint2 lo2 = __builtin_bit_cast(uint2, lo), hi2 = __builtin_bit_cast(uint2, hi);
            const uint4 va = make_uint4(lo2.x, lo2.y, hi2.x, hi2.y);
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
                acc[rb][dt] = mfma_qk<DT>(va, make_uint4(pk[rb][0], pk[rb][1], pk[rb][2], pk[rb][3]), acc[rb][dt]);
                if (PfSoftmax<DT>::kSplitWeights)
                    acc[rb][dt] = mfma_qk<DT>(va, make_uint4(pk_lo[rb][0], pk_lo[rb][1], pk_lo[rb][2], pk_lo[rb][3]), acc[rb][dt]);
            }
        }

    };

    const int pos_min = pos0 + tq0;                             // tiles ending at or below it need no causal mask

    fetch_tile(stage, kt0);
    store_tile(stage, kt0 & 1);
    fetch_tile(stage, kt0 + 1);
    __syncthreads();
    // Tiles wholly inside every row's visible range need no mask: those that end at or below the
    // first row's position (causal side) and start at or above the last row's window start.
    const int n_unmasked = min(ntiles, max(0, (pos_min + 1) / kPfKeys));
    const int n_window_cut = W > 0 ? (max(kmax - W, 0) + kPfKeys - 1) / kPfKeys : 0;
    // (three plain loops rather than one with a branch in it: the compiler schedules the loads of a
    // loop whose body is one straight line far better)
    auto run_tiles = [&](int from, int to, auto masked) __attribute__((always_inline)) {
        for (int kt = from; kt < to; ++kt) {
            compute_tile(kt, kt & 1, masked);
            if (kt + 1 < ntiles) store_tile(stage, (kt + 1) & 1);
            fetch_tile(stage, kt + 2);
            __syncthreads();
        }
    };
    const int cut_end = max(kt0, min(n_window_cut, n_unmasked));   // tiles cut by some row's window start
    const int plain_end = max(cut_end, n_unmasked);                // tiles no mask touches
    if (WIN) run_tiles(kt0, cut_end, std::true_type{});
    run_tiles(cut_end, plain_end, std::false_type{});
    run_tiles(plain_end, ntiles, std::true_type{});

    // ---- normalise and write: this lane holds dims 16dt + 4hg + v of its row --------------------
    uint16_t* __restrict__ op = static_cast<uint16_t*>(p.out);
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        float lt = lsum[rb];
        lt += __shfl_xor(lt, 16);
        lt += __shfl_xor(lt, 32);
        if (!row_ok[rb]) continue;
        const float inv = p.out_scale / lt;
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) {
            uint2 packed;
            packed.x = narrow2<DT>(acc[rb][dt][0] * inv, acc[rb][dt][1] * inv);
            packed.y = narrow2<DT>(acc[rb][dt][2] * inv, acc[rb][dt][3] * inv);
            *reinterpret_cast<uint2*>(op + out_off[rb] + 16 * dt + 4 * hg) = packed;
        }
    }
}

}  // namespace optgqa
