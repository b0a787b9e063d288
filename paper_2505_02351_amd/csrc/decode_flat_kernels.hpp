// Paged decode attention (head_dim 128 or 64) with the context split by EQUAL WORK instead of by
// fixed-size partitions (Section III-A splits the context into partitions whose results are
// carried forward and merged; here the partition boundaries are chosen so that every wave of
// the launch streams the same number of K/V bytes).
//
// Why: decode is a pure stream over the cache, and with drawn context lengths a fixed partition
// size leaves a ragged tail - late workgroups still hold a full partition while the rest of the
// chip idles - plus a start-up and a merge per workgroup.  Here the launch is exactly one
// resident wave per hardware wave slot, and the work is cut into that many equal pieces:
//
//   tiles      16 consecutive tokens of one (sequence b, KV head / head chunk y) "segment";
//              sequence b has n_b = ceil(L_b / 16) tiles per segment and Y segments
//   flat order F(b, y, tau) = Y * P_b + y * n_b + tau,  P_b = sum_{b' < b} n_b',  T = Y * P_B
//   unit u     (one wave) owns flat tiles [u*c, min((u+1)*c, T)),  c = ceil(T / U)
//
// A unit's range is a short list of pieces, each inside one segment; per piece the wave runs a
// register-prefetched matrix-core loop (K/V tiles fetched one tile ahead straight into VGPRs, as
// in the unsplit kernel of decode_mma_kernels.hpp) and leaves one partial result (reference, weight sum,
// un-normalised output) for the combine kernel.  The pairs
// (unit, segment) that occur form a staircase, so slot = u + s (s = b*Y + y) numbers them
// without collisions and without any bookkeeping: at most U + B*Y slots.
//
// Nothing is planned on the host (the context lengths live in device memory): every wave scans
// the context lengths itself (two memory round trips for any batch size), and the wave that
// processes the first tile of a sequence records P_b for the combine kernel.
//
// Arithmetic.  Unlike the unsplit kernel (fp32 output MFMAs, 32 per tile), both
// contractions here are 16-bit MFMAs, computed transposed so that no operand is transposed in
// registers (the scheme of the tiled prefill kernel): S^T = K Q^T leaves a lane with the scores of
// four tokens of ONE head, which after the softmax are exactly its slice of the B operand of
// O^T += V^T P^T; V^T is read with the transposing LDS load from a per-wave LDS copy of the V rows
// of two tiles.  The output contraction thus runs once per 32 tokens with 8 (fp16) or 16 (bf16)
// MFMAs of 16 cycles, where the fp32 version spent 64 MFMAs of 32 cycles - measured, that alone
// was 6 us of a 122 us launch (the matrix pipes' activity slows the stream even though the
// kernel is memory-bound).  Weights are rounded to the input type for this: fp16 keeps its
// softmax reference within 2^14 of the running maximum, bf16 splits every weight into head +
// tail (see prefill_kernels.hpp for the error budget); either way the normaliser is the sum of
// the weights AS ROUNDED, so the output stays an exact convex combination of V rows.
#pragma once
#include <type_traits>

#include "decode_mma_kernels.hpp"

namespace optgqa {

#ifndef OPTGQA_FLAT_WGS_PER_CU
#define OPTGQA_FLAT_WGS_PER_CU 1
#endif
#ifndef OPTGQA_FLAT_WGS_PER_CU_KV8
#define OPTGQA_FLAT_WGS_PER_CU_KV8 2      // workgroups per CU (= waves per SIMD) for 8-bit caches
#endif
#ifndef OPTGQA_FLAT_WAVES_PER_SIMD
#define OPTGQA_FLAT_WAVES_PER_SIMD 2
#endif

// LDS V row, elements: head_dim + 16, i.e. 288 bytes (see prefill_kernels.hpp, same reason) or 160 - either
// way the four rows that a group of 16 lanes transposes, and the next group's four, fall in distinct banks
template <int D> struct FlatRow { static constexpr int kV = D + 16; };

// What a wave can park in LDS before it has to write it out: the results of up to kStagePieces
// pieces, kStageCols query-head columns in all (one piece of a shared prefix, two at 8 heads per KV
// head, five at 4).  Sized so that two workgroups still fit a CU's LDS.
constexpr int kStagePieces = 5, kStageCols = 20, kStageHdrInts = 16;

// How far the softmax reference may lag behind the running maximum before the accumulators are
// rescaled, and how far above the maximum it is then put.  16-bit weights: fp16 must keep them
// inside its range; bf16 has the range but not the precision, so its weights are split in two.
template <int DT> struct FlatSoftmax;
template <> struct FlatSoftmax<kF16> {
    static constexpr float kThreshold = 14.f, kHeadroom = 2.f;
    static constexpr bool kSplitWeights = false;
};
template <> struct FlatSoftmax<kBF16> {
    static constexpr float kThreshold = kRescaleThreshold, kHeadroom = kRescaleHeadroom;
    static constexpr bool kSplitWeights = true;
};

// First token a decode query of a sequence of length L sees: with a sliding window of W > 0
// tokens (Alg. 1, local mask) the last W ones, positions L - W .. L - 1; W <= 0: all of them.
__device__ __forceinline__ int flat_first_token(int L, int W) { return W > 0 ? max(L - W, 0) : 0; }

// Tiles of one segment of a sequence of length L.  Plain: the 16-token tiles of the cache that
// hold a visible token (tile indices first_token / 16 .. (L - 1) / 16).  FUSED (the step's cache
// write happens inside the call): the same over the tokens already in the cache, L - 1 of
// them, plus - 2-byte caches - one tile that holds only the new token (8-bit caches: the new
// token's term is added by the combine kernel, no tile).
template <bool FUSED, bool KV8 = false> __device__ __forceinline__ int flat_tiles(int L, int W)
{
    if (L <= 0) return 0;
    const int lo = flat_first_token(L, W);
    const int reg = FUSED ? L - 1 : L;                          // tokens read from the cache
    const int regular = reg > lo ? (reg + kMmaTile - 1) / kMmaTile - lo / kMmaTile : 0;
    return regular + (FUSED && !KV8 ? 1 : 0);
}

__device__ __forceinline__ int wave_inclusive_scan(int x, int lane)
{
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int y = __shfl_up(x, off);
        if (lane >= off) x += y;
    }
    return x;
}

// ---- shared prefixes (Section III-B: cached key-value blocks are shared and reused) --------------
// Sequences whose block tables start with the same physical blocks (a common prompt) need those
// blocks read only once if their queries are batched against the shared tiles.  The score MFMA has
// 16 query-head columns and a KV head's group fills GH of them, so `bundle` = 16 / GH sequences ride
// through one pass: sequences come in aligned bundles of that many consecutive ones, led by
// sequence b0 = b - b % bundle, and shared_blocks[b] > 0 says that the first shared_blocks[b]
// block-table entries of b are the leader's.  The bundle's shared prefix is the part EVERY taking-part
// member shares: S tokens, a multiple of 16, never beyond any member's cached tokens.
//
// The flat order then runs over 2 * num_seqs "virtual sequences": v = 2b is the shared prefix of
// the bundle that b leads (tokens 0 .. S-1 through the leader's table, all members' heads in the
// columns; no tiles unless b is a leader with S > 0), v = 2b + 1 is what b reads alone (tokens S ..,
// or 0 .. if b shares nothing, and its new token's tile in the fused step).  Slots, plan entries
// and the staircase are indexed by v instead of b; every slot holds 16 columns.
template <bool UNIFORM> __device__ __forceinline__ int flat_ld(const int32_t* ptr)
{
    // wave-uniform addresses inside the streaming loop go through the scalar cache: a vector load
    // would make the wave wait for every tile load still in flight
    if constexpr (UNIFORM) return scalar_load_i32(ptr);
    else return *ptr;
}

template <bool UNIFORM>
__device__ __forceinline__ int shared_prefix_tokens(const DecodeParams& p, int b0, int fused)
{
    const int L0 = flat_ld<UNIFORM>(p.context_lens + b0);
    int S = 0x7fffffff;
    bool any = false;
    for (int i = 1; i < p.bundle && b0 + i < p.num_seqs; ++i) {
        const int s = flat_ld<UNIFORM>(p.shared_blocks + b0 + i), Li = flat_ld<UNIFORM>(p.context_lens + b0 + i);
        if (s > 0 && Li > 0) {
            any = true;
            S = min(S, min(s * p.block_size, Li - fused));
        }
    }
    if (!any || L0 <= 0) return 0;
    return max(min(S, L0 - fused), 0) & ~(kMmaTile - 1);
}

// What the segments of one (virtual) sequence cover: cached tokens [lo, hi) read through the block
// table of sequence tb, plus - fused step over 2-byte caches, not for a shared prefix - a last tile
// that is the new token of sequence b alone.  n = tiles per segment.
struct FlatSeg {
    int b, tb, L, lo, hi, n;
    int shared;             // (an int: a struct with padding bytes does not stay in registers)
};


template <bool FUSED, bool KV8, bool SHARED, bool UNIFORM>
__device__ __forceinline__ FlatSeg flat_seg(const DecodeParams& p, int v)
{
    FlatSeg s;
    if constexpr (!SHARED) {
        s.b = s.tb = v;
        s.L = flat_ld<UNIFORM>(p.context_lens + v);
        s.lo = flat_first_token(s.L, p.window);
        s.hi = FUSED ? s.L - 1 : s.L;
        s.shared = 0;
        s.n = flat_tiles<FUSED, KV8>(s.L, p.window);
    } else {
        const int b = v >> 1;
        const int b0 = b - b % p.bundle;
        const int S = shared_prefix_tokens<UNIFORM>(p, b0, FUSED ? 1 : 0);
        s.b = b;
        s.L = flat_ld<UNIFORM>(p.context_lens + b);
        s.shared = (v & 1) == 0 ? 1 : 0;
        if (s.shared) {
            s.tb = b0;
            s.lo = 0;
            s.hi = b == b0 ? S : 0;
            s.n = s.hi / kMmaTile;
        } else {
            const bool takes_part = S > 0 && (b == b0 || flat_ld<UNIFORM>(p.shared_blocks + b) > 0);
            s.tb = b;
            s.lo = takes_part ? S : 0;
            s.hi = FUSED ? s.L - 1 : s.L;
            s.n = s.L <= 0 ? 0 : (s.hi > s.lo ? (s.hi + kMmaTile - 1) / kMmaTile - s.lo / kMmaTile : 0) + (FUSED && !KV8 ? 1 : 0);
        }
    }
    return s;
}

//
// FUSED: the kernel also performs the step's cache write (Alg. 2 stores the new K/V, then attends
// over the cache).  The new token of sequence b is its last one; it is given a tile of its own at
// the end of every segment (so the tiles of the cache cover positions 0 .. L - 2 only), which the
// wave that gets it reads from k_new / v_new - a wave-uniform choice of base address, nothing per
// lane - and the wave that finishes a KV head's segment copies the row into the cache.  No wave
// reads that cache row during the launch, so there is nothing to order.
//
// KV8: the caches hold 1-byte E4M3 codes (largest finite value 448, no infinities) instead of
// 2-byte elements, with one scale per tensor: k_scale is folded into the score scale on the host,
// v_scale into the combine kernel's normalisation.  A token row is then 128 bytes; a lane's
// 16-byte K piece holds 16 consecutive dims and feeds two score MFMAs after widening to DT
// (exact: every E4M3 value is an fp16 and a bf16 number), a lane's 8-byte V piece widens to 8 DT
// values on its way into the LDS copy.  Not combined with FUSED.
//
// SHARED: shared prefixes are read once per bundle of sequences (above).  2-byte caches, no window.
//
// PARTS: fixed partitions (Section III-A: the context is cut into partitions of a given size whose
// results are merged) on the equal-work machinery: pieces end where a unit or a segment ends AND
// at every multiple of part_tiles tiles inside a segment, so no piece spans two partitions.  The
// waves still stream equal shares, with the prefetch chained from one partition to the next.  A
// unit is at least one partition long, so a unit boundary cuts a partition into at most two
// fragments: partition pi of segment (b, y) leaves its partial results in slots
// ((b * Y + y) * num_partitions + pi) * 2 + (0: the fragment that starts the partition, 1: the
// rest, if a unit boundary fell inside).  Plain attention over 2-byte caches only.
//
// Head dimension D (128 or 64).  A K row is D / 32 sixteen-byte pieces per lane group hg, one score MFMA each;
// a V tile (16 rows of D elements) is fetched D / 8 lanes to a row, 512 / D rows per load, D / 32 loads;
// the output is D / 16 blocks of 16 dims.
template <int D> struct FlatTile {
    uint4 k[D / 32];    // K: token j16, dims 32i + 8hg .. +7
    uint4 v[D / 32];    // V: token (512 / D) * r + lane / (D / 8), dims 8 * (lane % (D / 8)) .. +7
};
template <int D> struct FlatTile8 {
    uint4 k[D / 64];    // K: token j16, dims 64j + 16hg .. +15
    uint2 v[D / 32];    // V: as above, 8 one-byte codes
};

template <int DT, bool FUSED, bool KV8 = false, bool SHARED = false, bool PARTS = false, int D = 128>
__global__ __launch_bounds__(kDecodeWaves * 64, KV8 ? OPTGQA_FLAT_WGS_PER_CU_KV8 : OPTGQA_FLAT_WAVES_PER_SIMD) void paged_decode_flat_kernel(const DecodeParams p)
{
    static_assert(D == 128 || D == 64, "head_dim 128 or 64");
    static_assert(!(SHARED && KV8), "shared prefixes: 2-byte caches");
    static_assert(!(PARTS && (FUSED || KV8 || SHARED)), "fixed partitions: plain attention over 2-byte caches");
    constexpr bool NEW_TILE = FUSED && !KV8;            // the new token is a tile of its own, read from k_new / v_new
    typedef typename std::conditional<KV8, FlatTile8<D>, FlatTile<D>>::type Tile;
    constexpr int ES = KV8 ? 1 : 2;                     // bytes per cache element
    constexpr int TILE = kMmaTile;
    constexpr int kFlatVRow = FlatRow<D>::kV;
    constexpr int NQ = D / 32;                          // score MFMAs per tile (32 dims each)
    constexpr int NDB = D / 16;                         // 16-dim blocks of the output
    constexpr int LPR = D / 8;                          // lanes that fetch one V row (8 elements each)
    constexpr int RPL = 64 / LPR;                       // V rows per load
    constexpr int NVL = TILE / RPL;                     // V loads per tile
    static_assert(kMmaBufs == 2, "two register tile buffers: one in use, one in flight");

    // per wave: the V rows of two consecutive tiles (32 tokens) in their natural [token][dim] layout
    __shared__ __attribute__((aligned(16))) uint16_t v_lds[kDecodeWaves][2 * TILE][kFlatVRow];
    // per wave: what finished pieces leave behind, parked until the unit ends (see "side effects" below)
    constexpr int SROW = D + 4;                         // floats per parked column: D outputs, reference, weight sum; the
                                                        // odd stride spreads the columns over the LDS banks
    __shared__ __attribute__((aligned(16))) float st_lds[kDecodeWaves][kStageCols * SROW];
    __shared__ int st_hdr[kDecodeWaves][kStagePieces][kStageHdrInts];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int j16 = lane & 15;
    const int hg = lane >> 4;
    const int vcol = lane % LPR, vrow0 = lane / LPR;    // this lane's piece of a V tile: rows RPL * r + vrow0, dims 8 * vcol .. +7

    const int B = p.num_seqs, Y = p.segs_per_seq;
    const int NV = SHARED ? 2 * B : B;                  // (virtual) sequences of the flat order
    const int Hq = p.num_heads, Hkv = p.num_kv_heads, bs = p.block_size;
    const int bs_shift = __builtin_ctz(bs);
    const int GH = p.heads_per_wg;
    const int G = Hq / Hkv;
    const int chunks = G / GH;
    const int CS = SHARED ? 16 : GH;                    // columns (query heads) per partial-result slot
    const int u = blockIdx.x * kDecodeWaves + wave;
    const int32_t* __restrict__ ctx = p.context_lens;
    const int W = p.window;
    const int tp = PARTS ? p.part_tiles : 0;            // tiles per fixed partition

    // ---- where does this unit start?  level 1: lane i sums the tiles of sequences [i*k, (i+1)*k)
    const int k = (NV + 63) >> 6;
    int mine = 0, my_len = 0;
    for (int i = 0; i < k; ++i) {
        const int idx = lane * k + i;
        if constexpr (SHARED) {
            if (idx < NV) mine += flat_seg<FUSED, KV8, true, false>(p, idx).n;
        } else {
            my_len = idx < B ? ctx[idx] : 0;
            mine += flat_tiles<FUSED, KV8>(my_len, W);
        }
    }
    const int incl = wave_inclusive_scan(mine, lane);
    const int P_total = __builtin_amdgcn_readlane(incl, 63);
    const int T = Y * P_total;
    const int c = max(PARTS ? tp : 1, (T + p.num_units - 1) / p.num_units);     // (PARTS: at least one partition)
    const int f0 = u * c;
    const int f1 = min(f0 + c, T);
    if (f0 >= f1) return;                                   // no workgroup-wide barrier below

    // the lane whose chunk holds flat tile f0: the last one whose chunk starts at or before it
    const int cl = __builtin_popcountll(__builtin_amdgcn_ballot_w64(Y * (incl - mine) <= f0)) - 1;
    int v = cl * k;                                         // (virtual) sequence of the piece at hand
    int P_v = __builtin_amdgcn_readlane(incl - mine, cl);
    FlatSeg seg;
    if (k == 1) {
        if constexpr (SHARED) {
            seg = flat_seg<FUSED, KV8, true, true>(p, v);
        } else {
            seg.b = seg.tb = v;
            seg.n = __builtin_amdgcn_readlane(mine, cl);
            seg.L = __builtin_amdgcn_readlane(my_len, cl);
            seg.lo = flat_first_token(seg.L, W);
            seg.hi = FUSED ? seg.L - 1 : seg.L;
            seg.shared = 0;
        }
    } else {
        // level 2: the k sequences of that chunk, 64 at a time
        int n = 0;
        for (int base = 0; base < k; base += 64) {
            const int idx = cl * k + base + lane;
            const bool in = base + lane < k && idx < NV;
            int nl;
            if constexpr (SHARED) nl = in ? flat_seg<FUSED, KV8, true, false>(p, idx).n : 0;
            else nl = flat_tiles<FUSED, KV8>(in ? ctx[idx] : 0, W);
            const int inc2 = wave_inclusive_scan(nl, lane);
            const int tot = __builtin_amdgcn_readlane(inc2, 63);
            if (Y * (P_v + tot) > f0) {
                const int x = __builtin_popcountll(__builtin_amdgcn_ballot_w64(Y * (P_v + inc2 - nl) <= f0)) - 1;
                P_v += __builtin_amdgcn_readlane(inc2 - nl, x);
                n = __builtin_amdgcn_readlane(nl, x);
                v = cl * k + base + x;
                break;
            }
            P_v += tot;
        }
        if (n <= 0) return;                                 // cannot happen for consistent lengths
        seg = flat_seg<FUSED, KV8, SHARED, true>(p, v);
        if (seg.n != n) return;                             // the lengths changed under the kernel
    }
    if (seg.n <= 0) return;                                 // (as above)
    int y, tau;
    {
        const int r = f0 - Y * P_v;
        y = r / seg.n;
        tau = r - y * seg.n;
    }

    const uint16_t* __restrict__ qp = static_cast<const uint16_t*>(p.q);
    const unsigned char* __restrict__ kc = static_cast<const unsigned char*>(p.k_cache);
    const unsigned char* __restrict__ vc = static_cast<const unsigned char*>(p.v_cache);
    const unsigned char* __restrict__ k_new = static_cast<const unsigned char*>(p.k_new);
    const unsigned char* __restrict__ v_new = static_cast<const unsigned char*>(p.v_new);
    const int64_t block_stride = (int64_t)Hkv * bs * D;

    // Where a tile comes from, in wave-uniform terms: the byte address of its first K / V row, the
    // last row that exists (later rows re-read it and are masked out of the scores), and the tokens
    // it stands for.  A regular tile is 16 consecutive tokens of one physical block.  FUSED: the
    // last tile of a segment is the new token alone, read from k_new / v_new (row 0, nothing else).
    struct TileSrc {
        const unsigned char* k;
        const unsigned char* v;
        int last_row;           // >= 0
        int tok0;               // row r is token tok0 + r ...
        int rel0, span;         // ... and visible if 0 <= rel0 + r < span (first visible token .. end of the piece)
    };
    // (segment: block table row, element offset of the KV head inside a block, first cached token
    //  its tiles cover, length of the sequence, tiles, whether its last tile is the new token;
    //  reg_end: end of the regular tokens the piece covers; new_k / new_v: element offsets of the
    //  sequence's new rows in k_new / v_new, FUSED only; ti counts from the segment's first tile,
    //  the one that holds token lo)
    auto tile_src = [&](const int32_t* tab, int64_t head_off, int lo, int Lseg, int nseg, bool has_new, int reg_end,
                        int64_t new_k, int64_t new_v, int ti) __attribute__((always_inline)) {
        TileSrc s;
        if (NEW_TILE && has_new && ti == nseg - 1) {
            s.k = k_new + new_k * 2;
            s.v = v_new + new_v * 2;
            s.last_row = 0;
            s.tok0 = Lseg - 1;
            s.rel0 = 0;
            s.span = 1;
        } else {
            const int t0 = (ti + lo / TILE) * TILE;
            // through the scalar cache: a vector load here would make the wave wait for every tile
            // load still in flight before it could read the block number
            const int blk = scalar_load_i32(tab + (t0 >> bs_shift));
            const int64_t uni = blk * block_stride + head_off + (int64_t)(t0 & (bs - 1)) * D;
            s.k = kc + uni * ES;
            s.v = vc + uni * ES;
            s.last_row = max(reg_end - 1 - t0, 0);
            s.tok0 = t0;
            s.rel0 = t0 - lo;
            s.span = reg_end - lo;
        }
        return s;
    };
    // The tile's bytes into operand order: no branches, rows clamped.
    // (lane offsets are unsigned 32-bit on top of the tile's wave-uniform address, so that the loads
    // take that address from scalar registers and no 64-bit vector arithmetic is spent on them)
    auto load_tile = [&](Tile& Tl, const TileSrc& s) __attribute__((always_inline)) {
        const uint32_t last = (uint32_t)s.last_row;
        const uint32_t ko = min((uint32_t)j16, last) * (uint32_t)(D * ES) + 16u * (uint32_t)hg;
        if constexpr (KV8) {
#pragma unroll
            for (int j = 0; j < D / 64; ++j) Tl.k[j] = stream_load16(s.k + (ko + 64u * j));
#pragma unroll
            for (int r = 0; r < NVL; ++r)
                Tl.v[r] = stream_load8(s.v + (min((uint32_t)(RPL * r + vrow0), last) * (uint32_t)D + 8u * (uint32_t)vcol));
        } else {
#pragma unroll
            for (int i = 0; i < NQ; ++i) Tl.k[i] = stream_load16(s.k + (ko + 64u * i));
#pragma unroll
            for (int r = 0; r < NVL; ++r)
                Tl.v[r] = stream_load16(s.v + (min((uint32_t)(RPL * r + vrow0), last) * (uint32_t)(D * 2) + 16u * (uint32_t)vcol));
        }
    };
    // B operand of the score MFMAs for segment (sg, yy) - lane (column j16, k-slab hg) holds dims
    // 32i + 8hg .. +7 of its column's query row, unused columns zero - with that head's slope (base 2)
    // and the position of that query (the ALiBi term is relative to it).  A column is head j16 of the
    // segment's GH heads; in a shared prefix, head j16 % GH of the bundle's member j16 / GH.
    auto load_q = [&](uint4 (&qd)[NQ], float& sd, int& pos, int sg_b, int sg_L, bool sg_shared, int yy) __attribute__((always_inline)) {
        const int gg = yy / chunks;
        const int hh0 = gg * G + (yy - gg * chunks) * GH;
        int col_b = sg_b, col_h = min(j16, GH - 1);
        bool ok = j16 < GH;
        pos = sg_L - 1;
        if constexpr (SHARED) {
            if (sg_shared) {
                const int i = j16 / GH;                      // member of the bundle (sg_b is its leader)
                col_h = j16 - i * GH;
                ok = i < p.bundle && sg_b + i < B;
                col_b = min(sg_b + i, B - 1);
                const int Li = ctx[col_b];
                if (i > 0) ok = ok && p.shared_blocks[col_b] > 0 && Li > 0;
                pos = Li - 1;
            }
        }
        // (2-byte caches: MFMA i contracts dims 32i + 8hg .. +7; E4M3 caches: dims
        // 64(i/2) + 16hg + 8(i%2) .. +7, the order in which a lane's 16-byte K pieces arrive)
        const uint16_t* qrow = qp + ((int64_t)col_b * Hq + hh0 + col_h) * D + (KV8 ? 16 : 8) * hg;
        const uint32_t keep = ok ? 0xffffffffu : 0u;
#pragma unroll
        for (int i = 0; i < NQ; ++i) {
            const uint4 x = *reinterpret_cast<const uint4*>(qrow + (KV8 ? 64 * (i >> 1) + 8 * (i & 1) : 32 * i));
            qd[i] = make_uint4(x.x & keep, x.y & keep, x.z & keep, x.w & keep);
        }
        float sl = 0.f;
        if (p.slopes) sl = p.slopes[hh0 + col_h];
        sd = ok ? sl * kLog2e : 0.f;
    };

    Tile buf[2];
    TileSrc d0, d1;               // what buf[0] / buf[1] hold (or are receiving)
    uint4 qa[NQ];
    float slope2;                 // ALiBi slope (base 2) of column j16
    int q_pos;                    // position of column j16's query: its sequence's last token
    // (see "side effects" in the piece loop)
    auto side_effects = [&](int fx, int64_t row, int64_t new_k, int64_t new_v, int vv, int P_vv) __attribute__((always_inline)) {
        if constexpr (NEW_TILE) {
            if ((fx & 1) && lane < 2 * LPR) {                // LPR lanes move the K row, the next LPR the V row
                const int piece = 8 * vcol;
                const unsigned char* src = lane < LPR ? k_new + (new_k + piece) * 2 : v_new + (new_v + piece) * 2;
                uint16_t* dstp = (lane < LPR ? static_cast<uint16_t*>(p.k_cache_w) : static_cast<uint16_t*>(p.v_cache_w)) + row + piece;
                *reinterpret_cast<uint4*>(dstp) = *reinterpret_cast<const uint4*>(src);
            }
        }
        if (lane == 0) {
            if (fx & 2) p.plan[vv] = P_vv;
            if (fx & 4) p.plan[NV] = c;
        }
    };
    auto flush = [&](int count) __attribute__((always_inline)) {
        for (int k = 0; k < count; ++k) {
            const int* h = &st_hdr[wave][k][0];
            const int64_t slot = (int64_t)(((uint64_t)(uint32_t)h[1] << 32) | (uint32_t)h[0]);
            const int ncols = h[2];
            side_effects(h[3], (int64_t)(((uint64_t)(uint32_t)h[5] << 32) | (uint32_t)h[4]),
                         (int64_t)(((uint64_t)(uint32_t)h[7] << 32) | (uint32_t)h[6]),
                         (int64_t)(((uint64_t)(uint32_t)h[9] << 32) | (uint32_t)h[8]), h[10], h[11]);
            if (j16 < ncols) {
                const float* st = &st_lds[wave][0] + (h[12] + j16) * SROW;
                const int64_t e0 = slot * CS + j16;
                if (hg == 0) {
                    p.ws_m[e0] = st[D];
                    p.ws_l[e0] = st[D + 1];
                }
                float* o = p.ws_o + e0 * D + 4 * hg;
#pragma unroll
                for (int db = 0; db < NDB; ++db)
                    *reinterpret_cast<float4*>(o + 16 * db) = *reinterpret_cast<const float4*>(st + 16 * db + 4 * hg);
            }
        }
    };
    int staged = 0, staged_cols = 0;    // pieces parked in LDS, and the columns they take
    bool chained = false;         // buf[0] / d0 were filled by the previous piece
    bool same_q = false;          // ... and it was a piece of the same segment (PARTS): qa, slope2, q_pos still hold
    int f = f0;
    for (;;) {
        // ---- one piece: tiles [tau, tau_end) of segment (v, y) -------------------------------
        const int n = seg.n, L = seg.L, lo = seg.lo;
        const bool has_new = NEW_TILE && !(SHARED && seg.shared);   // the segment's last tile is the new token
        // (PARTS: a piece also ends where its partition ends)
        const int tau_end = min(PARTS ? min(n, (tau / tp + 1) * tp) : n, tau + (f1 - f));
        const int ntw = tau_end - tau;                      // >= 1
        const int j_last = ntw - 1;
        const int Lm1 = L - 1;
        // regular (cached) tokens the piece covers end here
        const int first = lo / TILE;                        // the segment's tiles start at this tile of the cache
        const int reg_end = min(seg.hi, ((has_new && tau_end == n ? tau_end - 1 : tau_end) + first) * TILE);
        const int g = y / chunks;
        // score scale (base 2); E4M3 caches with per-KV-head scales: times this KV head's k_scale
        float scale2 = p.scale2;
        if constexpr (KV8) {
            if (p.k_scales) scale2 *= __builtin_bit_cast(float, scalar_load_i32(reinterpret_cast<const int32_t*>(p.k_scales + g)));
        }
        const int32_t* table = p.block_tables + (int64_t)seg.tb * p.max_blocks_per_seq;
        const int64_t head_off = (int64_t)g * bs * D;
        const int64_t new_k = NEW_TILE ? seg.b * p.k_new_stride + (int64_t)g * D : 0;
        const int64_t new_v = NEW_TILE ? seg.b * p.v_new_stride + (int64_t)g * D : 0;

        if (!(PARTS && same_q)) load_q(qa, slope2, q_pos, seg.b, seg.L, seg.shared != 0, y);
        if (!chained) {
            d0 = tile_src(table, head_off, lo, L, n, has_new, reg_end, new_k, new_v, tau);
            load_tile(buf[0], d0);
        }
        // ---- side effects of the piece, none of which anything in this launch reads: its partial
        // result; the new token's K / V rows into the cache if the piece ends a KV head's segment (Alg. 2,
        // the cache store); P_v of a (virtual) sequence and the unit length, for the combine kernel.
        // A store in the middle of the stream would hold up the wave: loads complete in issue order
        // with stores, so the first tile fetched after a store cannot be used before the store is
        // acknowledged, several tile times later on a busy memory system.  All of them are therefore
        // parked in LDS (results) and in a header (the rest) and written after the unit's last tile.
        int fx = 0;
        int64_t fx_row = 0;                                  // element offset of the new token's cache row
        if (has_new && tau_end == n && y == g * chunks) {
            const int blk = scalar_load_i32(table + (Lm1 >> bs_shift));
            fx_row = blk * block_stride + head_off + (int64_t)(Lm1 & (bs - 1)) * D;
            fx |= 1;
        }
        if (y == 0 && tau == 0) fx |= 2;                     // plan[v] = P_v
        if (f == 0) fx |= 4;                                 // plan[NV] = c

        // ---- the piece after this one (same unit), so that its first tile is on its way before this
        // piece ends.  Without one, the spare prefetch slot re-reads this piece's last tile (a cache
        // hit, never consumed).
        bool has_next = f + ntw < f1;                        // (not PARTS: then this piece ends its segment)
        int nv = v, ny = y;
        int ntau = 0;                                        // first tile of the next piece in its segment
        FlatSeg nseg = seg;
        if (PARTS && has_next && tau_end < n) {
            ntau = tau_end;                                  // the next partition of the same segment
        } else if (has_next) {
            if (++ny == Y) {
                ny = 0;
                do {                                         // skip sequences without tiles
                    ++nv;
                    nseg = flat_seg<FUSED, KV8, SHARED, true>(p, nv);
                } while (nseg.n == 0 && nv + 1 < NV);
                if (nseg.n == 0) {                           // cannot happen for consistent lengths
                    has_next = false;
                    nv = v, ny = y, nseg = seg;
                }
            }
        }
        // arguments of tile_src for "the tile after this piece": the next piece's first one, or
        // (nothing follows) this piece's last one again
        const int nn = nseg.n;
        const bool n_has_new = NEW_TILE && !(SHARED && nseg.shared);
        const int n_tau_end = min(PARTS ? min(nn, (ntau / tp + 1) * tp) : nn, ntau + f1 - (f + ntw));
        const int32_t* x_table = has_next ? p.block_tables + (int64_t)nseg.tb * p.max_blocks_per_seq : table;
        const int64_t x_head_off = has_next ? (int64_t)(ny / chunks) * bs * D : head_off;
        const int x_L = has_next ? nseg.L : L, x_n = has_next ? nn : n, x_lo = has_next ? nseg.lo : lo;
        const bool x_has_new = has_next ? n_has_new : has_new;
        const int n_first = nseg.lo / TILE;
        const int x_reg_end = !has_next ? reg_end
                              : min(nseg.hi, ((n_has_new && n_tau_end == nn ? n_tau_end - 1 : n_tau_end) + n_first) * TILE);
        const int64_t x_new_k = !has_next ? new_k : NEW_TILE ? nseg.b * p.k_new_stride + (int64_t)(ny / chunks) * D : 0;
        const int64_t x_new_v = !has_next ? new_v : NEW_TILE ? nseg.b * p.v_new_stride + (int64_t)(ny / chunks) * D : 0;
        const int x_ti = has_next ? ntau : tau + j_last;

        // ---- both contractions on 16-bit MFMAs, transposed so that nothing is transposed in registers:
        //   S^T[token][head] = K Q^T : A = the K tile as fetched (lane (token j16, slab hg)), B = the query
        //       rows; a lane ends up with the scores of tokens 4hg + v (v = 0..3) for ONE head, j16.
        //   O^T[dim][head] += V^T P^T over 32 tokens (two tiles): B = this lane's own 8 weights (4 of the
        //       even tile, 4 of the odd one) rounded to DT; A = V^T, read out of the wave's LDS copy of
        //       the V rows with the transposing LDS load (see prefill_kernels.hpp for its lane layout).
        // The output MFMAs therefore run once per two tiles, 8 (fp16) or 16 (bf16, weights split in
        // a head and a tail) of them, instead of 32 fp32 MFMAs per tile.
        float m_ref = kNoMax;                 // reference of head j16 (equal in the 4 lanes that share it)
        float pend[4] = {0.f, 0.f, 0.f, 0.f}; // weights of the even tile, waiting for the odd one
        f32x4 lsum = f32x4{0.f, 0.f, 0.f, 0.f};
        f32x4 acc[NDB];                       // O^T: dims 16db + 4hg + v of head j16
#pragma unroll
        for (int e = 0; e < NDB; ++e) acc[e] = f32x4{0.f, 0.f, 0.f, 0.f};
        uint16_t* const v_rows = &v_lds[wave][0][0];
        typedef short i16x4 __attribute__((ext_vector_type(4)));
        typedef __attribute__((address_space(3))) i16x4* lds_i16x4_ptr;
        // position the ALiBi term is relative to: the segment's sequence, or (shared prefix) the column's
        const int rel_pos = SHARED ? q_pos : Lm1;

        auto weighted_sum = [&](const float (&w_even)[4], const float (&w_odd)[4]) __attribute__((always_inline)) {
            uint32_t hi[4], lo[4] = {0u, 0u, 0u, 0u};
            if (FlatSoftmax<DT>::kSplitWeights) {
                split_bf16(w_even[0], w_even[1], hi[0], lo[0]);
                split_bf16(w_even[2], w_even[3], hi[1], lo[1]);
                split_bf16(w_odd[0], w_odd[1], hi[2], lo[2]);
                split_bf16(w_odd[2], w_odd[3], hi[3], lo[3]);
            } else {
                hi[0] = narrow2<DT>(w_even[0], w_even[1]);
                hi[1] = narrow2<DT>(w_even[2], w_even[3]);
                hi[2] = narrow2<DT>(w_odd[0], w_odd[1]);
                hi[3] = narrow2<DT>(w_odd[2], w_odd[3]);
            }
            const uint4 ph = make_uint4(hi[0], hi[1], hi[2], hi[3]);
            const uint4 pl = make_uint4(lo[0], lo[1], lo[2], lo[3]);
            // sum of the weights as rounded (the output stays an exact convex combination of V rows)
            const uint32_t one2 = DT == kF16 ? 0x3c003c00u : 0x3f803f80u;
            const uint4 ones = make_uint4(one2, one2, one2, one2);
            lsum = mfma_qk<DT>(ones, ph, lsum);
            if (FlatSoftmax<DT>::kSplitWeights) lsum = mfma_qk<DT>(ones, pl, lsum);
            const uint16_t* vrow = v_rows + (4 * hg + (j16 >> 2)) * kFlatVRow + 4 * (j16 & 3);
#pragma unroll
            for (int db = 0; db < NDB; ++db) {
                const i16x4 r0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4_ptr)(vrow + 16 * db));
                const i16x4 r1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4_ptr)(vrow + 16 * kFlatVRow + 16 * db));
                const uint2 a0 = __builtin_bit_cast(uint2, r0), a1 = __builtin_bit_cast(uint2, r1);
                const uint4 va = make_uint4(a0.x, a0.y, a1.x, a1.y);
                acc[db] = mfma_qk<DT>(va, ph, acc[db]);
                if (FlatSoftmax<DT>::kSplitWeights) acc[db] = mfma_qk<DT>(va, pl, acc[db]);
            }
        };

        auto compute_tile = [&](const Tile& Tl, const TileSrc& src, auto odd_tile) __attribute__((always_inline)) {
            constexpr bool ODD = decltype(odd_tile)::value;
            // the tile's V rows go to LDS as they are (rows 16*ODD + RPL*r + vrow0, this lane's 8 dims)
#pragma unroll
            for (int r = 0; r < NVL; ++r) {
                uint4 vr;
                if constexpr (KV8) vr = widen8_e4m3<DT>(Tl.v[r].x, Tl.v[r].y);
                else vr = Tl.v[r];
                *reinterpret_cast<uint4*>(v_rows + (16 * ODD + RPL * r + vrow0) * kFlatVRow + 8 * vcol) = vr;
            }
            f32x4 S = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int i = 0; i < NQ; ++i) {
                if constexpr (KV8) {
                    const uint4 kk = Tl.k[i >> 1];
                    S = mfma_qk<DT>((i & 1) ? widen8_e4m3<DT>(kk.z, kk.w) : widen8_e4m3<DT>(kk.x, kk.y), qa[i], S);
                } else {
                    S = mfma_qk<DT>(Tl.k[i], qa[i], S);
                }
            }
            const int t0 = src.tok0 + 4 * hg;
            const int r0 = src.rel0 + 4 * hg;
            float x[4];
            bool need = false;
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4) {
                const int t = t0 + v4;
                // one unsigned compare covers both ends: rows before the first visible token and rows past the piece
                const bool visible = (unsigned)(r0 + v4) < (unsigned)src.span;
                x[v4] = visible ? fmaf(S[v4], scale2, slope2 * (float)(t - rel_pos)) : -INFINITY;   // eq. (3), base 2
                need |= x[v4] > m_ref + FlatSoftmax<DT>::kThreshold;
            }
            if (__builtin_expect(__builtin_amdgcn_ballot_w64(need) != 0, 0)) {   // rare: the reference moves lazily
                float mx = fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3]));
                mx = fmaxf(mx, __shfl_xor(mx, 16));              // a head's tokens live in 4 lanes (hg)
                mx = fmaxf(mx, __shfl_xor(mx, 32));
                const float m_new = fmaxf(m_ref, mx + FlatSoftmax<DT>::kHeadroom);
                const float alpha = fast_exp2(m_ref - m_new);    // 1 when unchanged, 0 on first use
                m_ref = m_new;
                lsum *= alpha;
#pragma unroll
                for (int v4 = 0; v4 < 4; ++v4) pend[v4] *= alpha;
#pragma unroll
                for (int e = 0; e < NDB; ++e) acc[e] *= alpha;
            }
            float w[4];
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4) w[v4] = fast_exp2(x[v4] - m_ref);                          // eq. (4) numerators
            if constexpr (ODD) {
                weighted_sum(pend, w);
            } else {
#pragma unroll
                for (int v4 = 0; v4 < 4; ++v4) pend[v4] = w[v4];
            }
        };

        // Two tiles per trip; every half issues exactly one tile of loads (no branches around
        // loads, so the number in flight at each use is a compile-time constant).  The first half
        // prefetches into buf[1], the second into buf[0]; past the end of the piece the second half
        // fetches the next piece's first tile, which is therefore always found in buf[0].
        const int trips = (ntw + 1) >> 1;
        for (int it = 0; it < trips; ++it) {
            const int j = 2 * it;
            d1 = tile_src(table, head_off, lo, L, n, has_new, reg_end, new_k, new_v, tau + min(j + 1, j_last));
            load_tile(buf[1], d1);
            compute_tile(buf[0], d0, std::false_type{});
            const bool more = j + 2 <= j_last;
            d0 = tile_src(more ? table : x_table, more ? head_off : x_head_off, more ? lo : x_lo, more ? L : x_L,
                          more ? n : x_n, more ? has_new : x_has_new, more ? reg_end : x_reg_end,
                          more ? new_k : x_new_k, more ? new_v : x_new_v, more ? tau + j + 2 : x_ti);
            load_tile(buf[0], d0);
            if (j + 1 <= j_last) {
                compute_tile(buf[1], d1, std::true_type{});
            } else {
                // odd number of tiles: the last even tile has no partner; give it rows of zeros
#pragma unroll
                for (int r = 0; r < NVL; ++r)
                    *reinterpret_cast<uint4*>(v_rows + (16 + RPL * r + vrow0) * kFlatVRow + 8 * vcol) = make_uint4(0u, 0u, 0u, 0u);
                const float none[4] = {0.f, 0.f, 0.f, 0.f};
                weighted_sum(pend, none);
            }
        }

        // ---- the piece's partial result belongs in slot u + s (s = v * Y + y): this lane holds dims
        // 16db + 4hg + v of column j16 ---------------------------------------------------------------
        const int64_t slot = PARTS ? ((((int64_t)v * Y + y) * p.num_partitions + tau / tp) << 1) + (tau % tp != 0)
                                   : (int64_t)u + (int64_t)v * Y + y;
        const int ncols = SHARED && seg.shared ? CS : GH;    // (a shared prefix fills all 16 columns of its slots)
        if (has_next) {
            if (staged == kStagePieces || staged_cols + ncols > kStageCols) {    // no room: write out what is parked
                flush(staged);
                staged = staged_cols = 0;
            }
            if (j16 < ncols) {
                float* st = &st_lds[wave][0] + (staged_cols + j16) * SROW;
#pragma unroll
                for (int db = 0; db < NDB; ++db)
                    *reinterpret_cast<float4*>(st + 16 * db + 4 * hg) = make_float4(acc[db][0], acc[db][1], acc[db][2], acc[db][3]);
                if (hg == 0) {
                    st[D] = m_ref;
                    st[D + 1] = lsum[0];
                }
            }
            if (lane == 0) {
                int* h = &st_hdr[wave][staged][0];
                h[0] = (int)(uint32_t)slot, h[1] = (int)(slot >> 32), h[2] = ncols, h[3] = fx;
                h[4] = (int)(uint32_t)fx_row, h[5] = (int)(fx_row >> 32);
                h[6] = (int)(uint32_t)new_k, h[7] = (int)(new_k >> 32);
                h[8] = (int)(uint32_t)new_v, h[9] = (int)(new_v >> 32);
                h[10] = v, h[11] = P_v, h[12] = staged_cols;
            }
            ++staged;
            staged_cols += ncols;
        } else {
            // the unit's last piece: straight from the registers, then everything that was parked
            side_effects(fx, fx_row, new_k, new_v, v, P_v);
            if (j16 < ncols) {
                const int64_t e0 = slot * CS + j16;
                if (hg == 0) {
                    p.ws_m[e0] = m_ref;
                    p.ws_l[e0] = lsum[0];
                }
                float* o = p.ws_o + e0 * D + 4 * hg;
#pragma unroll
                for (int db = 0; db < NDB; ++db)
                    *reinterpret_cast<float4*>(o + 16 * db) = make_float4(acc[db][0], acc[db][1], acc[db][2], acc[db][3]);
            }
            flush(staged);
            break;
        }

        // ---- next piece ------------------------------------------------------------------------
        f += ntw;
        if (ny != y || nv != v) {                            // the next piece starts a segment
            if (y + 1 == Y) P_v += n;                        // sequences skipped on the way have no tiles
        }
        same_q = nv == v && ny == y;
        v = nv, y = ny, seg = nseg, tau = ntau;
        chained = true;
    }
}

// Combine the partial results of the equal-work split: head h of sequence b collects slots
// u + s for the units u that touched its segment (a contiguous range found from P_v, n_v and c).
// Same arithmetic as the fixed-partition combine:
//   M = max_u m_u,  out = sum_u 2^(m_u-M) o_u / sum_u 2^(m_u-M) l_u.
//
// NEWTOK (decode step over E4M3 caches): the step's new token was not among the streamed tiles.
// Its term is added here from k_new / v_new - quantised exactly as the cache write quantises,
// so that it is the cache's own codes that are attended to - and the thread that holds dims
// od .. od + 3 of a KV head's first query head stores the four K and four V codes into the caches
// (Alg. 2, the cache-store step: nothing in the step has read that cache row).
//
// SHARED: a head's partial results lie in two staircases - the pieces of its own segment (virtual
// sequence 2b + 1, column = the head) and, if the sequence takes part in its bundle's shared
// prefix, the pieces of that segment (virtual sequence 2 * leader, column = member * GH + head).
template <int DT, bool NEWTOK = false, bool SHARED = false, int D = 128>
__global__ __launch_bounds__(kReduceThreads) void paged_decode_flat_reduce_kernel(const DecodeParams p)
{
    static_assert(!(NEWTOK && SHARED), "shared prefixes: 2-byte caches");
    constexpr int kVecPerHead = D / 4;
    constexpr int kHeads = kReduceThreads / kVecPerHead;
    const int h = blockIdx.y * kHeads + threadIdx.x / kVecPerHead;
    const int od = (threadIdx.x % kVecPerHead) * 4;
    const int b = blockIdx.x;                                // (sequences along x: no 16-bit limit)
    if (h >= p.num_heads) return;
    uint16_t* o = static_cast<uint16_t*>(p.out) + ((int64_t)b * p.num_heads + h) * D + od;
    const int NV = SHARED ? 2 * p.num_seqs : p.num_seqs;
    const int v_own = SHARED ? 2 * b + 1 : b;
    // (this kernel is a few dependent memory round trips and little else: the three values that
    // everything else depends on are fetched together, before the first branch)
    const int L = p.context_lens[b];
    const int plan_total = p.plan[NV], plan_own = p.plan[v_own];      // readable garbage where nobody wrote them
    if (L <= 0) {
        *reinterpret_cast<uint2*>(o) = make_uint2(0u, 0u);
        return;
    }
    const int GH = p.heads_per_wg;
    const int CS = SHARED ? 16 : GH;                         // columns per slot
    const int G = p.num_heads / p.num_kv_heads;
    const int chunks = G / GH;
    const int g = h / G;
    // NEWTOK: the new token's rows, the query and the block of the new row are fetched first, so that
    // they arrive while the partial results are being read
    uint2 kw = make_uint2(0u, 0u), vw = kw, qw = kw;
    int new_blk = 0;
    if constexpr (NEWTOK) {
        kw = *reinterpret_cast<const uint2*>(static_cast<const uint16_t*>(p.k_new) + (int64_t)b * p.k_new_stride + (int64_t)g * D + od);
        vw = *reinterpret_cast<const uint2*>(static_cast<const uint16_t*>(p.v_new) + (int64_t)b * p.v_new_stride + (int64_t)g * D + od);
        qw = *reinterpret_cast<const uint2*>(static_cast<const uint16_t*>(p.q) + ((int64_t)b * p.num_heads + h) * D + od);
        new_blk = p.block_tables[(int64_t)b * p.max_blocks_per_seq + (L - 1) / p.block_size];
    }
    const int within = h - g * G;
    const int chunk = within / GH;
    const int hh = within - chunk * GH;
    const int Y = p.segs_per_seq;
    const int y = g * chunks + chunk;
    const int c = max(plan_total, 1);
    // the numbering the main kernel used
    int n_own, n_shared = 0, col_shared = 0, plan_shared = 0, v_shared = 0;
    if constexpr (SHARED) {
        const bool fused = p.k_new != nullptr;
        const int b0 = b - b % p.bundle;
        const int S = shared_prefix_tokens<false>(p, b0, fused ? 1 : 0);
        const bool takes_part = S > 0 && (b == b0 || p.shared_blocks[b] > 0);
        const int lo = takes_part ? S : 0, hi = fused ? L - 1 : L;
        n_own = (hi > lo ? (hi + kMmaTile - 1) / kMmaTile - lo / kMmaTile : 0) + (fused ? 1 : 0);
        if (takes_part) {
            n_shared = S / kMmaTile;
            v_shared = 2 * b0;
            col_shared = (b - b0) * GH + hh;
            plan_shared = p.plan[v_shared];
        }
    } else {
        n_own = NEWTOK ? flat_tiles<true, true>(L, p.window)
                       : p.k_new ? flat_tiles<true>(L, p.window) : flat_tiles<false>(L, p.window);
    }
    // One pass in batches of 8 partial results with a running reference (a segment rarely has more
    // than 8 pieces, so this is one memory round trip; a separate pass for the maximum would be
    // a second chain of them).
    float M = -INFINITY;
    float den = 0.f;
    float4 num = make_float4(0.f, 0.f, 0.f, 0.f);
    bool any = false;                                        // something has been accumulated
    // the pieces of segment y of (virtual) sequence vv, which has n tiles per segment and tile prefix P
    auto collect = [&](int vv, int n, int P, int col) __attribute__((always_inline)) {
        int np = 0;
        int64_t base = 0;
        {
            // (the clamps only matter if the lengths changed under the kernels: they keep every read
            // inside the workspace; n == 0: nothing was streamed, nobody wrote the plan entry)
            const int F0 = n > 0 ? Y * P + y * n : 0;
            const int u0 = min(max(F0 / c, 0), p.num_units - 1);
            np = n > 0 ? min(max((F0 + n - 1) / c - u0 + 1, 1), p.num_units - u0) : 0;
            base = ((int64_t)u0 + (int64_t)vv * Y + y) * CS + col;          // slot stride between units: CS
        }
        for (int i0 = 0; i0 < np; i0 += 8) {
            float mm[8], ll[8];
            float4 x[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int64_t e = base + (int64_t)min(i0 + k, np - 1) * CS;
                mm[k] = p.ws_m[e];
                ll[k] = p.ws_l[e];
                x[k] = *reinterpret_cast<const float4*>(p.ws_o + e * D + od);
            }
            float Mn = M;                                            // clamped repeats of the last piece do not change it
#pragma unroll
            for (int k = 0; k < 8; ++k) Mn = fmaxf(Mn, mm[k]);
            const float keep = any ? fast_exp2(M - Mn) : 0.f;        // nothing accumulated before the first batch
            any = true;
            M = Mn;
            den *= keep;
            num.x *= keep;
            num.y *= keep;
            num.z *= keep;
            num.w *= keep;
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const float fct = i0 + k < np ? fast_exp2(mm[k] - M) : 0.f;
                den = fmaf(fct, ll[k], den);
                num.x = fmaf(fct, x[k].x, num.x);
                num.y = fmaf(fct, x[k].y, num.y);
                num.z = fmaf(fct, x[k].z, num.z);
                num.w = fmaf(fct, x[k].w, num.w);
            }
        }
    };
    collect(v_own, n_own, plan_own, hh);
    if constexpr (SHARED) collect(v_shared, n_shared, plan_shared, col_shared);
    // E4M3 caches with per-KV-head scales: this head's pair
    const float k_scale_g = p.k_scales ? p.k_scales[g] : 1.f, v_scale_g = p.v_scales ? p.v_scales[g] : 1.f;
    if constexpr (NEWTOK) {
        // the new token, at the query's own position (ALiBi term 0): codes, their values, its score
        const float k_inv = p.k_scales ? 1.0f / k_scale_g : p.k_inv_scale, v_inv = p.v_scales ? 1.0f / v_scale_g : p.v_inv_scale;
        const uint32_t kcodes = e4m3_codes2(widen_lo<DT>(kw.x) * k_inv, widen_hi<DT>(kw.x) * k_inv) |
                                e4m3_codes2(widen_lo<DT>(kw.y) * k_inv, widen_hi<DT>(kw.y) * k_inv) << 16;
        const uint32_t vcodes = e4m3_codes2(widen_lo<DT>(vw.x) * v_inv, widen_hi<DT>(vw.x) * v_inv) |
                                e4m3_codes2(widen_lo<DT>(vw.y) * v_inv, widen_hi<DT>(vw.y) * v_inv) << 16;
        const f32x2 k01 = __builtin_amdgcn_cvt_pk_f32_fp8(kcodes, false), k23 = __builtin_amdgcn_cvt_pk_f32_fp8(kcodes, true);
        const f32x2 v01 = __builtin_amdgcn_cvt_pk_f32_fp8(vcodes, false), v23 = __builtin_amdgcn_cvt_pk_f32_fp8(vcodes, true);
        float dot = widen_lo<DT>(qw.x) * k01[0];
        dot = fmaf(widen_hi<DT>(qw.x), k01[1], dot);
        dot = fmaf(widen_lo<DT>(qw.y), k23[0], dot);
        dot = fmaf(widen_hi<DT>(qw.y), k23[1], dot);
#pragma unroll
        for (int off = 1; off < kVecPerHead; off <<= 1) dot += __shfl_xor(dot, off);      // a head's threads: an aligned half or quarter of a wave
        const float s_new = dot * (p.scale2 * k_scale_g);                                 // eq. (3), base 2, k_scale folded in
        const float M2 = fmaxf(M, s_new);
        const float f_old = any ? fast_exp2(M - M2) : 0.f, f_new = fast_exp2(s_new - M2);
        den = fmaf(den, f_old, f_new);
        num.x = fmaf(num.x, f_old, f_new * v01[0]);
        num.y = fmaf(num.y, f_old, f_new * v01[1]);
        num.z = fmaf(num.z, f_old, f_new * v23[0]);
        num.w = fmaf(num.w, f_old, f_new * v23[1]);
        if (h == g * G) {
            const int pos = L - 1;
            const int64_t dst = (((int64_t)new_blk * p.num_kv_heads + g) * p.block_size + pos % p.block_size) * D + od;
            *reinterpret_cast<uint32_t*>(static_cast<unsigned char*>(p.k_cache_w) + dst) = kcodes;
            *reinterpret_cast<uint32_t*>(static_cast<unsigned char*>(p.v_cache_w) + dst) = vcodes;
        }
    }
    const float inv = p.out_scale * v_scale_g / den;     // out_scale: 1, or the v_scale of an E4M3 cache
    uint2 packed;
    packed.x = narrow2<DT>(num.x * inv, num.y * inv);
    packed.y = narrow2<DT>(num.z * inv, num.w * inv);
    *reinterpret_cast<uint2*>(o) = packed;
}

// Combine for fixed partitions run by the equal-work kernel (PARTS): head h of sequence b has two
// slots per partition, ((b * Y + y) * num_partitions + pi) * 2 + fragment; fragment 0 (the piece that
// starts the partition) always exists, fragment 1 only if a unit boundary - a multiple of c in the
// flat order - fell strictly inside the partition.  One workgroup per (head, sequence): eight groups of
// head_dim / 4 threads (4 output dims each) take every eighth slot with all their loads in flight at once,
// then the eight partial sums are merged through LDS - a long context has dozens of partitions and
// a single chain of memory round trips over them would cost more than the streaming they merge.
constexpr int kPartsReduceGroups = 8;

template <int DT, int D = 128>
__global__ __launch_bounds__(kPartsReduceGroups * (D / 4)) void paged_decode_parts_reduce_kernel(const DecodeParams p)
{
    constexpr int GW = D / 4;                                          // threads per group: 4 output dims each
    __shared__ float s_m[kPartsReduceGroups][GW], s_den[kPartsReduceGroups][GW];
    __shared__ float4 s_num[kPartsReduceGroups][GW];
    const int h = blockIdx.y, b = blockIdx.x;
    const int l32 = threadIdx.x % GW, grp = threadIdx.x / GW;
    const int od = l32 * 4;
    uint16_t* o = static_cast<uint16_t*>(p.out) + ((int64_t)b * p.num_heads + h) * D + od;
    const int L = p.context_lens[b];
    const int c = max(p.plan[p.num_seqs], 1), P = p.plan[b];          // readable garbage where nobody wrote them
    if (L <= 0) {                                                      // (uniform over the workgroup)
        if (grp == 0) *reinterpret_cast<uint2*>(o) = make_uint2(0u, 0u);
        return;
    }
    const int GH = p.heads_per_wg;
    const int G = p.num_heads / p.num_kv_heads;
    const int chunks = G / GH;
    const int g = h / G;
    const int within = h - g * G;
    const int chunk = within / GH;
    const int hh = within - chunk * GH;
    const int Y = p.segs_per_seq;
    const int y = g * chunks + chunk;
    const int tp = p.part_tiles;
    const int n = flat_tiles<false>(L, 0);
    const int parts = min((n + tp - 1) / tp, p.num_partitions);
    const int64_t first = (((int64_t)b * Y + y) * p.num_partitions) << 1;
    const int64_t F0 = (int64_t)Y * P + (int64_t)y * n;
    float M = -INFINITY, den = 0.f;
    float4 num = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int i0 = grp; i0 < 2 * parts; i0 += 8 * kPartsReduceGroups) {
        float mm[8], ll[8];
        float4 x[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int i = i0 + k * kPartsReduceGroups, pi = i >> 1;
            const int64_t start = F0 + (int64_t)pi * tp, len = min(tp, n - pi * tp);
            const bool there = i < 2 * parts && ((i & 1) == 0 || (start / c + 1) * c < start + len);
            const int64_t e = (first + i) * GH + hh;
            mm[k] = there ? p.ws_m[e] : -INFINITY;
            ll[k] = there ? p.ws_l[e] : 0.f;
            x[k] = there ? *reinterpret_cast<const float4*>(p.ws_o + e * D + od) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
        float Mn = M;
#pragma unroll
        for (int k = 0; k < 8; ++k) Mn = fmaxf(Mn, mm[k]);
        const float keep = Mn > -INFINITY ? fast_exp2(M - Mn) : 0.f;      // (M = -inf before the first slot: keep 0)
        M = Mn;
        den *= keep;
        num.x *= keep;
        num.y *= keep;
        num.z *= keep;
        num.w *= keep;
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const float fct = mm[k] > -INFINITY ? fast_exp2(mm[k] - M) : 0.f;
            den = fmaf(fct, ll[k], den);
            num.x = fmaf(fct, x[k].x, num.x);
            num.y = fmaf(fct, x[k].y, num.y);
            num.z = fmaf(fct, x[k].z, num.z);
            num.w = fmaf(fct, x[k].w, num.w);
        }
    }
    s_m[grp][l32] = M;
    s_den[grp][l32] = den;
    s_num[grp][l32] = num;
    __syncthreads();
    if (grp != 0) return;
    float Mt = -INFINITY;
#pragma unroll
    for (int k = 0; k < kPartsReduceGroups; ++k) Mt = fmaxf(Mt, s_m[k][l32]);
    float dt = 0.f;
    float4 nt = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int k = 0; k < kPartsReduceGroups; ++k) {
        const float mk = s_m[k][l32];
        const float fct = mk > -INFINITY ? fast_exp2(mk - Mt) : 0.f;
        const float4 nk = s_num[k][l32];
        dt = fmaf(fct, s_den[k][l32], dt);
        nt.x = fmaf(fct, nk.x, nt.x);
        nt.y = fmaf(fct, nk.y, nt.y);
        nt.z = fmaf(fct, nk.z, nt.z);
        nt.w = fmaf(fct, nk.w, nt.w);
    }
    const float inv = p.out_scale / dt;
    uint2 packed;
    packed.x = narrow2<DT>(nt.x * inv, nt.y * inv);
    packed.y = narrow2<DT>(nt.z * inv, nt.w * inv);
    *reinterpret_cast<uint2*>(o) = packed;
}

}  // namespace optgqa
