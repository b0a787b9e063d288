// Paged decode attention for head_dim 128 with the context split by EQUAL WORK instead of by
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
// A unit's range is a short list of pieces, each inside one segment; per piece the wave runs the
// same register-prefetched matrix-core loop as the fixed-partition kernel and leaves one partial
// result (reference, weight sum, un-normalised output) for the combine kernel.  The pairs
// (unit, segment) that occur form a staircase, so slot = u + s (s = b*Y + y) numbers them
// without collisions and without any bookkeeping: at most U + B*Y slots.
//
// Nothing is planned on the host (the context lengths live in device memory): every wave scans
// the context lengths itself (two memory round trips for any batch size), and the wave that
// processes the first tile of a sequence records P_b for the combine kernel.
#pragma once
#include <type_traits>

#include "decode_mma_kernels.hpp"

namespace optgqa {

#ifndef OPTGQA_FLAT_WGS_PER_CU
#define OPTGQA_FLAT_WGS_PER_CU 1
#endif
#ifndef OPTGQA_FLAT_WAVES_PER_SIMD
#define OPTGQA_FLAT_WAVES_PER_SIMD 2
#endif

__device__ __forceinline__ int flat_tiles(int L) { return (max(L, 0) + kMmaTile - 1) / kMmaTile; }

__device__ __forceinline__ int wave_inclusive_scan(int x, int lane)
{
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int y = __shfl_up(x, off);
        if (lane >= off) x += y;
    }
    return x;
}

//
// FUSED: the kernel also performs the step's cache write (Alg. 2 stores the new K/V, then attends
// over the cache).  The new token of sequence b is its last one; whichever wave handles the tile
// that contains it takes that row from k_new / v_new instead of the cache (a per-lane pointer
// select), and the wave that finishes a KV head's segment copies the row into the cache.  No
// wave reads that cache row during the launch, so there is nothing to order.
//
// KV8: the caches hold 1-byte E4M3 codes (largest finite value 448, no infinities) instead of
// 2-byte elements, with one scale per tensor: k_scale is folded into the score scale on the host,
// v_scale into the combine kernel's normalisation.  A token row is then 128 bytes; a lane's
// 16-byte K piece holds 16 consecutive dims and feeds two score MFMAs after widening to DT
// (exact: every E4M3 value is an fp16 and a bf16 number), a lane's 8-byte V piece widens to the
// same 8 fp32 values per lane as before.  Not combined with FUSED.
struct MmaTile8 {
    uint4 k[2];     // K: token j16, dims 64j + 16hg .. +15
    uint2 v[4];     // V: token 4s + hg, dims 8*j16 .. +7
};

typedef float f32x2 __attribute__((ext_vector_type(2)));

// eight E4M3 codes (two dwords) -> eight DT values (one MFMA operand)
template <int DT> __device__ __forceinline__ uint4 widen8_e4m3(uint32_t lo, uint32_t hi)
{
    const f32x2 a = __builtin_amdgcn_cvt_pk_f32_fp8(lo, false), b = __builtin_amdgcn_cvt_pk_f32_fp8(lo, true);
    const f32x2 c = __builtin_amdgcn_cvt_pk_f32_fp8(hi, false), d = __builtin_amdgcn_cvt_pk_f32_fp8(hi, true);
    return make_uint4(narrow2<DT>(a[0], a[1]), narrow2<DT>(b[0], b[1]), narrow2<DT>(c[0], c[1]), narrow2<DT>(d[0], d[1]));
}

template <int DT, bool FUSED, bool KV8 = false>
__global__ __launch_bounds__(kDecodeWaves * 64, OPTGQA_FLAT_WAVES_PER_SIMD) void paged_decode_flat_kernel(const DecodeParams p)
{
    static_assert(!(FUSED && KV8), "the fused cache write exists for 2-byte caches only");
    typedef typename std::conditional<KV8, MmaTile8, MmaTile>::type Tile;
    constexpr int ES = KV8 ? 1 : 2;                     // bytes per cache element
    constexpr int D = 128;
    constexpr int TILE = kMmaTile;
    constexpr int NB = kMmaBufs;
    constexpr int PT = NB - 1;

    __shared__ __attribute__((aligned(16))) float p_lds[kDecodeWaves][TILE][kMmaMaxHeads];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int j16 = lane & 15;
    const int hg = lane >> 4;
#ifdef OPTGQA_FLAT_TIMING
    const unsigned long long tm0 = wall_clock64();
    unsigned long long tm1 = 0, tm2 = 0;
#endif

    const int B = p.num_seqs, Y = p.segs_per_seq;
    const int Hq = p.num_heads, Hkv = p.num_kv_heads, bs = p.block_size;
    const int bs_shift = __builtin_ctz(bs);
    const int GH = p.heads_per_wg;
    const int G = Hq / Hkv;
    const int chunks = G / GH;
    const int u = blockIdx.x * kDecodeWaves + wave;
    const int32_t* __restrict__ ctx = p.context_lens;

    // ---- where does this unit start?  level 1: lane i sums the tiles of sequences [i*k, (i+1)*k)
    const int k = (B + 63) >> 6;
    int mine = 0, my_len = 0;
    for (int i = 0; i < k; ++i) {
        const int idx = lane * k + i;
        my_len = idx < B ? ctx[idx] : 0;
        mine += flat_tiles(my_len);
    }
    const int incl = wave_inclusive_scan(mine, lane);
    const int P_total = __builtin_amdgcn_readlane(incl, 63);
    const int T = Y * P_total;
    const int c = max(1, (T + p.num_units - 1) / p.num_units);
    const int f0 = u * c;
    const int f1 = min(f0 + c, T);
    if (f0 >= f1) return;                                   // no workgroup-wide barrier below

    // the lane whose chunk holds flat tile f0: the last one whose chunk starts at or before it
    const int cl = __builtin_popcountll(__builtin_amdgcn_ballot_w64(Y * (incl - mine) <= f0)) - 1;
    int b = cl * k;
    int P_b = __builtin_amdgcn_readlane(incl - mine, cl);
    int n, L;                                               // tiles per segment / length of sequence b
    if (k == 1) {
        n = __builtin_amdgcn_readlane(mine, cl);
        L = __builtin_amdgcn_readlane(my_len, cl);
    } else {
        // level 2: the k sequences of that chunk, 64 at a time
        n = 0;
        L = 0;
        for (int base = 0; base < k; base += 64) {
            const int idx = cl * k + base + lane;
            const int nl = flat_tiles(base + lane < k && idx < B ? ctx[idx] : 0);
            const int inc2 = wave_inclusive_scan(nl, lane);
            const int tot = __builtin_amdgcn_readlane(inc2, 63);
            if (Y * (P_b + tot) > f0) {
                const int x = __builtin_popcountll(__builtin_amdgcn_ballot_w64(Y * (P_b + inc2 - nl) <= f0)) - 1;
                P_b += __builtin_amdgcn_readlane(inc2 - nl, x);
                n = __builtin_amdgcn_readlane(nl, x);
                b = cl * k + base + x;
                L = __builtin_amdgcn_readfirstlane(ctx[b]);
                break;
            }
            P_b += tot;
        }
        if (n <= 0) return;                                 // cannot happen for consistent lengths
    }
    int y, tau;
    {
        const int r = f0 - Y * P_b;
        y = r / n;
        tau = r - y * n;
    }

    const uint16_t* __restrict__ qp = static_cast<const uint16_t*>(p.q);
    const unsigned char* __restrict__ kc = static_cast<const unsigned char*>(p.k_cache);
    const unsigned char* __restrict__ vc = static_cast<const unsigned char*>(p.v_cache);
    const float scale2 = p.scale2;
    const int64_t block_stride = (int64_t)Hkv * bs * D;
    float* const pw_write = &p_lds[wave][j16][4 * hg];
    const float* const pw_read = &p_lds[wave][hg][j16];

    // One 16-token tile of a segment into operand order.  All 16 tokens lie in one physical block;
    // rows past t_last (the piece's last token) re-read that row and are masked out of the scores.
    const uint16_t* __restrict__ k_new = static_cast<const uint16_t*>(p.k_new);
    const uint16_t* __restrict__ v_new = static_cast<const uint16_t*>(p.v_new);
    // (new_pos, new_off_k, new_off_v: position of the segment's new token and where its K / V
    // rows start in k_new / v_new; only read when FUSED)
    auto load_tile = [&](Tile& Tl, const int32_t* tab, int64_t head_off, int t_last, int tile_t0,
                         int new_pos, int64_t new_off_k, int64_t new_off_v) __attribute__((always_inline)) {
        // through the scalar cache: a vector load here would make the wave wait for every tile
        // load still in flight before it could read the block number
        const int blk = scalar_load_i32(tab + (tile_t0 >> bs_shift));
        const int64_t uni = blk * block_stride + head_off + (int64_t)(tile_t0 & (bs - 1)) * D;
        const int tk = min(tile_t0 + j16, t_last) - tile_t0;
        if constexpr (KV8) {
            const unsigned char* ka = kc + uni + tk * D + 16 * hg;
#pragma unroll
            for (int j = 0; j < 2; ++j) Tl.k[j] = *reinterpret_cast<const uint4*>(ka + 64 * j);
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const int tv = min(tile_t0 + 4 * s + hg, t_last) - tile_t0;
                Tl.v[s] = *reinterpret_cast<const uint2*>(vc + uni + tv * D + 8 * j16);
            }
        } else {
            const unsigned char* ka = kc + (uni + tk * D + 8 * hg) * ES;
            if (FUSED && tile_t0 + tk == new_pos) ka = reinterpret_cast<const unsigned char*>(k_new + new_off_k + 8 * hg);
#pragma unroll
            for (int i = 0; i < 4; ++i) Tl.k[i] = *reinterpret_cast<const uint4*>(ka + 64 * i);
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const int tv = min(tile_t0 + 4 * s + hg, t_last) - tile_t0;
                const unsigned char* va = vc + (uni + tv * D + 8 * j16) * ES;
                if (FUSED && tile_t0 + tv == new_pos) va = reinterpret_cast<const unsigned char*>(v_new + new_off_v + 8 * j16);
                Tl.v[s] = *reinterpret_cast<const uint4*>(va);
            }
        }
    };
    // A operand of the score MFMAs for segment (bb, yy) - lane (head j16, k-slab hg) holds dims
    // 32i + 8hg .. +7 of its head, rows >= GH zero - and the slopes (base 2) of heads 4hg + v.
    auto load_q = [&](uint4 (&qd)[4], float (&sd)[4], int bb, int yy) __attribute__((always_inline)) {
        const int gg = yy / chunks;
        const int hh0 = gg * G + (yy - gg * chunks) * GH;
        // (2-byte caches: MFMA i contracts dims 32i + 8hg .. +7; E4M3 caches: dims
        // 64(i/2) + 16hg + 8(i%2) .. +7, the order in which a lane's 16-byte K pieces arrive)
        const uint16_t* qrow = qp + ((int64_t)bb * Hq + hh0 + min(j16, GH - 1)) * D + (KV8 ? 16 : 8) * hg;
        const uint32_t keep = j16 < GH ? 0xffffffffu : 0u;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint4 x = *reinterpret_cast<const uint4*>(qrow + (KV8 ? 64 * (i >> 1) + 8 * (i & 1) : 32 * i));
            qd[i] = make_uint4(x.x & keep, x.y & keep, x.z & keep, x.w & keep);
        }
        float sl[4] = {0.f, 0.f, 0.f, 0.f};
        if (p.slopes) {
#pragma unroll
            for (int v = 0; v < 4; ++v) sl[v] = p.slopes[hh0 + min(4 * hg + v, GH - 1)];
        }
#pragma unroll
        for (int v = 0; v < 4; ++v) sd[v] = 4 * hg + v < GH ? sl[v] * kLog2e : 0.f;
    };

    static_assert(NB == 2, "the hand-over of the next piece's first tile assumes two register buffers");
    Tile buf[NB];
    uint4 qa[4], qn[4];
    float slope2[4], slope2n[4];
    bool chained = false;         // buf[0], qa, slope2 were filled by the previous piece
    int f = f0;
    for (;;) {
        // ---- one piece: tiles [tau, tau_end) of segment (b, y) -------------------------------
        const int tau_end = min(n, tau + (f1 - f));
        const int ntw = tau_end - tau;                      // >= 1
        const int j_last = ntw - 1;
        const int t_begin = tau * TILE;
        const int t_end = min(L, tau_end * TILE);
        const int t_last = t_end - 1;
        const int Lm1 = L - 1;
        const int g = y / chunks;
        const int32_t* table = p.block_tables + (int64_t)b * p.max_blocks_per_seq;
        const int64_t head_off = (int64_t)g * bs * D;
        const int64_t new_off_k = FUSED ? b * p.k_new_stride + (int64_t)g * D : 0;
        const int64_t new_off_v = FUSED ? b * p.v_new_stride + (int64_t)g * D : 0;

        if (!chained) {
            load_q(qa, slope2, b, y);
            load_tile(buf[0], table, head_off, t_last, t_begin, Lm1, new_off_k, new_off_v);
        }
        if (FUSED && tau_end == n && y == g * chunks) {
            // this piece ends the KV head's segment: store the new token's K and V rows (Alg. 2)
            const int blk = scalar_load_i32(table + (Lm1 >> bs_shift));
            const int64_t dst = blk * block_stride + head_off + (int64_t)(Lm1 & (bs - 1)) * D;
            if (lane < 32) {
                const int piece = 8 * (lane & 15);
                const uint16_t* src = lane < 16 ? k_new + new_off_k + piece : v_new + new_off_v + piece;
                uint16_t* dstp = (lane < 16 ? static_cast<uint16_t*>(p.k_cache_w) : static_cast<uint16_t*>(p.v_cache_w)) + dst + piece;
                *reinterpret_cast<uint4*>(dstp) = *reinterpret_cast<const uint4*>(src);
            }
        }
        if (lane == 0) {
            // the combine kernel needs P_b of every non-empty sequence and the unit length
            if (y == 0 && tau == 0) p.plan[b] = P_b;
            if (f == 0) p.plan[B] = c;
        }

        // ---- the piece after this one (same unit), so that its first tile and its query rows are
        // on their way before this piece ends.  Without one, the spare prefetch slot re-reads this
        // piece's last tile (a cache hit, never consumed).
        bool has_next = f + ntw < f1;                        // then this piece ends its segment
        int nb = b, ny = y, nL = L, nn = n;
        if (has_next) {
            if (++ny == Y) {
                ny = 0;
                do {                                         // skip sequences without tokens
                    ++nb;
                    nL = scalar_load_i32(ctx + nb);
                    nn = flat_tiles(nL);
                } while (nn == 0 && nb + 1 < B);
                if (nn == 0) {                               // cannot happen for consistent lengths
                    has_next = false;
                    nb = b, ny = y, nL = L, nn = n;
                }
            }
        }
        const int32_t* ntable = has_next ? p.block_tables + (int64_t)nb * p.max_blocks_per_seq : table;
        const int64_t nhead_off = has_next ? (int64_t)(ny / chunks) * bs * D : head_off;
        const int nt_last = has_next ? min(nL, min(nn, f1 - (f + ntw)) * TILE) - 1 : t_last;
        const int nt0 = has_next ? 0 : t_begin + j_last * TILE;
        const int64_t nnew_off_k = FUSED ? nb * p.k_new_stride + (int64_t)(ny / chunks) * D : 0;
        const int64_t nnew_off_v = FUSED ? nb * p.v_new_stride + (int64_t)(ny / chunks) * D : 0;
        load_q(qn, slope2n, nb, ny);

        float m_ref[4], l[4];
        f32x4 acc[8];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            m_ref[v] = kNoMax;
            l[v] = 0.f;
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = f32x4{0.f, 0.f, 0.f, 0.f};
        // the A operand of the output MFMA reads all 16 head columns: start them finite
        reinterpret_cast<float4*>(&p_lds[wave][0][0])[lane] = make_float4(0.f, 0.f, 0.f, 0.f);

        auto compute_tile = [&](const Tile& Tl, int j) __attribute__((always_inline)) {
#if defined(OPTGQA_FLAT_ABLATE) && OPTGQA_FLAT_ABLATE == 1
            // development only: consume the loads without arithmetic
            uint32_t x = 0;
            for (int i = 0; i < (KV8 ? 2 : 4); ++i) x ^= Tl.k[i].x ^ Tl.k[i].y ^ Tl.k[i].z ^ Tl.k[i].w;
            for (int i = 0; i < 4; ++i) x ^= Tl.v[i].x ^ Tl.v[i].y;
            acc[0][0] += __uint_as_float(x & 0x3fffffffu);
            l[0] += (float)j;
            return;
#endif
            f32x4 S = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if constexpr (KV8) {
                    const uint4 kk = Tl.k[i >> 1];
                    S = mfma_qk<DT>(qa[i], (i & 1) ? widen8_e4m3<DT>(kk.z, kk.w) : widen8_e4m3<DT>(kk.x, kk.y), S);
                } else {
                    S = mfma_qk<DT>(qa[i], Tl.k[i], S);
                }
            }
            const int t = t_begin + j * TILE + j16;
            const bool valid = t < t_end;
            const float rel = (float)(t - Lm1);
            float s2[4];
            bool need = false;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                s2[v] = valid ? fmaf(S[v], scale2, slope2[v] * rel) : -INFINITY;     // eq. (3), base 2
                need |= s2[v] > m_ref[v] + kRescaleThreshold;
            }
            if (__builtin_amdgcn_ballot_w64(need) != 0) {
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const float m_new = fmaxf(m_ref[v], row16_max(s2[v]) + kRescaleHeadroom);
                    const float alpha = fast_exp2(m_ref[v] - m_new);
                    m_ref[v] = m_new;
                    l[v] *= alpha;
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc[e][v] *= alpha;
                }
            }
            float4 pw;
            pw.x = fast_exp2(s2[0] - m_ref[0]);                                       // eq. (4) numerators
            pw.y = fast_exp2(s2[1] - m_ref[1]);
            pw.z = fast_exp2(s2[2] - m_ref[2]);
            pw.w = fast_exp2(s2[3] - m_ref[3]);
            l[0] += pw.x;
            l[1] += pw.y;
            l[2] += pw.z;
            l[3] += pw.w;
            *reinterpret_cast<float4*>(pw_write) = pw;
            float a[4];
#pragma unroll
            for (int s = 0; s < 4; ++s) a[s] = pw_read[4 * s * kMmaMaxHeads];
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                float vf[8];
                if constexpr (KV8) {
                    const f32x2 v01 = __builtin_amdgcn_cvt_pk_f32_fp8(Tl.v[s].x, false), v23 = __builtin_amdgcn_cvt_pk_f32_fp8(Tl.v[s].x, true);
                    const f32x2 v45 = __builtin_amdgcn_cvt_pk_f32_fp8(Tl.v[s].y, false), v67 = __builtin_amdgcn_cvt_pk_f32_fp8(Tl.v[s].y, true);
                    vf[0] = v01[0], vf[1] = v01[1], vf[2] = v23[0], vf[3] = v23[1];
                    vf[4] = v45[0], vf[5] = v45[1], vf[6] = v67[0], vf[7] = v67[1];
                } else {
                    const uint4 vr = Tl.v[s];
                    vf[0] = widen_lo<DT>(vr.x), vf[1] = widen_hi<DT>(vr.x), vf[2] = widen_lo<DT>(vr.y), vf[3] = widen_hi<DT>(vr.y);
                    vf[4] = widen_lo<DT>(vr.z), vf[5] = widen_hi<DT>(vr.z), vf[6] = widen_lo<DT>(vr.w), vf[7] = widen_hi<DT>(vr.w);
                }
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[e] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[s], vf[e], acc[e], 0, 0, 0);
            }
        };

        // Two tiles per trip; every half issues exactly one tile of loads (no branches around
        // loads, so the number in flight at each use is a compile-time constant).  The first half
        // prefetches into buf[1], the second into buf[0]; past the end of the piece the second half
        // fetches the next piece's first tile, which is therefore always found in buf[0].
        const int trips = (ntw + 1) >> 1;
        for (int it = 0; it < trips; ++it) {
            const int j = 2 * it;
            load_tile(buf[1], table, head_off, t_last, t_begin + min(j + 1, j_last) * TILE, Lm1, new_off_k, new_off_v);
            compute_tile(buf[0], j);
#ifdef OPTGQA_FLAT_TIMING
            if (tm1 == 0) tm1 = wall_clock64();
#endif
            const bool more = j + 2 <= j_last;
            load_tile(buf[0], more ? table : ntable, more ? head_off : nhead_off, more ? t_last : nt_last,
                      more ? t_begin + (j + 2) * TILE : nt0, more ? Lm1 : nL - 1, more ? new_off_k : nnew_off_k,
                      more ? new_off_v : nnew_off_v);
            if (j + 1 <= j_last) compute_tile(buf[1], j + 1);
        }

#ifdef OPTGQA_FLAT_TIMING
        tm2 = wall_clock64();
#endif
        // ---- leave the piece's partial result in slot u + s ----------------------------------
#pragma unroll
        for (int v = 0; v < 4; ++v) l[v] = row_group_sum<16>(l[v]);
        const int64_t slot = (int64_t)u + (int64_t)b * Y + y;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int hh = 4 * hg + v;
            if (hh < GH) {
                const int64_t e0 = slot * GH + hh;
                if (j16 == 0) {
                    p.ws_m[e0] = m_ref[v];
                    p.ws_l[e0] = l[v];
                }
                float* o = p.ws_o + e0 * D + 8 * j16;
                *reinterpret_cast<float4*>(o) = make_float4(acc[0][v], acc[1][v], acc[2][v], acc[3][v]);
                *reinterpret_cast<float4*>(o + 4) = make_float4(acc[4][v], acc[5][v], acc[6][v], acc[7][v]);
            }
        }

        // ---- next piece ------------------------------------------------------------------------
#ifdef OPTGQA_FLAT_TIMING
        if (!has_next && p.timing && lane == 0) {
            p.timing[4 * u + 0] = tm0;
            p.timing[4 * u + 1] = tm1;
            p.timing[4 * u + 2] = tm2;
            p.timing[4 * u + 3] = wall_clock64();
        }
#endif
        if (!has_next) break;
        f += ntw;
        if (y + 1 == Y) P_b += n;                            // sequences skipped on the way have no tiles
        b = nb, y = ny, L = nL, n = nn, tau = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) qa[i] = qn[i];
#pragma unroll
        for (int v = 0; v < 4; ++v) slope2[v] = slope2n[v];
        chained = true;
    }
}

// Combine the partial results of the equal-work split: head h of sequence b collects slots
// u + s for the units u that touched its segment (a contiguous range found from P_b, n_b and c).
// Same arithmetic as the fixed-partition combine:
//   M = max_u m_u,  out = sum_u 2^(m_u-M) o_u / sum_u 2^(m_u-M) l_u.
template <int DT>
__global__ __launch_bounds__(kReduceThreads) void paged_decode_flat_reduce_kernel(const DecodeParams p)
{
    constexpr int D = 128;
    constexpr int kVecPerHead = D / 4;
    constexpr int kHeads = kReduceThreads / kVecPerHead;
    const int h = blockIdx.x * kHeads + threadIdx.x / kVecPerHead;
    const int od = (threadIdx.x % kVecPerHead) * 4;
    const int b = blockIdx.y;
    if (h >= p.num_heads) return;
    uint16_t* o = static_cast<uint16_t*>(p.out) + ((int64_t)b * p.num_heads + h) * D + od;
    const int L = p.context_lens[b];
    if (L <= 0) {
        *reinterpret_cast<uint2*>(o) = make_uint2(0u, 0u);
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
    const int n = flat_tiles(L);
    // (the clamps only matter if the lengths changed under the kernels: they keep every read
    // inside the workspace)
    const int c = max(p.plan[p.num_seqs], 1);
    const int F0 = Y * p.plan[b] + y * n;
    const int u0 = min(max(F0 / c, 0), p.num_units - 1);
    const int np = min(max((F0 + n - 1) / c - u0 + 1, 1), p.num_units - u0);
    const int64_t base = ((int64_t)u0 + (int64_t)b * Y + y) * GH + hh;       // slot stride between units: GH
    float M = -INFINITY;
    for (int i = 0; i < np; ++i) M = fmaxf(M, p.ws_m[base + (int64_t)i * GH]);
    float den = 0.f;
    float4 num = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int i0 = 0; i0 < np; i0 += 8) {
        float mm[8], ll[8];
        float4 x[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int64_t e = base + (int64_t)min(i0 + k, np - 1) * GH;
            mm[k] = p.ws_m[e];
            ll[k] = p.ws_l[e];
            x[k] = *reinterpret_cast<const float4*>(p.ws_o + e * D + od);
        }
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
    const float inv = p.out_scale / den;                 // out_scale: 1, or v_scale of an E4M3 cache
    uint2 packed;
    packed.x = narrow2<DT>(num.x * inv, num.y * inv);
    packed.y = narrow2<DT>(num.z * inv, num.w * inv);
    *reinterpret_cast<uint2*>(o) = packed;
}

}  // namespace optgqa
