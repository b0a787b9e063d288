// Paged decode attention for head_dim 128, unsplit: one workgroup walks the whole context of one
// (sequence, KV head [x head chunk]), any group size up to 16 heads per workgroup.  It runs when
// the context is too short to be worth splitting or the caller forbids the split; every split
// runs on the equal-work kernel (decode_flat_kernels.hpp), which took this kernel's tile loop.
//
// Decode reads every K/V byte once and does G multiply-adds per byte; on MI355X that is still
// HBM-bound only if the arithmetic stays off the critical path, and the vector ALU alone
// cannot keep up at G = 8 (measured: a dot-product/FMA formulation of this kernel saturates
// instruction issue at about half the achievable HBM rate).  So both contractions run on the
// matrix cores, with the operands arranged so that the loads stay plain 16-byte pieces:
//
//   scores  S[head][token] = Q K^T : v_mfma_f32_16x16x32 (bf16 / fp16 inputs, fp32 accumulate).
//           A = the group's query rows (rows >= GH are zero padding), B = a 16-token K tile.
//           Lane (token n, k-slab kc) of the B operand needs dims 32i + 8kc .. +7 of token n:
//           exactly one 16-byte piece of the cache row, so the tile is fetched straight into
//           operand order (four loads per 16 tokens, each covering 64 contiguous bytes per row).
//   output  O[head][dim] += P V    : v_mfma_f32_16x16x4 (all fp32: the softmax weights are
//           never rounded to 16 bits).  B = V widened to fp32 in the natural layout (lane
//           16r + c holds dims 8c..8c+7 of token row r of the step), A = the weights
//           transposed through 1 KiB of LDS.
//
// The ALU is left with the softmax (4 scores per lane per 16 tokens), the widening of V and
// addresses, which leaves registers to spare: K/V tiles are fetched straight into VGPRs,
// kMmaBufs - 1 tiles (8 KiB each per wave) ahead of the arithmetic, in a rotating set of
// register buffers (the loop is unrolled by kMmaBufs so that the rotation costs no moves).
// One K/V fetch serves all heads of the group (Section II: a group shares one key-value pair).
//
// Softmax uses a lazily moved reference instead of the exact running maximum: with ALiBi the
// scores climb steadily along the context and an exact running maximum would rescale the
// accumulators at every tile.  The reference only moves when a score exceeds it by
// 2^kRescaleThreshold and is then placed 2^kRescaleHeadroom above the tile maximum; weights
// stay inside [2^-90, 2^30] relative to any maximum that matters, and softmax does not depend
// on the reference.
#pragma once
#include "decode_mc_kernels.hpp"

namespace optgqa {

#ifndef OPTGQA_MMA_BUFS
#define OPTGQA_MMA_BUFS 2
#endif
#ifndef OPTGQA_MMA_WAVES_PER_SIMD
#define OPTGQA_MMA_WAVES_PER_SIMD 2
#endif
constexpr int kMmaBufs = OPTGQA_MMA_BUFS;              // register tile buffers per wave (in flight + in use)
constexpr int kMmaTile = 16;                           // tokens per wave tile
constexpr int kMmaMaxHeads = 16;                       // MFMA M dimension

struct MmaTile {
    uint4 k[4];     // K: token j16, dims 32i + 8hg .. +7   (B operand of score MFMA i)
    uint4 v[4];     // V: token 4s + hg, dims 8*j16 .. +7    (B operand of the output MFMAs of step s)
};

template <int DT> __device__ __forceinline__ f32x4 mfma_qk(uint4 a, uint4 b, f32x4 c);
template <> __device__ __forceinline__ f32x4 mfma_qk<kF16>(uint4 a, uint4 b, f32x4 c)
{
    typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}
template <> __device__ __forceinline__ f32x4 mfma_qk<kBF16>(uint4 a, uint4 b, f32x4 c)
{
    typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

template <int CTRL> __device__ __forceinline__ float dpp_max(float x) { return fmaxf(x, dpp<CTRL>(x)); }
__device__ __forceinline__ float row16_max(float x)
{
    x = dpp_max<kDppXor1>(x);
    x = dpp_max<kDppXor2>(x);
    x = dpp_max<kDppHalfMirror>(x);
    return dpp_max<kDppMirror>(x);
}

template <int DT>
__global__ __launch_bounds__(kDecodeWaves * 64, OPTGQA_MMA_WAVES_PER_SIMD) void paged_decode_mma_kernel(const DecodeParams p)
{
    constexpr int D = 128;
    constexpr int NW = kDecodeWaves;
    constexpr int TILE = kMmaTile;
    constexpr int NB = kMmaBufs;
    constexpr int PT = NB - 1;                      // tiles of lookahead

    __shared__ __attribute__((aligned(16))) float merge[NW][kMmaMaxHeads][D];      // epilogue only
    __shared__ __attribute__((aligned(16))) float p_lds[NW][TILE][kMmaMaxHeads];   // tile weights [token][head]
    __shared__ float sm_m[NW][kMmaMaxHeads];
    __shared__ float sm_l[NW][kMmaMaxHeads];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int j16 = lane & 15;                      // token of the tile (scores) / dim chunk (V, output)
    const int hg = lane >> 4;                       // head quad (scores, output) / k-slab (K) / token row (V)

    const int row = p.row_offset + blockIdx.z;
    const int Hq = p.num_heads, Hkv = p.num_kv_heads, bs = p.block_size;
    const int bs_shift = __builtin_ctz(bs);
    const int GH = p.heads_per_wg;
    const int G = Hq / Hkv;
    const int chunks = G / GH;
    const int g = blockIdx.y / chunks;
    const int h0 = g * G + (blockIdx.y - g * chunks) * GH;

    int b, L;
    if (!row_to_seq(p, row, b, L)) return;
    const int t_begin = 0, t_end = L;                   // the whole context in one workgroup
    if (t_begin >= t_end) {                             // an empty context still owes an output row (all +0)
        uint16_t* o = static_cast<uint16_t*>(p.out) + ((int64_t)row * Hq + h0) * D;
        for (int i = threadIdx.x; i < GH * D; i += NW * 64) o[i] = 0;
        return;
    }
    const uint16_t* __restrict__ qp = static_cast<const uint16_t*>(p.q);
    const uint16_t* __restrict__ kc = static_cast<const uint16_t*>(p.k_cache);
    const uint16_t* __restrict__ vc = static_cast<const uint16_t*>(p.v_cache);
    const int32_t* __restrict__ table = p.block_tables + (int64_t)b * p.max_blocks_per_seq;

    const float scale2 = p.scale2;
    const int Lm1 = L - 1;
    const uint16_t* __restrict__ kc_g = kc + (int64_t)g * bs * D;
    const uint16_t* __restrict__ vc_g = vc + (int64_t)g * bs * D;
    const int64_t block_stride = (int64_t)Hkv * bs * D;
    const int t_last = t_end - 1;

    // Each wave owns a contiguous quarter of the context's tiles.
    const int ntiles = (t_end - t_begin + TILE - 1) / TILE;
    const int tpw = (ntiles + NW - 1) / NW;
    const int tile_first = wave * tpw;
    const int ntw = max(0, min(tpw, ntiles - tile_first));

    // All 16 tokens of a tile lie in one physical block (tiles are 16-aligned, blocks >= 16 tokens).
    // Loads are unconditional and in bounds: rows past the end of the range re-read the last valid
    // row and are masked out of the scores.
    auto load_tile = [&](MmaTile& T, int j) {
        const int tile_t0 = t_begin + (tile_first + j) * TILE;                       // < t_end
        const int blk = __builtin_amdgcn_readfirstlane(table[tile_t0 >> bs_shift]);
        const int64_t uni = blk * block_stride + (int64_t)(tile_t0 & (bs - 1)) * D;
        const int tk = min(tile_t0 + j16, t_last) - tile_t0;
        const uint16_t* ka = kc_g + uni + tk * D + 8 * hg;
#pragma unroll
        for (int i = 0; i < 4; ++i) T.k[i] = stream_load16(ka + 32 * i);
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int tv = min(tile_t0 + 4 * s + hg, t_last) - tile_t0;
            T.v[s] = stream_load16(vc_g + uni + tv * D + 8 * j16);
        }
    };

    // Start the first tiles' loads before anything else touches memory, so that the query rows
    // and slopes arrive in their shadow.
    MmaTile buf[NB];
    const int j_last = max(ntw - 1, 0);
    if (ntw > 0) {
#pragma unroll
        for (int i = 0; i < PT; ++i) load_tile(buf[i], min(i, j_last));
    }

    // A operand of the score MFMAs: lane (head j16, k-slab hg) holds dims 32i + 8hg .. +7 of its head.
    // (Loaded unconditionally from a clamped head and zeroed afterwards: no branches around loads.)
    uint4 qa[4];
    {
        const uint16_t* qrow = qp + ((int64_t)row * Hq + h0 + min(j16, GH - 1)) * D + 8 * hg;
        const uint32_t keep = j16 < GH ? 0xffffffffu : 0u;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint4 x = *reinterpret_cast<const uint4*>(qrow + 32 * i);
            qa[i] = make_uint4(x.x & keep, x.y & keep, x.z & keep, x.w & keep);
        }
    }
    // Softmax state and output accumulators of heads 4hg + v (v = 0..3); scores of those heads for
    // token j16 arrive in this lane, and the output MFMA leaves the same heads here for dims 8*j16 + e.
    float slope2[4], m_ref[4], l[4];
    f32x4 acc[8];
    {
        float sl[4] = {0.f, 0.f, 0.f, 0.f};
        if (p.slopes) {                                          // uniform; one batch of loads
#pragma unroll
            for (int v = 0; v < 4; ++v) sl[v] = p.slopes[h0 + min(4 * hg + v, GH - 1)];
        }
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            slope2[v] = 4 * hg + v < GH ? sl[v] * kLog2e : 0.f;
            m_ref[v] = kNoMax;
            l[v] = 0.f;
        }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = f32x4{0.f, 0.f, 0.f, 0.f};
    // the A operand of the output MFMA reads all 16 head columns: start them finite
    reinterpret_cast<float4*>(&p_lds[wave][0][0])[lane] = make_float4(0.f, 0.f, 0.f, 0.f);

    float* const pw_write = &p_lds[wave][j16][4 * hg];      // this lane's 4 weights of token j16
    const float* const pw_read = &p_lds[wave][hg][j16];     // + 4s*16: weight of head j16 for token 4s + hg

    auto compute_tile = [&](const MmaTile& T, int j) {
        // scores of heads 4hg..4hg+3 for token j16 of the tile: eq. (3) in base 2
        f32x4 S = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < 4; ++i) S = mfma_qk<DT>(qa[i], T.k[i], S);
        const int t = t_begin + (tile_first + j) * TILE + j16;
        const bool valid = t < t_end;
        const float rel = (float)(t - Lm1);                  // exact: |rel| < 2^24
        float s2[4];
        bool need = false;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            s2[v] = valid ? fmaf(S[v], scale2, slope2[v] * rel) : -INFINITY;
            need |= s2[v] > m_ref[v] + kRescaleThreshold;
        }
        if (__builtin_amdgcn_ballot_w64(need) != 0) {
            // move the references of all heads; a row of 16 lanes holds the 16 tokens of one head quad
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float m_new = fmaxf(m_ref[v], row16_max(s2[v]) + kRescaleHeadroom);
                const float alpha = fast_exp2(m_ref[v] - m_new);      // 1 when unchanged, 0 on first use
                m_ref[v] = m_new;
                l[v] *= alpha;
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[e][v] *= alpha;
            }
        }
        float4 pw;
        pw.x = fast_exp2(s2[0] - m_ref[0]);                  // eq. (4) numerators; 0 for absent keys
        pw.y = fast_exp2(s2[1] - m_ref[1]);
        pw.z = fast_exp2(s2[2] - m_ref[2]);
        pw.w = fast_exp2(s2[3] - m_ref[3]);
        l[0] += pw.x;
        l[1] += pw.y;
        l[2] += pw.z;
        l[3] += pw.w;
        *reinterpret_cast<float4*>(pw_write) = pw;            // [token][head] ...
        float a[4];
#pragma unroll
        for (int s = 0; s < 4; ++s) a[s] = pw_read[4 * s * kMmaMaxHeads];   // ... read back as [head][token]
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const uint4 vr = T.v[s];
            const float vf[8] = {widen_lo<DT>(vr.x), widen_hi<DT>(vr.x), widen_lo<DT>(vr.y), widen_hi<DT>(vr.y),
                                 widen_lo<DT>(vr.z), widen_hi<DT>(vr.z), widen_lo<DT>(vr.w), widen_hi<DT>(vr.w)};
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[s], vf[e], acc[e], 0, 0, 0);
        }
    };

    // ---- main loop: NB rotating register buffers, unrolled by NB ----------------------------
    // Every iteration issues exactly one tile of loads, so the number of loads in flight at each
    // use is a compile-time constant.  Past the end of the wave's range the prefetch re-reads the
    // wave's last tile (a cache hit, never consumed) instead of branching around the loads.
    if (ntw > 0) {
        const int trips = (ntw + NB - 1) / NB;
        for (int it = 0; it < trips; ++it) {
            const int j0 = it * NB;
#pragma unroll
            for (int i = 0; i < NB; ++i) {
                const int j = j0 + i;
                load_tile(buf[(i + PT) % NB], min(j + PT, j_last));
                if (j <= j_last) compute_tile(buf[i], j);
            }
        }
    }

    // ---- merge the four waves ---------------------------------------------------------------
#pragma unroll
    for (int v = 0; v < 4; ++v) l[v] = row_group_sum<16>(l[v]);      // over the 16 token lanes
    if (j16 == 0) {
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            sm_m[wave][4 * hg + v] = m_ref[v];
            sm_l[wave][4 * hg + v] = l[v];
        }
    }
    __syncthreads();
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        const int h = 4 * hg + v;
        float M = sm_m[0][h];
#pragma unroll
        for (int w = 1; w < NW; ++w) M = fmaxf(M, sm_m[w][h]);
        const float f = fast_exp2(m_ref[v] - M);             // a wave without keys: 2^(-1e30 - M) = 0
        *reinterpret_cast<float4*>(&merge[wave][h][8 * j16]) =
            make_float4(acc[0][v] * f, acc[1][v] * f, acc[2][v] * f, acc[3][v] * f);
        *reinterpret_cast<float4*>(&merge[wave][h][8 * j16 + 4]) =
            make_float4(acc[4][v] * f, acc[5][v] * f, acc[6][v] * f, acc[7][v] * f);
    }
    __syncthreads();
    for (int vec = threadIdx.x; vec < GH * (D / 4); vec += NW * 64) {
        const int oh = vec / (D / 4), od = (vec - oh * (D / 4)) * 4;
        float M = sm_m[0][oh];
#pragma unroll
        for (int w = 1; w < NW; ++w) M = fmaxf(M, sm_m[w][oh]);
        float den = 0.f;
        float4 num = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            den = fmaf(fast_exp2(sm_m[w][oh] - M), sm_l[w][oh], den);
            const float4 x = *reinterpret_cast<const float4*>(&merge[w][oh][od]);
            num.x += x.x;
            num.y += x.y;
            num.z += x.z;
            num.w += x.w;
        }
        const int h = h0 + oh;
        const float inv = 1.f / den;
        uint2 packed;
        packed.x = narrow2<DT>(num.x * inv, num.y * inv);
        packed.y = narrow2<DT>(num.z * inv, num.w * inv);
        *reinterpret_cast<uint2*>(static_cast<uint16_t*>(p.out) + ((int64_t)row * Hq + h) * D + od) = packed;
    }
}

}  // namespace optgqa
