// Paged decode attention: one query token per sequence against the block-indirected KV cache.
//
// Work unit: one workgroup (4 waves) per (KV head [x head chunk], sequence), the whole context.
// The GH query heads of the group that the workgroup serves all consume the SAME K and V
// registers, so every KV element is fetched from HBM once per KV-head group (Section II: a group
// shares one key-value pair), with 16-byte loads that cover a token row with D/8 consecutive lanes.
//
// Lane layout inside a wave: LPR = D/8 lanes share one token row (lane c holds dims 8c..8c+7),
// TPS = 64/LPR token rows are processed per step.  Each row group keeps its own running
// softmax state (m, l, acc); the states are merged once at the end (exactly, by the
// max / rescale / add identity of Section III-A's carried partial results).
#pragma once
#include "common.hpp"

namespace optgqa {

struct DecodeParams {
    void* out;                  // [B][Hq][D] dtype
    float* ws_m;                // split context (equal-work kernel): per partial-result slot and head,
    float* ws_l;                //   the softmax reference (base-2 domain), the sum of weights and the
    float* ws_o;                //   un-normalised weighted sum [D]
    const void* q;              // [B][Hq][D]
    const void* k_cache;        // [NB][Hkv][bs][D]
    const void* v_cache;
    const int32_t* block_tables;
    const int32_t* context_lens;
    const float* slopes;        // [Hq] or nullptr
    float scale2;               // scale * log2(e)
    int num_heads, num_kv_heads, block_size, max_blocks_per_seq;
    int num_partitions;         // fixed partitions on the equal-work kernel: partitions per segment, else 1
    int num_seqs;
    int row_offset;             // first row handled by this launch (grid.z/y counts from here)
    int heads_per_wg;           // query heads one workgroup serves (divides the group size)
    // Equal-work kernel: one unit per wave, see decode_flat_kernels.hpp; ws_m / ws_l are
    // [slot][columns] and ws_o is [slot][columns][D].
    int num_units;              // waves of the launch
    int segs_per_seq;           // KV heads x head chunks
    int32_t* plan;              // [num_seqs + 1]: tile prefix P_b per non-empty sequence, then tiles per unit
    float out_scale;            // multiplies the combined output (v_scale of an E4M3 cache, else 1)
    // E4M3 decode step: the new token is not among the streamed tiles; the combine kernel adds its term
    // (quantised with these reciprocal scales, as the cache write does) and stores its codes
    int new_token_in_combine;
    float k_inv_scale, v_inv_scale;
    // E4M3 caches with one scale pair per KV head: device arrays of num_kv_heads values (then scale2
    // holds no k_scale, out_scale is 1 and the two reciprocals above are unused), else nullptr
    const float* k_scales;
    const float* v_scales;
    int window;                 // > 0: a query sees only the last `window` tokens up to its own (equal-work kernel only)
    // Fused decode step (cache write inside the attention kernel): the new token of sequence b
    // sits at position context_lens[b] - 1; its rows come from k_new / v_new instead of the cache.
    const void* k_new;          // [num_seqs][Hkv][D], token stride k_new_stride elements
    const void* v_new;
    int64_t k_new_stride, v_new_stride;
    void* k_cache_w;            // the caches again, writable
    void* v_cache_w;
    // Shared prefixes (equal-work kernel only): sequences come in aligned bundles of `bundle`
    // consecutive ones; shared_blocks[b] > 0 says that the first shared_blocks[b] block-table
    // entries of sequence b are the bundle leader's (sequence b - b % bundle), 0 that b shares nothing.
    const int32_t* shared_blocks;   // [num_seqs] or nullptr
    int bundle;                     // sequences whose heads fit the score tile together: 16 / heads_per_wg
    // Fixed partitions through the equal-work kernel: pieces also end at every multiple of part_tiles
    // tiles of 16 tokens (partition_size / 16) inside a segment, and num_partitions bounds the
    // partitions of a segment; 0 = pieces end only where a unit or a segment ends.
    int part_tiles;
};

// Sequence and number of visible keys of one output row (decode: row = sequence).
__device__ __forceinline__ bool row_to_seq(const DecodeParams& p, int row, int& b, int& L)
{
    b = row;
    L = p.context_lens[b];
    return true;
}

constexpr int kDecodeWaves = 4;

template <int DT, int D, int GH>
__global__ __launch_bounds__(kDecodeWaves * 64) void paged_decode_kernel(const DecodeParams p)
{
    constexpr int LPR = D / 8;            // lanes per token row
    constexpr int TPS = 64 / LPR;         // token rows per wave step
    constexpr int NW = kDecodeWaves;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r = lane / LPR, c = lane % LPR;

    const int row = p.row_offset + blockIdx.z;
    const int Hq = p.num_heads, Hkv = p.num_kv_heads, bs = p.block_size;
    const int G = Hq / Hkv;
    const int chunks = G / GH;
    const int g = blockIdx.y / chunks;
    const int h0 = g * G + (blockIdx.y - g * chunks) * GH;

    int b, L;
    if (!row_to_seq(p, row, b, L)) return;
    const int t_begin = 0, t_end = L;                   // the whole context in one workgroup
    const uint16_t* __restrict__ qp = static_cast<const uint16_t*>(p.q);
    const uint16_t* __restrict__ kc = static_cast<const uint16_t*>(p.k_cache);
    const uint16_t* __restrict__ vc = static_cast<const uint16_t*>(p.v_cache);

    if (t_begin >= t_end) {
        // an empty context still owes an output row (all +0)
        uint16_t* o = static_cast<uint16_t*>(p.out) + ((int64_t)row * Hq + h0) * D;
        for (int i = threadIdx.x; i < GH * D; i += NW * 64) o[i] = 0;
        return;
    }

    // q for the GH heads, this lane's 8 dims, still packed (consumed by 2-way dot products).
    uint4 qv[GH];
    float slope2[GH];
#pragma unroll
    for (int i = 0; i < GH; ++i) {
        qv[i] = *reinterpret_cast<const uint4*>(qp + ((int64_t)row * Hq + h0 + i) * D + 8 * c);
        slope2[i] = p.slopes ? p.slopes[h0 + i] * kLog2e : 0.f;
    }

    float m[GH], l[GH], acc[GH][8];
#pragma unroll
    for (int i = 0; i < GH; ++i) {
        m[i] = -INFINITY;
        l[i] = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[i][e] = 0.f;
    }

    const int32_t* __restrict__ table = p.block_tables + (int64_t)b * p.max_blocks_per_seq;
    const int nsteps = (t_end - t_begin + TPS - 1) / TPS;
    for (int s = wave; s < nsteps; s += NW) {
        const int t0 = t_begin + s * TPS;                 // wave-uniform, never straddles a block
        const int64_t blk = table[t0 / bs];
        const int t = t0 + r;
        const bool valid = t < t_end;
        const int64_t off = ((blk * Hkv + g) * bs + (t0 % bs) + r) * D + 8 * c;
        uint4 kr = make_uint4(0, 0, 0, 0), vr = make_uint4(0, 0, 0, 0);
        if (valid) {
            kr = stream_load16(kc + off);
            vr = stream_load16(vc + off);
        }
        const float vf[8] = {widen_lo<DT>(vr.x), widen_hi<DT>(vr.x), widen_lo<DT>(vr.y), widen_hi<DT>(vr.y),
                             widen_lo<DT>(vr.z), widen_hi<DT>(vr.z), widen_lo<DT>(vr.w), widen_hi<DT>(vr.w)};
        const float rel = (float)(t - (L - 1));           // exact: |rel| < 2^24
#pragma unroll
        for (int i = 0; i < GH; ++i) {
            float d = dot2<DT>(qv[i].x, kr.x, 0.f);
            d = dot2<DT>(qv[i].y, kr.y, d);
            d = dot2<DT>(qv[i].z, kr.z, d);
            d = dot2<DT>(qv[i].w, kr.w, d);
            d = row_group_sum<LPR>(d);
            const float s2 = valid ? fmaf(d, p.scale2, slope2[i] * rel) : -INFINITY;   // eq. (3), base 2
            const float m_new = fmaxf(m[i], s2);
            const bool none = m_new == -INFINITY;
            const float alpha = none ? 1.f : fast_exp2(m[i] - m_new);
            const float pj = none ? 0.f : fast_exp2(s2 - m_new);                        // eq. (4)
            m[i] = m_new;
            l[i] = fmaf(l[i], alpha, pj);
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[i][e] = fmaf(acc[i][e], alpha, pj * vf[e]);
        }
    }

    // ---- merge the TPS row groups of this wave (lanes with equal c, different r) ----------
#pragma unroll
    for (int i = 0; i < GH; ++i) {
        float mw = m[i];
#pragma unroll
        for (int off = LPR; off < 64; off <<= 1) mw = fmaxf(mw, __shfl_xor(mw, off));
        const float f = (mw == -INFINITY) ? 0.f : fast_exp2(m[i] - mw);
        float lw = l[i] * f;
#pragma unroll
        for (int off = LPR; off < 64; off <<= 1) lw += __shfl_xor(lw, off);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float a = acc[i][e] * f;
#pragma unroll
            for (int off = LPR; off < 64; off <<= 1) a += __shfl_xor(a, off);
            acc[i][e] = a;
        }
        m[i] = mw;
        l[i] = lw;
    }

    // ---- merge the waves through LDS and write the result ---------------------------------
    __shared__ float sm_m[NW][GH];
    __shared__ float sm_l[NW][GH];
    __shared__ float sm_o[NW][GH][D];
    if (r == 0) {
#pragma unroll
        for (int i = 0; i < GH; ++i) {
            if (c == 0) {
                sm_m[wave][i] = m[i];
                sm_l[wave][i] = l[i];
            }
            *reinterpret_cast<float4*>(&sm_o[wave][i][8 * c]) = make_float4(acc[i][0], acc[i][1], acc[i][2], acc[i][3]);
            *reinterpret_cast<float4*>(&sm_o[wave][i][8 * c + 4]) = make_float4(acc[i][4], acc[i][5], acc[i][6], acc[i][7]);
        }
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < GH * D; idx += NW * 64) {
        const int i = idx / D, d = idx - i * D;
        float M = sm_m[0][i];
#pragma unroll
        for (int w = 1; w < NW; ++w) M = fmaxf(M, sm_m[w][i]);
        float num = 0.f, den = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const float f = fast_exp2(sm_m[w][i] - M);    // a wave without tokens has m = -inf -> 0
            num = fmaf(f, sm_o[w][i][d], num);
            den = fmaf(f, sm_l[w][i], den);
        }
        const int h = h0 + i;
        static_cast<uint16_t*>(p.out)[((int64_t)row * Hq + h) * D + d] = narrow<DT>(num / den);
    }
}

constexpr int kReduceThreads = 256;      // threads of a combine workgroup (decode_flat_kernels.hpp)

}  // namespace optgqa
