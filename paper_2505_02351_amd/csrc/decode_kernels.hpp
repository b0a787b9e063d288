// Paged decode attention: one query token per sequence against the block-indirected KV cache.
//
// Work unit: one workgroup (4 waves) per (context partition, KV head [x head chunk], sequence).
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
    float* ws_m;                // split path: [B][Hq][NP]   running max (base-2 domain)
    float* ws_l;                //             [B][Hq][NP]   sum of weights
    float* ws_o;                //             [B][Hq][NP][D] un-normalised weighted sum
    const void* q;              // [B][Hq][D]
    const void* k_cache;        // [NB][Hkv][bs][D]
    const void* v_cache;
    const int32_t* block_tables;
    const int32_t* context_lens;
    const float* slopes;        // [Hq] or nullptr
    float scale2;               // scale * log2(e)
    int num_heads, num_kv_heads, block_size, max_blocks_per_seq;
    int partition_size;         // tokens per workgroup; >= max context when unsplit
    int num_partitions;         // 1 = unsplit: the kernel writes `out` itself
    int num_seqs;
    int row_offset;             // first row handled by this launch (grid.z/y counts from here)
    int heads_per_wg;           // query heads one workgroup serves (divides the group size)
    // Equal-work split (head_dim 128): one unit per wave, see decode_flat_kernels.hpp.
    // There ws_m / ws_l are [slot][heads_per_wg] and ws_o is [slot][heads_per_wg][D].
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

// Partition index of this workgroup.  Workgroups go to the 8 XCDs round-robin by flat id; with
// grid.x = number of partitions and late partitions mostly empty (short sequences), the plain
// mapping would give some XCDs all the work whenever grid.x shares a factor with 8.  Rotating
// the partition index by the other two grid coordinates hands every XCD the same mix.
__device__ __forceinline__ int skewed_partition(int num_partitions)
{
    return (blockIdx.x + blockIdx.y + blockIdx.z) % num_partitions;
}

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
    const int part = skewed_partition(p.num_partitions);
    const int Hq = p.num_heads, Hkv = p.num_kv_heads, bs = p.block_size;
    const int G = Hq / Hkv;
    const int chunks = G / GH;
    const int g = blockIdx.y / chunks;
    const int h0 = g * G + (blockIdx.y - g * chunks) * GH;

    int b, L;
    if (!row_to_seq(p, row, b, L)) return;
    // Sliding window (Alg. 1, local mask; unsplit launches only): the query at position L - 1 sees
    // tokens lo .. L - 1; the steps start at the row group that holds token lo.
    const int lo = (p.window > 0 && p.num_partitions == 1) ? max(L - p.window, 0) : 0;
    const int t_begin = max(part * p.partition_size, lo / TPS * TPS);
    const int t_end = min(L, part * p.partition_size + p.partition_size);
    const uint16_t* __restrict__ qp = static_cast<const uint16_t*>(p.q);
    const uint16_t* __restrict__ kc = static_cast<const uint16_t*>(p.k_cache);
    const uint16_t* __restrict__ vc = static_cast<const uint16_t*>(p.v_cache);

    if (t_begin >= t_end) {
        // An empty context still owes an output row (all +0); empty partitions owe nothing.
        if (p.num_partitions == 1) {
            uint16_t* o = static_cast<uint16_t*>(p.out) + ((int64_t)row * Hq + h0) * D;
            for (int i = threadIdx.x; i < GH * D; i += NW * 64) o[i] = 0;
        }
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
        const bool valid = t < t_end && t >= lo;
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
        if (p.num_partitions == 1) {
            static_cast<uint16_t*>(p.out)[((int64_t)row * Hq + h) * D + d] = narrow<DT>(num / den);
        } else {
            const int64_t slot = ((int64_t)row * Hq + h) * p.num_partitions + part;
            if (d == 0) {
                p.ws_m[slot] = M;
                p.ws_l[slot] = den;
            }
            p.ws_o[slot * D + d] = num;
        }
    }
}

// Combine the per-partition (max, sum, weighted sum) triples of the split path:
//   M = max_p m_p,  out = sum_p 2^(m_p-M) o_p / sum_p 2^(m_p-M) l_p
// (Section III-A: the per-partition results are carried forward and merged).
// One thread per 4 output dims; kReduceHeads heads per workgroup; grid = (ceil(Hq / kReduceHeads), rows).
// Partitions are taken in batches of 8 whose loads are all issued before the first use: the
// kernel is a few microseconds of pure memory latency, so the loads must overlap.
constexpr int kReduceThreads = 256;

template <int DT, int D>
__global__ __launch_bounds__(kReduceThreads) void paged_decode_reduce_kernel(const DecodeParams p)
{
    constexpr int kVecPerHead = D / 4;
    constexpr int kHeads = kReduceThreads / kVecPerHead;
    const int h = blockIdx.x * kHeads + threadIdx.x / kVecPerHead;
    const int od = (threadIdx.x % kVecPerHead) * 4;
    const int row = p.row_offset + blockIdx.y;
    if (h >= p.num_heads) return;
    int b, L;
    if (!row_to_seq(p, row, b, L)) return;
    uint16_t* o = static_cast<uint16_t*>(p.out) + ((int64_t)row * p.num_heads + h) * D + od;
    if (L <= 0) {
        *reinterpret_cast<uint2*>(o) = make_uint2(0u, 0u);
        return;
    }
    const int np = (L + p.partition_size - 1) / p.partition_size;
    const int64_t base = ((int64_t)row * p.num_heads + h) * p.num_partitions;
    // One pass in batches of 8 partitions with a running reference (a separate pass for the maximum
    // would be a second chain of memory round trips).
    float M = -INFINITY;
    float den = 0.f;
    float4 num = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int i0 = 0; i0 < np; i0 += 8) {
        float mm[8], ll[8];
        float4 x[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int i = min(i0 + k, np - 1);
            mm[k] = p.ws_m[base + i];
            ll[k] = p.ws_l[base + i];
            x[k] = *reinterpret_cast<const float4*>(p.ws_o + (base + i) * D + od);
        }
        float Mn = M;                                            // clamped repeats of the last partition do not change it
#pragma unroll
        for (int k = 0; k < 8; ++k) Mn = fmaxf(Mn, mm[k]);
        const float keep = i0 == 0 ? 0.f : fast_exp2(M - Mn);    // nothing accumulated before the first batch
        M = Mn;
        den *= keep;
        num.x *= keep;
        num.y *= keep;
        num.z *= keep;
        num.w *= keep;
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const float f = i0 + k < np ? fast_exp2(mm[k] - M) : 0.f;
            den = fmaf(f, ll[k], den);
            num.x = fmaf(f, x[k].x, num.x);
            num.y = fmaf(f, x[k].y, num.y);
            num.z = fmaf(f, x[k].z, num.z);
            num.w = fmaf(f, x[k].w, num.w);
        }
    }
    const float inv = 1.f / den;
    uint2 packed;
    packed.x = narrow2<DT>(num.x * inv, num.y * inv);
    packed.y = narrow2<DT>(num.z * inv, num.w * inv);
    *reinterpret_cast<uint2*>(o) = packed;
}

}  // namespace optgqa
