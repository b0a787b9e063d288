// Paged decode attention, group sizes that are multiples of 4: the fast path.
//
// Same work decomposition and the same K/V register layout as paged_decode_kernel (16-byte
// loads, D/8 consecutive lanes per token row, one K/V fetch per KV-head group), but with the
// arithmetic re-balanced for CDNA4:
//   * q.k: 2-way dot instructions on the packed 2-byte data, then a TRANSPOSING reduction
//     inside each quad of lanes, so that lane u of every quad ends up owning the finished
//     scores of heads u and u+4 (no score is computed redundantly, softmax work is 4x less);
//   * softmax: fp32, against a lazily updated reference instead of the exact running maximum.
//     ALiBi makes scores climb steadily along the context, so an exact running maximum would
//     rescale the accumulators every tile.  The reference is only moved when a tile maximum
//     exceeds it by 2^kRescaleThreshold, and is then placed 2^kRescaleHeadroom above that
//     maximum: weights live in [2^-90, 2^30] relative to any later maximum that matters, well
//     inside fp32 range, and softmax is invariant to the choice of reference;
//   * p.V: the matrix cores.  v_mfma_f32_4x4x1 performs 16 independent 4x4 outer products:
//     block = quad of lanes, A = the quad's four weights (one head per lane), B = each lane's
//     own widened V element.  All operands are fp32, so the weights are never rounded, and no
//     tile row is padding: the instruction does exactly GH x 8 multiply-adds per lane that the
//     vector ALU would otherwise issue one by one, and it runs beside the vector ALU.
// K/V tiles travel HBM -> LDS with direct-to-LDS loads (no VGPRs held while in flight) into a
// per-wave ring of kMcRingTiles tiles, kMcRingTiles-1 tiles ahead of the arithmetic; each lane
// later reads back exactly the 16 bytes it fetched.  The ring is private to a wave, so the
// only synchronisation is a vmcnt wait.
#pragma once
#include "decode_kernels.hpp"

namespace optgqa {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr float kRescaleThreshold = 30.f;    // log2 units: rescale when a tile maximum exceeds the reference by this
constexpr float kRescaleHeadroom = 60.f;     // ... and then put the reference this far ABOVE the maximum
constexpr float kNoMax = -1.0e30f;           // "no key seen yet"; finite so that differences stay finite
constexpr int kMcSteps = 2;                  // steps per wave tile
#ifndef OPTGQA_RING_TILES
#define OPTGQA_RING_TILES 3
#endif
constexpr int kMcRingTiles = OPTGQA_RING_TILES;  // ring slots per wave (tiles in flight + the one in use)

template <int V> __device__ __forceinline__ float quad_bcast(float x)
{
    return dpp<V * 0x55>(x);                 // quad_perm [V,V,V,V]
}

// Sum over the quads of a token row group for values that differ between the lanes of a quad.
template <int LPR> __device__ __forceinline__ float cross_quad_sum(float x);
template <> __device__ __forceinline__ float cross_quad_sum<16>(float x)
{
    x += dpp<kDppRowRor8>(x);                // lane i ^ 8
    x += dpp<kDppRowRor4>(x);                // now symmetric under ^8, so i-4 completes the four quads
    return x;
}
template <> __device__ __forceinline__ float cross_quad_sum<8>(float x)
{
    // partner quad is lane i ^ 4: take i+4 in even quads, i-4 in odd quads
    int v = __builtin_bit_cast(int, x);
    int t = __builtin_amdgcn_update_dpp(0, v, 0x104, 0xf, 0x5, false);     // row_shl:4, quads 0 and 2
    t = __builtin_amdgcn_update_dpp(t, v, 0x114, 0xf, 0xa, false);         // row_shr:4, quads 1 and 3
    return x + __builtin_bit_cast(float, t);
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Wait until at most NEWER direct-to-LDS loads issued after the wanted tile are still in
// flight, then read the tile's four 16-byte pieces (K step 0, K step 1, V step 0, V step 1)
// back from this lane's place in the ring.  The wait and the reads are one asm block because
// the compiler cannot be told which outstanding load a given LDS read depends on (it would
// wait for all of them, the newest prefetch included).
template <int NEWER>
__device__ __forceinline__ void ring_read2(uint32_t lds_addr, u32x4& k0, u32x4& k1, u32x4& v0, u32x4& v1)
{
    asm volatile(
        "s_waitcnt vmcnt(%5)\n\t"
        "ds_read_b128 %0, %4\n\t"
        "ds_read_b128 %1, %4 offset:1024\n\t"
        "ds_read_b128 %2, %4 offset:2048\n\t"
        "ds_read_b128 %3, %4 offset:3072\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&v"(k0), "=&v"(k1), "=&v"(v0), "=&v"(v1)
        : "v"(lds_addr), "n"(NEWER)
        : "memory");
}

// Read one block-table entry through the scalar (constant) cache.  Written as asm because the
// compiler stops selecting scalar loads once direct-to-LDS loads (which it must treat as
// stores it cannot see through) are in flight, and a vector load here would force a wait for
// every outstanding prefetch.  Read-only; the table is never written while the kernel runs.
__device__ __forceinline__ int scalar_load_i32(const int32_t* uniform_ptr)
{
    int v;
    asm volatile("s_load_dword %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)" : "=s"(v) : "s"(uniform_ptr) : "memory");
    return v;
}

// Dynamic LDS of the kernel: [ring of all waves | merge buffer] followed by the per-stream
// (max, sum) pairs.
template <int D, int GH>
struct McSmem {
    static constexpr int kStreams = kDecodeWaves * (64 / (D / 8));
    static constexpr int kRingBytes = kDecodeWaves * kMcRingTiles * kMcSteps * 2 * 1024;
    static constexpr int kMergeBytes = (kStreams / 2) * GH * D * 4;
    static constexpr int kBulkBytes = kRingBytes > kMergeBytes ? kRingBytes : kMergeBytes;
    static constexpr int kBytes = kBulkBytes + 2 * kStreams * GH * 4;
};

template <int DT, int D, int GH>
__global__ __launch_bounds__(kDecodeWaves * 64, 2) void paged_decode_mc_kernel(const DecodeParams p)
{
    static_assert(GH == 4 || GH == 8, "heads per workgroup must be 4 or 8");
    static_assert(kMcSteps == 2, "ring_read2 reads two steps per tile");
    static_assert(kMcSteps * (64 / (D / 8)) <= 16, "a wave tile must not straddle a 16-token block");
    constexpr int LPR = D / 8;               // lanes per token row
    constexpr int TPS = 64 / LPR;            // token rows per step
    constexpr int NW = kDecodeWaves;
    constexpr int U = kMcSteps;
    constexpr int TILE = U * TPS;            // tokens per wave tile
    constexpr int HPL = GH / 4;              // heads owned per lane after the reduction
    constexpr int NSTREAM = NW * TPS;        // independent softmax streams per workgroup
    constexpr int NT = kMcRingTiles;
    constexpr int PT = NT - 1;               // tiles of lookahead
    constexpr int kTileBytes = U * 2 * 1024; // K and V, 1 KiB per step each
    using Smem = McSmem<D, GH>;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];      // ring, later the merge buffer
    float (*sm_m)[GH] = reinterpret_cast<float (*)[GH]>(smem + Smem::kBulkBytes);
    float (*sm_l)[GH] = sm_m + NSTREAM;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r = lane / LPR, c = lane % LPR, u = lane & 3;

    const int row = p.row_offset + blockIdx.z;
    const int Hq = p.num_heads, Hkv = p.num_kv_heads, bs = p.block_size;
    const int bs_shift = __builtin_ctz(bs);
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

    // q, this lane's 8 dims, still packed, in a lane-dependent head order: slot 4i+k holds head
    // 4i + (u ^ k).  With that order the transposing reduction needs no selects: slot 0 is the
    // head this lane ends up owning, slots 1..3 are the partial sums it hands to lanes u^1, u^2.
    uint4 qv[GH];
#pragma unroll
    for (int i = 0; i < GH; ++i)
        qv[i] = *reinterpret_cast<const uint4*>(qp + ((int64_t)row * Hq + h0 + (i & ~3) + (u ^ (i & 3))) * D + 8 * c);
    float slope2[HPL], m_ref[HPL], l[HPL];
    f32x4 acc[8][HPL];
#pragma unroll
    for (int i = 0; i < HPL; ++i) {
        slope2[i] = p.slopes ? p.slopes[h0 + u + 4 * i] * kLog2e : 0.f;
        m_ref[i] = kNoMax;
        l[i] = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e][i] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    const float scale2 = p.scale2;
    const int Lm1 = L - 1;
    // Addresses: a wave-uniform 64-bit part (physical block, KV head, first row of the step)
    // plus a small per-lane part (row inside the step, dim chunk).  Every load is in bounds and
    // unconditional: steps or rows past the end of the range re-read the last valid row and are
    // masked out of the scores instead.
    const uint16_t* __restrict__ kc_g = kc + (int64_t)g * bs * D;
    const uint16_t* __restrict__ vc_g = vc + (int64_t)g * bs * D;
    const int64_t block_stride = (int64_t)Hkv * bs * D;
    const int t_last = t_end - 1;
    const int t_last0 = t_last & ~(TPS - 1);                         // first row of the last valid step

    // Each wave owns a contiguous quarter of the tiles (so that the ALiBi bias climbs slowly
    // along a wave's stream); its j-th tile lives in ring slot j % NT.
    const int ntiles = (t_end - t_begin + TILE - 1) / TILE;
    const int tpw = (ntiles + NW - 1) / NW;
    const int tile_first = wave * tpw;
    const int ntw = max(0, min(tpw, ntiles - tile_first));
    unsigned char* const ring = smem + wave * (NT * kTileBytes);

    auto issue_tile = [&](int j) {
        const int tile = tile_first + j;
        unsigned char* const slot = ring + (j % NT) * kTileBytes;
        const int tile_t0 = t_begin + tile * TILE;                                    // < t_end
        const int blk = scalar_load_i32(table + (tile_t0 >> bs_shift));               // one block per tile
#pragma unroll
        for (int s = 0; s < U; ++s) {
            const int t0 = min(tile_t0 + s * TPS, t_last0);                           // wave-uniform
            const int64_t uni = blk * block_stride + (int64_t)(t0 & (bs - 1)) * D;
            const int lane_off = (min(t0 + r, t_last) - t0) * D + 8 * c;
            // (last operand: cache policy; 2 = the non-temporal hint, see stream_load16)
            __builtin_amdgcn_global_load_lds(kc_g + uni + lane_off, slot + s * 1024, 16, 0, OPTGQA_STREAM_NT ? 2 : 0);
            __builtin_amdgcn_global_load_lds(vc_g + uni + lane_off, slot + (U + s) * 1024, 16, 0, OPTGQA_STREAM_NT ? 2 : 0);
        }
    };

    auto compute_tile = [&](const u32x4 (&kt)[U], const u32x4 (&vt)[U], int tile) {
        float sc[U][HPL], tmax[HPL];
#pragma unroll
        for (int i = 0; i < HPL; ++i) tmax[i] = -INFINITY;
#pragma unroll
        for (int s = 0; s < U; ++s) {
            const int t = t_begin + tile * TILE + s * TPS + r;
            const bool valid = t < t_end;
            const u32x4 kr = kt[s];
            float part[GH];
#pragma unroll
            for (int i = 0; i < GH; ++i) {
                float d = dot2<DT>(qv[i].x, kr[0], 0.f);
                d = dot2<DT>(qv[i].y, kr[1], d);
                d = dot2<DT>(qv[i].z, kr[2], d);
                part[i] = dot2<DT>(qv[i].w, kr[3], d);
            }
            // transposing reduction inside the quad (see the order of qv): afterwards lane u holds
            // the finished dot products of heads 4i + u
            const float rel = (float)(t - Lm1);                      // exact: |rel| < 2^24
#pragma unroll
            for (int i = 0; i < HPL; ++i) {
                const float yk = part[4 * i + 0] + dpp<kDppXor1>(part[4 * i + 1]);
                const float ys = part[4 * i + 2] + dpp<kDppXor1>(part[4 * i + 3]);
                float z = yk + dpp<kDppXor2>(ys);                    // head 4i + u, summed over the quad
                z = cross_quad_sum<LPR>(z);                          // ... and over the whole token row
                const float s2 = valid ? fmaf(z, scale2, slope2[i] * rel) : -INFINITY;   // eq. (3), base 2
                sc[s][i] = s2;
                tmax[i] = fmaxf(tmax[i], s2);
            }
        }
        // lazy rescale: when some head's tile maximum runs away from its reference, move every
        // reference of the wave to kRescaleHeadroom above the current maxima
        bool need = false;
#pragma unroll
        for (int i = 0; i < HPL; ++i) need |= tmax[i] > m_ref[i] + kRescaleThreshold;
        if (__builtin_amdgcn_ballot_w64(need) != 0) {
#pragma unroll
            for (int i = 0; i < HPL; ++i) {
                const float m_new = fmaxf(m_ref[i], tmax[i] + kRescaleHeadroom);
                const float alpha = fast_exp2(m_ref[i] - m_new);     // 1 when unchanged, 0 on first use
                l[i] *= alpha;
                m_ref[i] = m_new;
                const float a0 = quad_bcast<0>(alpha), a1 = quad_bcast<1>(alpha);
                const float a2 = quad_bcast<2>(alpha), a3 = quad_bcast<3>(alpha);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    acc[e][i][0] *= a0;
                    acc[e][i][1] *= a1;
                    acc[e][i][2] *= a2;
                    acc[e][i][3] *= a3;
                }
            }
        }
#pragma unroll
        for (int s = 0; s < U; ++s) {
            const u32x4 vr = vt[s];
            const float vf[8] = {widen_lo<DT>(vr[0]), widen_hi<DT>(vr[0]), widen_lo<DT>(vr[1]), widen_hi<DT>(vr[1]),
                                 widen_lo<DT>(vr[2]), widen_hi<DT>(vr[2]), widen_lo<DT>(vr[3]), widen_hi<DT>(vr[3])};
            float pw[HPL];
#pragma unroll
            for (int i = 0; i < HPL; ++i) {
                pw[i] = fast_exp2(sc[s][i] - m_ref[i]);              // eq. (4) numerator; 0 for absent keys
                l[i] += pw[i];
            }
#pragma unroll
            for (int e = 0; e < 8; ++e)
#pragma unroll
                for (int i = 0; i < HPL; ++i)
                    acc[e][i] = __builtin_amdgcn_mfma_f32_4x4x1f32(pw[i], vf[e], acc[e][i], 0, 0, 0);
        }
    };

    // ---- main loop -------------------------------------------------------------------------
    const uint32_t ring_lane = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)ring + lane * 16;
    for (int j = 0; j < PT && j < ntw; ++j) issue_tile(j);
    for (int j = 0; j < ntw; ++j) {
        if (j + PT < ntw) issue_tile(j + PT);
        const int newer = min(ntw - 1 - j, PT);              // tiles issued after tile j (uniform)
        const uint32_t addr = ring_lane + (j % NT) * kTileBytes;
        u32x4 kt[U], vt[U];
        static_assert(PT <= 7, "extend the switch");
        switch (newer) {
        case 0: ring_read2<0>(addr, kt[0], kt[1], vt[0], vt[1]); break;
        case 1: ring_read2<2 * U>(addr, kt[0], kt[1], vt[0], vt[1]); break;
        case 2: ring_read2<4 * U>(addr, kt[0], kt[1], vt[0], vt[1]); break;
        case 3: ring_read2<6 * U>(addr, kt[0], kt[1], vt[0], vt[1]); break;
        case 4: ring_read2<8 * U>(addr, kt[0], kt[1], vt[0], vt[1]); break;
        case 5: ring_read2<10 * U>(addr, kt[0], kt[1], vt[0], vt[1]); break;
        case 6: ring_read2<12 * U>(addr, kt[0], kt[1], vt[0], vt[1]); break;
        default: ring_read2<14 * U>(addr, kt[0], kt[1], vt[0], vt[1]); break;
        }
        compute_tile(kt, vt, tile_first + j);
    }

    // ---- merge the NSTREAM softmax streams of the workgroup --------------------------------
    float (*sm_o)[GH][D] = reinterpret_cast<float (*)[GH][D]>(smem);
    const int stream = wave * TPS + r;
    if (c < 4) {
#pragma unroll
        for (int i = 0; i < HPL; ++i) {
            sm_m[stream][u + 4 * i] = m_ref[i];
            sm_l[stream][u + 4 * i] = l[i];
        }
    }
    __syncthreads();                                        // also: every wave is done with its ring
    // every lane: the workgroup maximum of each head and this stream's factor against it
    float f[GH];
#pragma unroll
    for (int h = 0; h < GH; ++h) {
        float M = sm_m[0][h];
#pragma unroll
        for (int s = 1; s < NSTREAM; ++s) M = fmaxf(M, sm_m[s][h]);
        f[h] = fast_exp2(sm_m[stream][h] - M);              // a stream without keys: 2^(-1e30 - M) = 0
    }
    // output element(s) this thread finishes: one float4 of one head
    constexpr int kVecs = GH * D / 4;
    const int idx = threadIdx.x;
    const int oh = idx / (D / 4), od = (idx - oh * (D / 4)) * 4;
    float4 num = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        if (half) __syncthreads();                          // first half fully consumed
        if ((stream >= NSTREAM / 2) == (half == 1)) {
            const int sl = stream - half * (NSTREAM / 2);
#pragma unroll
            for (int h = 0; h < GH; ++h) {
                const int i = h >> 2, v = h & 3;
                *reinterpret_cast<float4*>(&sm_o[sl][h][8 * c]) =
                    make_float4(acc[0][i][v] * f[h], acc[1][i][v] * f[h], acc[2][i][v] * f[h], acc[3][i][v] * f[h]);
                *reinterpret_cast<float4*>(&sm_o[sl][h][8 * c + 4]) =
                    make_float4(acc[4][i][v] * f[h], acc[5][i][v] * f[h], acc[6][i][v] * f[h], acc[7][i][v] * f[h]);
            }
        }
        __syncthreads();
        if (idx < kVecs) {
#pragma unroll
            for (int s = 0; s < NSTREAM / 2; ++s) {
                const float4 x = *reinterpret_cast<const float4*>(&sm_o[s][oh][od]);
                num.x += x.x;
                num.y += x.y;
                num.z += x.z;
                num.w += x.w;
            }
        }
    }
    if (idx < kVecs) {
        float M = sm_m[0][oh];
#pragma unroll
        for (int s = 1; s < NSTREAM; ++s) M = fmaxf(M, sm_m[s][oh]);
        float den = 0.f;
#pragma unroll
        for (int s = 0; s < NSTREAM; ++s) den = fmaf(fast_exp2(sm_m[s][oh] - M), sm_l[s][oh], den);
        const int h = h0 + oh;
        const float inv = 1.f / den;
        uint2 packed;
        packed.x = narrow2<DT>(num.x * inv, num.y * inv);
        packed.y = narrow2<DT>(num.z * inv, num.w * inv);
        *reinterpret_cast<uint2*>(static_cast<uint16_t*>(p.out) + ((int64_t)row * Hq + h) * D + od) = packed;
    }
}

}  // namespace optgqa
