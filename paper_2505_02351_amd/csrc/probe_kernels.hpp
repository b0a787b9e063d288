// Measurement aid: the decode kernels' memory access pattern with no arithmetic behind it.
//
// Persistent waves, one per SIMD (or more, the caller chooses), each streaming its own list of
// 16-token tiles out of the real K and V pools: per tile four 16-byte loads per lane in the K
// operand order of the decode kernels (16 rows x 64 contiguous bytes per load) and four in the V
// order (4 rows x 256 contiguous bytes per load), one tile of loads ahead of the consumer, which
// only XORs the registers together.  Whatever this reaches is what the memory system delivers
// for this pattern on this chip; the attention kernels are priced against it as well as against
// the nominal HBM peak.
#pragma once
#include "common.hpp"

namespace optgqa {

struct ProbeTile { uint4 r[8]; };

__global__ __launch_bounds__(256, 2) void stream_probe_kernel(
    const unsigned char* __restrict__ k_pool, const unsigned char* __restrict__ v_pool,
    const int32_t* __restrict__ tile_list,      // [waves][tiles_per_wave]: index of a 4 KiB piece of each pool
    int tiles_per_wave, uint4* __restrict__ sink)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int32_t* __restrict__ mine = tile_list + (int64_t)(blockIdx.x * 4 + wave) * tiles_per_wave;
    const int row = lane & 15, slab = lane >> 4;
    auto load = [&](ProbeTile& T, int j) __attribute__((always_inline)) {
        const int64_t piece = __builtin_amdgcn_readfirstlane(mine[j]);
        const unsigned char* kp = k_pool + piece * 4096;
        const unsigned char* vp = v_pool + piece * 4096;
#pragma unroll
        for (int i = 0; i < 4; ++i) T.r[i] = stream_load16(kp + row * 256 + 64 * i + 16 * slab);
#pragma unroll
        for (int i = 0; i < 4; ++i) T.r[4 + i] = stream_load16(vp + lane * 16 + 1024 * i);
    };
    ProbeTile buf[2];
    uint4 acc = make_uint4(0, 0, 0, 0);
    const int j_last = tiles_per_wave - 1;
    load(buf[0], 0);
    for (int j = 0; j < tiles_per_wave; j += 2) {
        load(buf[1], min(j + 1, j_last));
#pragma unroll
        for (int e = 0; e < 8; ++e) { acc.x ^= buf[0].r[e].x; acc.y ^= buf[0].r[e].y; acc.z ^= buf[0].r[e].z; acc.w ^= buf[0].r[e].w; }
        load(buf[0], min(j + 2, j_last));
        if (j + 1 <= j_last) {
#pragma unroll
            for (int e = 0; e < 8; ++e) { acc.x ^= buf[1].r[e].x; acc.y ^= buf[1].r[e].y; acc.z ^= buf[1].r[e].z; acc.w ^= buf[1].r[e].w; }
        }
    }
    // keeps the loads alive; the store itself practically never happens
    if (acc.x == 0x12345678u && acc.y == 0x9abcdef0u && acc.z == 0x0fedcba9u) sink[0] = acc;
}

}  // namespace optgqa
