// KV-cache write and the un-paging diagnostic: pure index work and bit copies.
#pragma once
#include "common.hpp"

namespace optgqa {

// Cache store of Alg. 1 / eq. (2).  One thread moves one 16-byte piece (8 elements) of one
// token's K row or V row; pieces of a row are handled by consecutive lanes, so reads and
// writes are contiguous runs of head_dim * 2 bytes.
//   grid.x covers num_tokens * pieces_per_token * 2 threads (K pieces then V pieces).
//   slot_mapping == nullptr (decode step): token t is the newest token of sequence t and goes to
//   position context_lens[t] - 1, whose slot is read from the block table; empty sequences skip.
template <typename VecT>
__global__ __launch_bounds__(256) void reshape_and_cache_kernel(
    const uint16_t* __restrict__ k, const uint16_t* __restrict__ v, uint16_t* __restrict__ k_cache,
    uint16_t* __restrict__ v_cache, const int64_t* __restrict__ slot_mapping, int num_tokens,
    int num_kv_heads, int head_dim, int block_size, int64_t k_token_stride, int64_t v_token_stride,
    const int32_t* __restrict__ block_tables = nullptr, const int32_t* __restrict__ context_lens = nullptr,
    int max_blocks_per_seq = 0)
{
    constexpr int kElems = sizeof(VecT) / 2;
    const int pieces_per_head = head_dim / kElems;
    const int pieces_per_token = num_kv_heads * pieces_per_head;
    const int64_t total = (int64_t)num_tokens * pieces_per_token * 2;
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const int which = (int)(idx / ((int64_t)num_tokens * pieces_per_token));   // 0 = K, 1 = V
    const int64_t rem = idx - (int64_t)which * num_tokens * pieces_per_token;
    const int t = (int)(rem / pieces_per_token);
    const int piece = (int)(rem - (int64_t)t * pieces_per_token);
    int64_t slot;
    if (slot_mapping) {
        slot = slot_mapping[t];
    } else {
        const int pos = context_lens[t] - 1;
        if (pos < 0) return;
        slot = (int64_t)block_tables[(int64_t)t * max_blocks_per_seq + pos / block_size] * block_size + pos % block_size;
    }
    if (slot < 0) return;                                   // padding token
    const int g = piece / pieces_per_head;
    const int d0 = (piece - g * pieces_per_head) * kElems;
    const int64_t block = slot / block_size;
    const int64_t row = slot - block * block_size;
    const int64_t dst = ((block * num_kv_heads + g) * block_size + row) * head_dim + d0;
    const int64_t src_off = (int64_t)g * head_dim + d0;
    if (which == 0)
        *reinterpret_cast<VecT*>(k_cache + dst) = *reinterpret_cast<const VecT*>(k + t * k_token_stride + src_off);
    else
        *reinterpret_cast<VecT*>(v_cache + dst) = *reinterpret_cast<const VecT*>(v + t * v_token_stride + src_off);
}

// Cache store with a quantiser in front, for caches that hold 1-byte E4M3 codes (largest finite
// value 448, no infinities) and one scale per tensor, or - k_scales / v_scales given, device arrays
// of num_kv_heads values - one per KV head:
//     code = nearest_e4m3( fp32(x) * inv_scale ),  inv_scale = fp32(1 / scale): one correctly rounded
// fp32 division, on the host for the per-tensor scale, here for a KV head's.
// One fp32 multiplication, then e4m3_codes2 (round to nearest even, saturating, NaN -> 0x7f).
// One thread moves 8 elements of one token's K or V row: 16 bytes in, 8 bytes out.
template <int DT>
__global__ __launch_bounds__(256) void reshape_and_cache_e4m3_kernel(
    const uint16_t* __restrict__ k, const uint16_t* __restrict__ v, unsigned char* __restrict__ k_cache,
    unsigned char* __restrict__ v_cache, const int64_t* __restrict__ slot_mapping, int num_tokens,
    int num_kv_heads, int head_dim, int block_size, int64_t k_token_stride, int64_t v_token_stride,
    float k_inv_scale, float v_inv_scale, const float* __restrict__ k_scales, const float* __restrict__ v_scales)
{
    const int pieces_per_head = head_dim / 8;
    const int pieces_per_token = num_kv_heads * pieces_per_head;
    const int64_t total = (int64_t)num_tokens * pieces_per_token * 2;
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const int which = (int)(idx / ((int64_t)num_tokens * pieces_per_token));   // 0 = K, 1 = V
    const int64_t rem = idx - (int64_t)which * num_tokens * pieces_per_token;
    const int t = (int)(rem / pieces_per_token);
    const int piece = (int)(rem - (int64_t)t * pieces_per_token);
    const int64_t slot = slot_mapping[t];
    if (slot < 0) return;                                   // padding token
    const int g = piece / pieces_per_head;
    const int d0 = (piece - g * pieces_per_head) * 8;
    const int64_t block = slot / block_size;
    const int64_t row = slot - block * block_size;
    const int64_t dst = ((block * num_kv_heads + g) * block_size + row) * head_dim + d0;
    const uint16_t* src = which == 0 ? k + t * k_token_stride : v + t * v_token_stride;
    float inv = which == 0 ? k_inv_scale : v_inv_scale;
    if (k_scales) inv = 1.0f / (which == 0 ? k_scales[g] : v_scales[g]);
    const uint4 x = *reinterpret_cast<const uint4*>(src + (int64_t)g * head_dim + d0);
    const uint32_t w[4] = {x.x, x.y, x.z, x.w};
    uint32_t packed[2] = {0u, 0u};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t two = e4m3_codes2(widen_lo<DT>(w[i]) * inv, widen_hi<DT>(w[i]) * inv);
        packed[i >> 1] |= two << (16 * (i & 1));
    }
    unsigned char* out = (which == 0 ? k_cache : v_cache) + dst;
    *reinterpret_cast<uint2*>(out) = make_uint2(packed[0], packed[1]);
}

// Un-paging: copy token j of sequence b, all KV heads, to dense [B][max_context_len][Hkv][D].
// One thread per 16-byte piece; grid = (ceil(max_context_len * pieces_per_token / 256), B, 2).
__global__ __launch_bounds__(256) void gather_kv_kernel(
    uint16_t* __restrict__ k_out, uint16_t* __restrict__ v_out, const uint16_t* __restrict__ k_cache,
    const uint16_t* __restrict__ v_cache, const int32_t* __restrict__ block_tables,
    const int32_t* __restrict__ context_lens, int num_kv_heads, int head_dim, int block_size,
    int max_blocks_per_seq, int max_context_len)
{
    const int b = blockIdx.y;
    const int pieces_per_head = head_dim / 8;
    const int pieces_per_token = num_kv_heads * pieces_per_head;
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int j = (int)(idx / pieces_per_token);
    if (j >= context_lens[b] || j >= max_context_len) return;
    const int piece = (int)(idx - (int64_t)j * pieces_per_token);
    const int g = piece / pieces_per_head;
    const int d0 = (piece - g * pieces_per_head) * 8;
    const int64_t block = block_tables[(int64_t)b * max_blocks_per_seq + j / block_size];
    const int64_t src = ((block * num_kv_heads + g) * block_size + (j % block_size)) * head_dim + d0;
    const int64_t dst = (((int64_t)b * max_context_len + j) * num_kv_heads + g) * head_dim + d0;
    const uint16_t* cache = blockIdx.z == 0 ? k_cache : v_cache;
    uint16_t* out = blockIdx.z == 0 ? k_out : v_out;
    *reinterpret_cast<uint4*>(out + dst) = *reinterpret_cast<const uint4*>(cache + src);
}

}  // namespace optgqa
