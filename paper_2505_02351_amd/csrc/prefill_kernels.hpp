// Prefill over the paged cache: several new query tokens per sequence, causal mask + ALiBi.
#pragma once
#include "common.hpp"

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
    float scale2;               // scale * log2(e)
    int num_heads, num_kv_heads, block_size, max_blocks_per_seq;
};

}  // namespace optgqa
