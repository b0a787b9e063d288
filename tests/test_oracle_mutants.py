"""Planted mistakes, on the CPU, in copies of the oracle: each must fail at least one pin.

A copy of the oracle's C source gets one plausible slip (a sign, an index, a dropped term, a
transposed layout), is compiled to a temporary library, and the whole pin list is run against
it.  This shows the pins are strong enough to notice; the committed oracle is never modified.
"""
import ctypes
import os
import subprocess

import pytest

import oracle as O
import pins

SRC = os.path.join(os.path.dirname(O.__file__), "optgqa_oracle.c")

MUTANTS = {
    "bias_sign": ("slope * (double)(j - pos_q)", "slope * (double)(pos_q - j)"),
    "bias_scaled": ("s[j] = scale * dot + slope * (double)(j - pos_q);",
                    "s[j] = scale * (dot + slope * (double)(j - pos_q));"),
    "scale_dropped": ("s[j] = scale * dot + slope", "s[j] = dot + slope"),
    "bias_dropped": ("s[j] = scale * dot + slope * (double)(j - pos_q);", "s[j] = scale * dot;"),
    "group_map_interleaved": ("L, L - 1, h / group,\n                   slope, (double)scale, num_kv_heads, head_dim, block_size, dtype);\n    }\n}\n\n/* Same",
                              "L, L - 1, h % num_kv_heads,\n                   slope, (double)scale, num_kv_heads, head_dim, block_size, dtype);\n    }\n}\n\n/* Same"),
    "row_off_by_one": ("int64_t row = j % block_size;\n        const uint16_t *k_j",
                       "int64_t row = (j + 1) % block_size;\n        const uint16_t *k_j"),
    "v_row_off_by_one": ("int64_t row = j % block_size;\n        const uint16_t *v_j",
                         "int64_t row = (j + 1) % block_size;\n        const uint16_t *v_j"),
    "layout_transposed": ("const uint16_t *k_j = k_cache + ((block * num_kv_heads + kv_head) * block_size + row) * head_dim;",
                          "const uint16_t *k_j = k_cache + ((block * block_size + row) * num_kv_heads + kv_head) * head_dim;"),
    "not_normalised": ("double w = s[j] / denom;", "double w = s[j];"),
    "k_used_for_v": ("const uint16_t *v_j = v_cache + ((block * num_kv_heads + kv_head)",
                     "const uint16_t *v_j = k_cache + ((block * num_kv_heads + kv_head)"),
    "prefill_not_causal": ("block_tables + (int64_t)b * max_blocks_per_seq, pos + 1, pos, h / group,\n                   slope, (double)scale, num_kv_heads, head_dim, block_size, dtype);\n    }\n}\n\n/* Prefill for",
                           "block_tables + (int64_t)b * max_blocks_per_seq, context_lens[b], pos, h / group,\n                   slope, (double)scale, num_kv_heads, head_dim, block_size, dtype);\n    }\n}\n\n/* Prefill for"),
    "prefill_ignores_prefix": ("int pos = context_lens[b] - q_len + (t - cu_q_lens[b]);\n        double slope = alibi_slopes ? (double)alibi_slopes[h] : 0.0;\n        attend_row(out + (int64_t)u",
                               "int pos = (t - cu_q_lens[b]);\n        double slope = alibi_slopes ? (double)alibi_slopes[h] : 0.0;\n        attend_row(out + (int64_t)u"),
    "cache_write_layout": ("int64_t dst = ((block * num_kv_heads + g) * block_size + row) * head_dim;",
                           "int64_t dst = ((block * block_size + row) * num_kv_heads + g) * head_dim;"),
    "cache_write_v_gets_k": ("v_cache[dst + d] = v[t * v_token_stride", "v_cache[dst + d] = k[t * v_token_stride"),
    "f16_exponent": ("ldexp((double)(m + 1024), e - 25)", "ldexp((double)(m + 1024), e - 24)"),
    "f16_subnormal": ("ldexp((double)m, -24)", "ldexp((double)m, -25)"),
    "bf16_shift": ("((uint32_t)h) << 16", "((uint32_t)h) << 15"),
    "partition_drops_l": ("double w = exp(m_p[p] - m) * l_p[p] / denom;", "double w = exp(m_p[p] - m) / denom;"),
    "partition_wrong_max": ("if (m_p[p] > m) m = m_p[p];", "if (m_p[p] < m || p == 0) m = m_p[p];"),
    "decode_pos_is_L": ("block_tables + (int64_t)b * max_blocks_per_seq, L, L - 1, h / group,\n                   slope, (double)scale, num_kv_heads, head_dim, block_size, dtype);\n    }\n}\n\n/* Same",
                        "block_tables + (int64_t)b * max_blocks_per_seq, L - 1, L - 1, h / group,\n                   slope, (double)scale, num_kv_heads, head_dim, block_size, dtype);\n    }\n}\n\n/* Same"),
}


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_mutant_is_caught(name, tmp_path, oracle):
    old, new = MUTANTS[name]
    text = open(SRC).read()
    assert text.count(old) >= 1, f"mutation site for {name} not found in the oracle source"
    mutated = text.replace(old, new, 1)
    src = tmp_path / f"mutant_{name}.c"
    src.write_text(mutated)
    lib_path = str(tmp_path / f"libmutant_{name}.so")
    subprocess.check_call(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-fopenmp",
                           "-ffp-contract=off", "-o", lib_path, str(src), "-lm"])
    lib = O.load(lib_path)
    failed = []
    for check in pins.ALL_CHECKS:
        try:
            check(lib)
        except AssertionError:
            failed.append(check.__name__)
    assert failed, f"mutant {name} passed every pin"
