"""The oracle's 8-bit (E4M3) KV-cache clauses against their pins, and planted mistakes in a copy
of that source (each must fail at least one pin)."""
import ctypes
import os
import subprocess

import pytest

import oracle as O
import pins_e4m3


@pytest.mark.parametrize("check", pins_e4m3.ALL_CHECKS, ids=lambda f: f.__name__)
def test_pin(oracle, check):
    check(None)


SRC = os.path.join(os.path.dirname(O.__file__), "optgqa_oracle_e4m3.c")

MUTANTS = {
    "exponent_bias": ("else v = ldexp(1.0 + (double)m / 8.0, e - 7);\n    return sign ? -v : v;\n}\n\n/* The two decoders",
                      "else v = ldexp(1.0 + (double)m / 8.0, e - 8);\n    return sign ? -v : v;\n}\n\n/* The two decoders"),
    "subnormal_step": ("else if (e == 0) v = ldexp((double)m, -9);", "else if (e == 0) v = ldexp((double)m, -10);"),
    "nan_code_is_a_number": ("if (e == 15 && m == 7) v = NAN;", "if (0) v = NAN;"),
    "truncates": ("int q = (int)nearbyint(ldexp(f, 4)) - 8;", "int q = (int)floor(ldexp(f, 4)) - 8;"),
    "ties_away": ("int q = (int)nearbyint(ldexp(f, 4)) - 8;", "int q = (int)round(ldexp(f, 4)) - 8;"),
    "subnormal_truncates": ("int q = (int)nearbyint(ldexp(a, 9));", "int q = (int)floor(ldexp(a, 9));"),
    "no_saturation": ("if (a > 448.0) return sign | 0x7e;", "if (a > 448.0) return sign | 0x7f;"),
    "mantissa_carry_lost": ("if (q == 8) { q = 0; e += 1; }", "if (q == 8) { q = 7; }"),
    "wrong_exponent_bias_in_encoder": ("return sign | (uint8_t)(((e + 7) << 3) | q);", "return sign | (uint8_t)(((e + 8) << 3) | q);"),
    "v_uses_k_scale": ("volatile float vp = vf * v_inv;", "volatile float vp = vf * k_inv;"),
    "multiplies_by_scale": ("const float k_inv = 1.0f / k_scale, v_inv = 1.0f / v_scale;",
                            "const float k_inv = k_scale, v_inv = v_scale;"),
    "cache_layout": ("int64_t dst = ((block * num_kv_heads + g) * block_size + row) * head_dim;",
                     "int64_t dst = ((block * block_size + row) * num_kv_heads + g) * head_dim;"),
    "k_scale_dropped": ("s[j] = scale * k_scale * dot + slope", "s[j] = scale * dot + slope"),
    "v_scale_dropped": ("for (int d = 0; d < head_dim; ++d) out_row[d] *= v_scale;", ""),
    "bias_scaled_by_k_scale": ("s[j] = scale * k_scale * dot + slope * (double)(j - pos_q);",
                               "s[j] = k_scale * (scale * dot + slope * (double)(j - pos_q));"),
    "prefill_not_causal": ("block_tables + (int64_t)b * max_blocks_per_seq, pos + 1, pos,\n                        h / group",
                           "block_tables + (int64_t)b * max_blocks_per_seq, context_lens[b], pos,\n                        h / group"),
    "prefill_ignores_prefix": ("int pos = context_lens[b] - new_tokens + (t - cu_q_lens[b]);", "int pos = (t - cu_q_lens[b]);"),
    "v_read_from_k": ("out_row[d] += w * e4m3_value(v_cache[at + d]);", "out_row[d] += w * e4m3_value(k_cache[at + d]);"),
    # one scale pair per KV head
    "heads_write_uses_head_zero": ("const float k_inv_g = 1.0f / k_scales[g], v_inv_g = 1.0f / v_scales[g];",
                                   "const float k_inv_g = 1.0f / k_scales[0], v_inv_g = 1.0f / v_scales[0];"),
    "heads_write_v_with_k_scales": ("volatile float vq = vf * v_inv_g;", "volatile float vq = vf * k_inv_g;"),
    "heads_decode_scale_of_query_head": ("int kv = h / group;                                  /* the KV head this query head reads */",
                                         "int kv = h % num_kv_heads;"),
    "heads_decode_v_scale_of_next_head": ("kv, slope, (double)scale, (double)k_scales[kv], (double)v_scales[kv],\n                        num_kv_heads, head_dim, block_size, dtype);\n    }\n}\n\nvoid oracle_paged_prefill_e4m3_heads",
                                          "kv, slope, (double)scale, (double)k_scales[kv], (double)v_scales[(kv + 1) % num_kv_heads],\n                        num_kv_heads, head_dim, block_size, dtype);\n    }\n}\n\nvoid oracle_paged_prefill_e4m3_heads"),
    "heads_prefill_k_scale_of_head_zero": ("int kv = h / group;\n        double slope = alibi_slopes ? (double)alibi_slopes[h] : 0.0;\n        attend_row_e4m3(out + (int64_t)r * head_dim, q + ((int64_t)t * num_heads + h) * head_dim,\n                        k_cache, v_cache, block_tables + (int64_t)b * max_blocks_per_seq, pos + 1, pos,\n                        kv, slope, (double)scale, (double)k_scales[kv],",
                                           "int kv = h / group;\n        double slope = alibi_slopes ? (double)alibi_slopes[h] : 0.0;\n        attend_row_e4m3(out + (int64_t)r * head_dim, q + ((int64_t)t * num_heads + h) * head_dim,\n                        k_cache, v_cache, block_tables + (int64_t)b * max_blocks_per_seq, pos + 1, pos,\n                        kv, slope, (double)scale, (double)k_scales[0],"),
    # the file's own 2-byte decoder (queries and new-token rows)
    "two_byte_f16_subnormal_step": ("if (e == 0) v = ldexp((double)m, -24);\n        else if (e == 31) v = m ? NAN : INFINITY;\n        else v = ldexp(1.0 + (double)m / 1024.0, e - 15);\n    } else {\n        int e = (h >> 7) & 0xFF, m = h & 0x7F;\n        if (e == 0) v = ldexp((double)m, -133);\n        else if (e == 255) v = m ? NAN : INFINITY;\n        else v = ldexp(1.0 + (double)m / 128.0, e - 127);\n    }\n    return sign ? -v : v;\n}\n\nstatic double e4m3_value_formula",
                                    "if (e == 0) v = ldexp((double)m, -25);\n        else if (e == 31) v = m ? NAN : INFINITY;\n        else v = ldexp(1.0 + (double)m / 1024.0, e - 15);\n    } else {\n        int e = (h >> 7) & 0xFF, m = h & 0x7F;\n        if (e == 0) v = ldexp((double)m, -133);\n        else if (e == 255) v = m ? NAN : INFINITY;\n        else v = ldexp(1.0 + (double)m / 128.0, e - 127);\n    }\n    return sign ? -v : v;\n}\n\nstatic double e4m3_value_formula"),
    "two_byte_bf16_infinity_is_finite": ("else if (e == 255) v = m ? NAN : INFINITY;\n        else v = ldexp(1.0 + (double)m / 128.0, e - 127);\n    }\n    return sign ? -v : v;\n}\n\nstatic double e4m3_value_formula",
                                         "else if (e == 255 && m) v = NAN;\n        else v = ldexp(1.0 + (double)m / 128.0, e - 127);\n    }\n    return sign ? -v : v;\n}\n\nstatic double e4m3_value_formula"),
    "two_byte_bf16_mantissa_width": ("else v = ldexp(1.0 + (double)m / 128.0, e - 127);\n    }\n    return sign ? -v : v;\n}\n\nstatic double e4m3_value_formula",
                                     "else v = ldexp(1.0 + (double)m / 256.0, e - 127);\n    }\n    return sign ? -v : v;\n}\n\nstatic double e4m3_value_formula"),
}


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_mutant_is_caught(name, tmp_path, oracle):
    old, new = MUTANTS[name]
    text = open(SRC).read()
    assert text.count(old) == 1, f"mutation site for {name} not found exactly once"
    src = tmp_path / f"mutant_{name}.c"
    src.write_text(text.replace(old, new, 1))
    lib_path = str(tmp_path / f"libmutant_{name}.so")
    subprocess.check_call(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
                           "-o", lib_path, str(src), "-lm"])
    lib = ctypes.CDLL(lib_path)
    failed = []
    for check in pins_e4m3.ALL_CHECKS:
        try:
            check(lib)
        except AssertionError:
            failed.append(check.__name__)
    assert failed, f"mutant {name} passed every pin"
