"""The oracle's sliding-window clauses against their pins, and planted mistakes in a copy of that
source (each must fail at least one pin)."""
import ctypes
import os
import subprocess

import pytest

import oracle as O
import pins_window


@pytest.mark.parametrize("check", pins_window.ALL_CHECKS, ids=lambda f: f.__name__)
def test_pin(oracle, check):
    check(None)


SRC = os.path.join(os.path.dirname(O.__file__), "optgqa_oracle_window.c")

MUTANTS = {
    "window_one_key_too_many": ("int local_ok = window <= 0 || j > pos - window;",
                                "int local_ok = window <= 0 || j >= pos - window;"),
    "window_one_key_too_few": ("int local_ok = window <= 0 || j > pos - window;",
                               "int local_ok = window <= 0 || j > pos - window + 1;"),
    "window_counted_from_the_context_end": ("int local_ok = window <= 0 || j > pos - window;",
                                            "int local_ok = window <= 0 || j > n_ctx - 1 - window;"),
    "not_causal": ("int causal_ok = j <= pos;", "int causal_ok = 1;"),
    "strictly_causal": ("int causal_ok = j <= pos;", "int causal_ok = j < pos || pos == 0;"),
    "bias_relative_to_window_start": ("s[j] = scale * dot + slope * (double)(j - pos) + mask;",
                                      "s[j] = scale * dot + slope * (double)(j - (pos - window + 1)) * (window > 0 ? -1 : 1) + mask;"),
    "bias_sign": ("s[j] = scale * dot + slope * (double)(j - pos) + mask;",
                  "s[j] = scale * dot + slope * (double)(pos - j) + mask;"),
    "masked_keys_counted_in_the_sum": ("s[j] = exp(s[j] - m);              /* exp(-inf) = 0 for masked keys */\n        denom += s[j];",
                                       "s[j] = exp(s[j] - m);\n        denom += s[j] > 0 ? s[j] : 1e-3;"),
    "prefill_position_from_chunk_start": ("int pos = context_lens[b] - new_tokens + (t - cu_q_lens[b]);",
                                          "int pos = (t - cu_q_lens[b]);"),
    "decode_position_is_context_length": ("block_tables + (int64_t)b * max_blocks_per_seq, L, L - 1,",
                                          "block_tables + (int64_t)b * max_blocks_per_seq, L, L,"),
    "v_read_from_k": ("out_row[d] += w * elem_value(v_cache[at + d], dtype);",
                      "out_row[d] += w * elem_value(k_cache[at + d], dtype);"),
    "kv_head_of_the_wrong_group": ("window, h / group, slope, (double)scale, num_kv_heads, head_dim,\n                          block_size, dtype);\n    }\n}\n\n/* Prefill",
                                   "window, h % num_kv_heads, slope, (double)scale, num_kv_heads, head_dim,\n                          block_size, dtype);\n    }\n}\n\n/* Prefill"),
    "scale_dropped": ("s[j] = scale * dot + slope * (double)(j - pos) + mask;",
                      "s[j] = dot + slope * (double)(j - pos) + mask;"),
    # the file's own 2-byte decoder
    "decoder_bf16_subnormal_step": ("if (e == 0) v = ldexp((double)m, -133);", "if (e == 0) v = ldexp((double)m, -134);"),
    "decoder_f16_nan_is_infinity": ("else if (e == 31) v = m ? NAN : INFINITY;", "else if (e == 31) v = INFINITY;"),
    "decoder_f16_sign_lost_on_subnormals": ("if (e == 0) v = ldexp((double)m, -24);", "if (e == 0) return ldexp((double)m, -24);"),
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
    for check in pins_window.ALL_CHECKS:
        try:
            check(lib)
        except AssertionError:
            failed.append(check.__name__)
    assert failed, f"mutant {name} passed every pin"
