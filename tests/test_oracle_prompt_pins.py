"""The oracle's whole-prompt clause against its pins, and planted mistakes in a copy of that
source (each must fail at least one pin)."""
import ctypes
import os
import subprocess

import pytest

import oracle as O
import pins_prompt


@pytest.mark.parametrize("check", pins_prompt.ALL_CHECKS, ids=lambda f: f.__name__)
def test_pin(oracle, check):
    check(None)


SRC = os.path.join(os.path.dirname(O.__file__), "optgqa_oracle_prompt.c")

MUTANTS = {
    "own_key_left_out": ("for (int j = 0; j <= i; ++j) {\n            const uint16_t *k_row",
                   "for (int j = 0; j <= i; ++j) {\n            if (j == i && i + 1 < cu_seq_lens[b + 1] - first) { s[j] = -1e300; continue; }\n            const uint16_t *k_row"),
    "keys_from_the_batch_start": ("const uint16_t *k_row = k + ((int64_t)(first + j) * num_kv_heads + g) * head_dim;",
                                  "const uint16_t *k_row = k + ((int64_t)(j) * num_kv_heads + g) * head_dim;"),
    "values_from_the_batch_start": ("const uint16_t *v_row = v + ((int64_t)(first + j) * num_kv_heads + g) * head_dim;",
                                    "const uint16_t *v_row = v + ((int64_t)(j) * num_kv_heads + g) * head_dim;"),
    "position_in_the_batch": ("int i = t - first;                     /* this query's position */",
                              "int i = t;"),
    "bias_sign": ("s[j] = (double)scale * dot + slope * (double)(j - i);", "s[j] = (double)scale * dot + slope * (double)(i - j);"),
    "bias_scaled": ("s[j] = (double)scale * dot + slope * (double)(j - i);", "s[j] = (double)scale * (dot + slope * (double)(j - i));"),
    "scale_dropped": ("s[j] = (double)scale * dot + slope * (double)(j - i);", "s[j] = dot + slope * (double)(j - i);"),
    "kv_head_interleaved": ("int g = h / group;", "int g = h % num_kv_heads;"),
    "values_are_keys": ("for (int d = 0; d < head_dim; ++d) o[d] += w * prompt_elem(v_row[d], dtype);",
                        "for (int d = 0; d < head_dim; ++d) o[d] += w * prompt_elem(k[(v_row - v) + d], dtype);"),
    "not_normalised": ("double w = s[j] / denom;", "double w = s[j];"),
    "sequence_boundary_off_by_one": ("while (b + 1 < num_seqs && cu_seq_lens[b + 1] <= t) ++b;",
                                     "while (b + 1 < num_seqs && cu_seq_lens[b + 1] < t) ++b;"),
    # the file's own 2-byte decoder
    "decoder_f16_subnormal_step": ("if (e == 0) v = ldexp((double)m, -24);", "if (e == 0) v = ldexp((double)m, -23);"),
    "decoder_bf16_infinity_is_nan": ("else if (e == 255) v = m ? NAN : INFINITY;", "else if (e == 255) v = NAN;"),
    "decoder_bf16_exponent_bias": ("else v = ldexp(1.0 + (double)m / 128.0, e - 127);", "else v = ldexp(1.0 + (double)m / 128.0, e - 126);"),
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
    for check in pins_prompt.ALL_CHECKS:
        try:
            check(lib)
        except AssertionError:
            failed.append(check.__name__)
    assert failed, f"mutant {name} passed every pin"
