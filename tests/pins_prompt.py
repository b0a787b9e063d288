"""Pins of the oracle's whole-prompt clause (oracle/optgqa_oracle_prompt.c): checks against things
other than that file - the already pinned paged prefill oracle, a dense numpy / scipy formulation,
special cases.  Each check takes the ctypes library to test (None: the built oracle)."""
import numpy as np
import scipy.special

import oracle as O
import workloads as W


def _case(dtype, seed, Hq=8, Hkv=2, batch=3):
    # q_len >= the longest context: every token of every sequence is new
    cfg = W.small_config(name="prompt", kind="prefill", dtype=dtype, batch=batch, num_heads=Hq, num_kv_heads=Hkv,
                         head_dim=16, block_size=4, num_blocks=64, ctx_lo=1, ctx_hi=33, q_len=33, seed=seed)
    case = W.make_case(cfg)
    assert np.array_equal(case.q_lens, case.context_lens)
    return case


def check_equals_paged_prefill_after_the_cache_write(lib=None):
    """Writing the prompt's K/V into the paged cache and running the pinned prefill oracle over the
    cache (all tokens new) computes the same thing by another route."""
    for dtype, Hq, Hkv in ((W.F16, 8, 2), (W.BF16, 6, 6), (W.BF16, 4, 1)):
        case = _case(dtype, 11 + Hq, Hq, Hkv)
        kc, vc = case.k_cache.copy(), case.v_cache.copy()
        O.reshape_and_cache(case.k_new, case.v_new, kc, vc, case.slot_mapping)
        ref = O.paged_prefill(case.q, kc, vc, case.block_tables, case.context_lens, case.cu_q_lens, case.slopes,
                              case.scale, dtype)
        got = O.prompt_attention(case.q, case.k_new, case.v_new, case.cu_q_lens, case.slopes, case.scale, dtype,
                                 lib=lib)
        np.testing.assert_allclose(got, ref, rtol=1e-13, atol=1e-13)
        got = O.prompt_attention(case.q, case.k_new, case.v_new, case.cu_q_lens, None, case.scale, dtype, lib=lib)
        ref = O.paged_prefill(case.q, kc, vc, case.block_tables, case.context_lens, case.cu_q_lens, None,
                              case.scale, dtype)
        np.testing.assert_allclose(got, ref, rtol=1e-13, atol=1e-13)


def check_against_dense_lower_triangular_mask(lib=None):
    for dtype in (W.F16, W.BF16):
        case = _case(dtype, 21)
        got = O.prompt_attention(case.q, case.k_new, case.v_new, case.cu_q_lens, case.slopes, case.scale, dtype,
                                 lib=lib)
        Q = W.from_bits(case.q, dtype)
        K = W.from_bits(case.k_new, dtype)
        V = W.from_bits(case.v_new, dtype)
        G = case.cfg.num_heads // case.cfg.num_kv_heads
        for b in range(case.cfg.batch):
            a, e = int(case.cu_q_lens[b]), int(case.cu_q_lens[b + 1])
            n = e - a
            mask = np.where(np.tril(np.ones((n, n))) > 0, 0.0, -np.inf)
            rel = np.arange(n)[None, :] - np.arange(n)[:, None]
            for h in range(case.cfg.num_heads):
                scores = float(case.scale) * Q[a:e, h] @ K[a:e, h // G].T + float(case.slopes[h]) * rel + mask
                np.testing.assert_allclose(got[a:e, h], scipy.special.softmax(scores, axis=1) @ V[a:e, h // G],
                                           rtol=1e-11, atol=1e-12)


def check_first_token_returns_its_own_value_row(lib=None):
    case = _case(W.F16, 23)
    got = O.prompt_attention(case.q, case.k_new, case.v_new, case.cu_q_lens, case.slopes, case.scale, W.F16, lib=lib)
    V = W.from_bits(case.v_new, W.F16)
    for b in range(case.cfg.batch):
        t = int(case.cu_q_lens[b])
        for h in range(case.cfg.num_heads):
            assert np.array_equal(got[t, h], V[t, h // 4])


def check_decoder_on_every_two_byte_pattern(lib=None):
    """All 65 536 fp16 and bf16 patterns (subnormals, infinities, NaNs) as the V row of a one-token
    prompt: token 0 attends to itself with weight exactly 1, so the output is the decoder's value
    of each pattern, compared with numpy's own decoding."""
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    for dtype in (W.F16, W.BF16):
        want = W.from_bits(bits, dtype)
        D = 65536
        zeros = np.zeros((1, 1, D), np.uint16)
        out = O.prompt_attention(zeros, zeros, bits.reshape(1, 1, D).copy(), np.array([0, 1], np.int32),
                                 np.ones(1, np.float32), 1.0, dtype, lib=lib)[0, 0]
        fin = np.isfinite(want)
        assert np.array_equal(out[fin], want[fin]), f"{dtype} decoding"
        inf = np.isinf(want)
        assert np.array_equal(out[inf], want[inf]), f"{dtype} infinities"
        assert np.all(np.isnan(out[np.isnan(want)])), f"{dtype} NaN patterns"


def check_sequences_do_not_see_each_other(lib=None):
    """Each sequence alone gives the rows it gives inside the batch; row lists pick the same rows."""
    case = _case(W.BF16, 25)
    full = O.prompt_attention(case.q, case.k_new, case.v_new, case.cu_q_lens, case.slopes, case.scale, W.BF16,
                              lib=lib)
    for b in range(case.cfg.batch):
        a, e = int(case.cu_q_lens[b]), int(case.cu_q_lens[b + 1])
        alone = O.prompt_attention(case.q[a:e], case.k_new[a:e], case.v_new[a:e], np.array([0, e - a], np.int32),
                                   case.slopes, case.scale, W.BF16, lib=lib)
        np.testing.assert_allclose(alone, full[a:e], rtol=0, atol=0)
    T = case.num_tokens
    rows = [(0, 0), (T - 1, 7), (T // 2, 3), (1, 5)]
    sub = O.prompt_attention(case.q, case.k_new, case.v_new, case.cu_q_lens, case.slopes, case.scale, W.BF16,
                             rows=rows, lib=lib)
    assert np.array_equal(sub, np.stack([full[t, h] for t, h in rows]))


ALL_CHECKS = [
    check_equals_paged_prefill_after_the_cache_write,
    check_against_dense_lower_triangular_mask,
    check_first_token_returns_its_own_value_row,
    check_decoder_on_every_two_byte_pattern,
    check_sequences_do_not_see_each_other,
]
