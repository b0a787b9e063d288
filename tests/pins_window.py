"""Pins of the oracle's sliding-window clauses (oracle/optgqa_oracle_window.c): checks against
things other than that file - the already pinned full-context oracle, numpy indexing, a dense
numpy / scipy formulation with an explicit banded mask matrix.  Each check takes the ctypes
library to test (None: the built oracle), so that planted mistakes can be run through them."""
import numpy as np
import scipy.special

import oracle as O
import workloads as W


def _filled(case):
    """Cache images with the step's new rows put in (plain indexing)."""
    bs = case.cfg.block_size
    kc, vc = case.k_cache.copy(), case.v_cache.copy()
    s = case.slot_mapping
    kc[s // bs, :, s % bs, :] = case.k_new
    vc[s // bs, :, s % bs, :] = case.v_new
    return kc, vc


def _decode_case(dtype, seed=71, slopes=True):
    cfg = W.small_config(name="win", dtype=dtype, batch=4, num_heads=8, num_kv_heads=2, head_dim=16,
                         block_size=4, num_blocks=96, ctx_lo=1, ctx_hi=61, seed=seed)
    case = W.make_case(cfg)
    return case, (case.slopes if slopes else None)


def _prefill_case(dtype, seed=73):
    cfg = W.small_config(name="winpf", kind="prefill", dtype=dtype, batch=3, num_heads=6, num_kv_heads=2,
                         head_dim=16, block_size=4, num_blocks=96, ctx_lo=5, ctx_hi=45, q_len=9, seed=seed)
    return W.make_case(cfg)


def _sequence_rows(case, kc, vc, b):
    """[L, Hkv, D] K and V rows of sequence b in logical order (numpy indexing through the table)."""
    bs = case.cfg.block_size
    j = np.arange(int(case.context_lens[b]))
    blk = case.block_tables[b, j // bs].astype(np.int64)
    return kc[blk, :, j % bs, :], vc[blk, :, j % bs, :]


def check_wide_window_is_full_attention(lib=None):
    """W >= context (and W <= 0) must give what the pinned full-context oracle gives."""
    for dtype in (W.F16, W.BF16):
        case, sl = _decode_case(dtype)
        kc, vc = _filled(case)
        ref = O.paged_attention(case.q, kc, vc, case.block_tables, case.context_lens, sl, case.scale, dtype)
        for window in (int(case.context_lens.max()), 10 ** 6, 0, -3):
            got = O.paged_attention_window(case.q, kc, vc, case.block_tables, case.context_lens, sl, case.scale,
                                           window, dtype, lib=lib)
            np.testing.assert_allclose(got, ref, rtol=1e-13, atol=1e-13)
        pf = _prefill_case(dtype)
        kc, vc = _filled(pf)
        ref = O.paged_prefill(pf.q, kc, vc, pf.block_tables, pf.context_lens, pf.cu_q_lens, pf.slopes, pf.scale,
                              dtype)
        for window in (int(pf.context_lens.max()), 0):
            got = O.paged_prefill_window(pf.q, kc, vc, pf.block_tables, pf.context_lens, pf.cu_q_lens, pf.slopes,
                                         pf.scale, window, dtype, lib=lib)
            np.testing.assert_allclose(got, ref, rtol=1e-13, atol=1e-13)


def _full_oracle_on_tokens(q_row, k_rows, v_rows, slopes, scale, dtype, Hq):
    """The pinned full-context decode oracle on a one-sequence cache that holds exactly the given
    token rows ([n, Hkv, D]) in identity block order."""
    n, Hkv, D = k_rows.shape
    bs = 4
    nb = (n + bs - 1) // bs
    kc = np.zeros((nb, Hkv, bs, D), np.uint16)
    vc = np.zeros((nb, Hkv, bs, D), np.uint16)
    j = np.arange(n)
    kc[j // bs, :, j % bs, :] = k_rows
    vc[j // bs, :, j % bs, :] = v_rows
    table = np.arange(nb, dtype=np.int32)[None, :]
    return O.paged_attention(q_row[None], kc, vc, table, np.array([n], np.int32), slopes, scale, dtype)[0]


def check_window_equals_full_attention_over_the_window_tokens(lib=None):
    """A windowed row == the pinned oracle run on a cache that holds only the last W tokens up to
    the query's position: the ALiBi term depends on j - pos alone, so it does not see the shift."""
    for dtype, window in ((W.BF16, 7), (W.F16, 16), (W.BF16, 1), (W.F16, 3)):
        case, sl = _decode_case(dtype, seed=75 + window)
        kc, vc = _filled(case)
        got = O.paged_attention_window(case.q, kc, vc, case.block_tables, case.context_lens, sl, case.scale,
                                       window, dtype, lib=lib)
        for b in range(case.cfg.batch):
            L = int(case.context_lens[b])
            ks, vs = _sequence_rows(case, kc, vc, b)
            lo = max(0, L - window)
            ref = _full_oracle_on_tokens(case.q[b], ks[lo:L], vs[lo:L], sl, case.scale, dtype, case.cfg.num_heads)
            np.testing.assert_allclose(got[b], ref, rtol=1e-12, atol=1e-13)
        pf = _prefill_case(dtype, seed=90 + window)
        kc, vc = _filled(pf)
        got = O.paged_prefill_window(pf.q, kc, vc, pf.block_tables, pf.context_lens, pf.cu_q_lens, pf.slopes,
                                     pf.scale, window, dtype, lib=lib)
        for b in range(pf.cfg.batch):
            L, n_b = int(pf.context_lens[b]), int(pf.q_lens[b])
            ks, vs = _sequence_rows(pf, kc, vc, b)
            for i in range(n_b):
                pos = L - n_b + i
                lo = max(0, pos + 1 - window)
                t = int(pf.cu_q_lens[b]) + i
                ref = _full_oracle_on_tokens(pf.q[t], ks[lo:pos + 1], vs[lo:pos + 1], pf.slopes, pf.scale, dtype,
                                             pf.cfg.num_heads)
                np.testing.assert_allclose(got[t], ref, rtol=1e-12, atol=1e-13)


def check_window_of_one_returns_own_value_row(lib=None):
    """W = 1: the softmax has one term, the output is the query token's own V row, exactly."""
    case, sl = _decode_case(W.F16, seed=77)
    kc, vc = _filled(case)
    got = O.paged_attention_window(case.q, kc, vc, case.block_tables, case.context_lens, sl, case.scale, 1,
                                   W.F16, lib=lib)
    for b in range(case.cfg.batch):
        _, vs = _sequence_rows(case, kc, vc, b)
        own = W.from_bits(vs[-1], W.F16).astype(np.float64)        # [Hkv, D]
        for h in range(case.cfg.num_heads):
            assert np.array_equal(got[b, h], own[h // 4])


def check_decoder_on_every_two_byte_pattern(lib=None):
    """All 65 536 fp16 and bf16 patterns (subnormals, infinities, NaNs) as the V row of a one-token
    context read with W = 1: the single weight is exactly 1, so the output is the decoder's value of
    each pattern, compared with numpy's own decoding."""
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    for dtype in (W.F16, W.BF16):
        want = W.from_bits(bits, dtype)
        D = 65536
        kc = np.zeros((1, 1, 1, D), np.uint16)
        vc = bits.reshape(1, 1, 1, D).copy()
        q = np.zeros((1, 1, D), np.uint16)
        out = O.paged_attention_window(q, kc, vc, np.zeros((1, 1), np.int32), np.ones(1, np.int32),
                                       np.ones(1, np.float32), 1.0, 1, dtype, lib=lib)[0, 0]
        fin = np.isfinite(want)
        assert np.array_equal(out[fin], want[fin]), f"{dtype} decoding"
        inf = np.isinf(want)
        assert np.array_equal(out[inf], want[inf]), f"{dtype} infinities"
        assert np.all(np.isnan(out[np.isnan(want)])), f"{dtype} NaN patterns"


def check_against_dense_mask_matrix(lib=None):
    """Dense formulation with library pieces: scores = Q K^T, bias matrix, a banded 0 / -inf mask
    built with numpy's triangle routines, scipy's softmax, weights @ V."""
    for dtype, window, with_slopes in ((W.BF16, 5, True), (W.F16, 12, False), (W.F16, 2, True)):
        pf = _prefill_case(dtype, seed=120 + window)
        kc, vc = _filled(pf)
        sl = pf.slopes if with_slopes else None
        got = O.paged_prefill_window(pf.q, kc, vc, pf.block_tables, pf.context_lens, pf.cu_q_lens, sl, pf.scale,
                                     window, dtype, lib=lib)
        G = pf.cfg.num_heads // pf.cfg.num_kv_heads
        for b in range(pf.cfg.batch):
            L, n_b = int(pf.context_lens[b]), int(pf.q_lens[b])
            ks, vs = _sequence_rows(pf, kc, vc, b)
            K = W.from_bits(ks, dtype).astype(np.float64)          # [L, Hkv, D]
            V = W.from_bits(vs, dtype).astype(np.float64)
            t0 = int(pf.cu_q_lens[b])
            Q = W.from_bits(pf.q[t0:t0 + n_b], dtype).astype(np.float64)   # [n_b, Hq, D]
            # row i of the L x L band matrix is position i; the new tokens are its last n_b rows
            ones = np.ones((L, L))
            band = np.tril(ones) * np.triu(ones, -(window - 1))
            mask = np.where(band[L - n_b:] > 0, 0.0, -np.inf)      # [n_b, L]
            rel = np.arange(L)[None, :] - np.arange(L - n_b, L)[:, None]   # j - pos
            for h in range(pf.cfg.num_heads):
                scores = float(pf.scale) * Q[:, h] @ K[:, h // G].T
                if sl is not None:
                    scores = scores + float(sl[h]) * rel
                wts = scipy.special.softmax(scores + mask, axis=1)
                np.testing.assert_allclose(got[t0:t0 + n_b, h], wts @ V[:, h // G], rtol=1e-11, atol=1e-12)
    # decode is the last row of the same matrix
    case, sl = _decode_case(W.BF16, seed=131)
    kc, vc = _filled(case)
    window = 9
    got = O.paged_attention_window(case.q, kc, vc, case.block_tables, case.context_lens, sl, case.scale, window,
                                   W.BF16, lib=lib)
    for b in range(case.cfg.batch):
        L = int(case.context_lens[b])
        ks, vs = _sequence_rows(case, kc, vc, b)
        K = W.from_bits(ks, W.BF16).astype(np.float64)
        V = W.from_bits(vs, W.BF16).astype(np.float64)
        ones = np.ones((L, L))
        mask = np.where((np.tril(ones) * np.triu(ones, -(window - 1)))[-1] > 0, 0.0, -np.inf)
        for h in range(case.cfg.num_heads):
            qv = W.from_bits(case.q[b, h], W.BF16).astype(np.float64)
            scores = float(case.scale) * K[:, h // 4] @ qv + float(sl[h]) * (np.arange(L) - (L - 1)) + mask
            np.testing.assert_allclose(got[b, h], scipy.special.softmax(scores) @ V[:, h // 4], rtol=1e-11,
                                       atol=1e-12)


def check_row_lists_pick_the_same_rows(lib=None):
    pf = _prefill_case(W.BF16, seed=140)
    kc, vc = _filled(pf)
    full = O.paged_prefill_window(pf.q, kc, vc, pf.block_tables, pf.context_lens, pf.cu_q_lens, pf.slopes, pf.scale,
                                  6, W.BF16, lib=lib)
    rows = [(0, 0), (5, 3), (pf.num_tokens - 1, 5), (7, 1)]
    sub = O.paged_prefill_window(pf.q, kc, vc, pf.block_tables, pf.context_lens, pf.cu_q_lens, pf.slopes, pf.scale,
                                 6, W.BF16, rows=rows, lib=lib)
    assert np.array_equal(sub, np.stack([full[t, h] for t, h in rows]))
    case, sl = _decode_case(W.F16, seed=141)
    kc, vc = _filled(case)
    full = O.paged_attention_window(case.q, kc, vc, case.block_tables, case.context_lens, sl, case.scale, 6, W.F16,
                                    lib=lib)
    rows = [(3, 7), (0, 0), (2, 4)]
    sub = O.paged_attention_window(case.q, kc, vc, case.block_tables, case.context_lens, sl, case.scale, 6, W.F16,
                                   rows=rows, lib=lib)
    assert np.array_equal(sub, np.stack([full[b, h] for b, h in rows]))


ALL_CHECKS = [
    check_wide_window_is_full_attention,
    check_window_equals_full_attention_over_the_window_tokens,
    check_window_of_one_returns_own_value_row,
    check_decoder_on_every_two_byte_pattern,
    check_against_dense_mask_matrix,
    check_row_lists_pick_the_same_rows,
]
