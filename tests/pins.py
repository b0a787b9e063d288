"""Pins for the CPU oracle: checks against things other than the oracle itself.

Every check takes ``lib`` (a loaded oracle shared library, or None for the committed one)
so that the same checks can be pointed at a deliberately broken build of the oracle
(tests/test_oracle_mutants.py) to show that a plausible mistake fails at least one of them.

What fixes the expected values:
  * brute force: dense scores with explicitly repeated K/V and an explicit bias matrix (numpy);
  * a library attention routine in fp64 (torch scaled_dot_product_attention with an additive
    mask and grouped heads) on the un-paged tensors;
  * closed forms: geometric ALiBi weights for q = 0, mean of V, constants, one-hot limits,
    a two-key case worked by hand;
  * identities the paper's definitions imply (eq. (2)-(4), Section II, Section III-A).
"""
from __future__ import annotations

import numpy as np

import oracle as O
import workloads as W


# ---------------------------------------------------------------- helpers (own index arithmetic)
def filled(case: W.Case, lib=None):
    """Cache image after the step's cache write (oracle's own write)."""
    kc, vc = case.k_cache.copy(), case.v_cache.copy()
    O.reshape_and_cache(case.k_new, case.v_new, kc, vc, case.slot_mapping, lib=lib)
    return kc, vc


def numpy_cache_write(case: W.Case):
    """The same write, stated with numpy fancy indexing instead of loops."""
    kc, vc = case.k_cache.copy(), case.v_cache.copy()
    bs = case.cfg.block_size
    keep = case.slot_mapping >= 0
    blk = case.slot_mapping[keep] // bs
    row = case.slot_mapping[keep] % bs
    kc[blk, :, row, :] = case.k_new[keep]
    vc[blk, :, row, :] = case.v_new[keep]
    return kc, vc


def unpage(case: W.Case, cache: np.ndarray, b: int, n: int) -> np.ndarray:
    """Tokens 0..n-1 of sequence b as a dense float64 [n, Hkv, D] array."""
    bs = case.cfg.block_size
    j = np.arange(n)
    blocks = case.block_tables[b, j // bs]
    return W.from_bits(cache[blocks, :, j % bs, :], case.dtype)


def dense_attention(qf, kf, vf, slopes, scale, pos_q):
    """Brute force for one sequence: qf [R, Hq, D] rows at positions pos_q [R];
    kf, vf [n, Hkv, D].  Scores are materialised as [Hq, R, n] with K/V repeated per group."""
    R, Hq, D = qf.shape
    n, Hkv, _ = kf.shape
    G = Hq // Hkv
    k_rep = np.repeat(kf, G, axis=1)          # [n, Hq, D]
    v_rep = np.repeat(vf, G, axis=1)
    s = np.einsum("rhd,nhd->hrn", qf, k_rep) * np.float64(scale)
    j = np.arange(n)[None, None, :]
    rel = j - np.asarray(pos_q)[None, :, None]
    s = s + np.asarray(slopes, dtype=np.float64)[:, None, None] * rel
    s = np.where(rel > 0, -np.inf, s)         # keys after the query do not exist for it
    s = s - s.max(axis=-1, keepdims=True)
    p = np.exp(s)
    p = p / p.sum(axis=-1, keepdims=True)
    return np.einsum("hrn,nhd->rhd", p, v_rep)


def run_decode(case, kc, vc, lib=None, slopes="case", rows=None):
    sl = case.slopes if isinstance(slopes, str) else slopes
    return O.paged_attention(case.q, kc, vc, case.block_tables, case.context_lens, sl,
                             case.scale, case.dtype, rows=rows, lib=lib)


def run_prefill(case, kc, vc, lib=None, rows=None):
    return O.paged_prefill(case.q, kc, vc, case.block_tables, case.context_lens, case.cu_q_lens,
                           case.slopes, case.scale, case.dtype, rows=rows, lib=lib)


TINY = [
    dict(dtype=W.F16, batch=2, num_heads=4, num_kv_heads=2, head_dim=8, block_size=4, ctx_hi=40),
    dict(dtype=W.BF16, batch=2, num_heads=6, num_kv_heads=3, head_dim=4, block_size=2, ctx_hi=23),
    dict(dtype=W.F16, batch=1, num_heads=8, num_kv_heads=1, head_dim=8, block_size=4, ctx_hi=17),
    dict(dtype=W.BF16, batch=2, num_heads=3, num_kv_heads=3, head_dim=8, block_size=4, ctx_hi=9),
    dict(dtype=W.F16, batch=3, num_heads=8, num_kv_heads=2, head_dim=6, block_size=3, ctx_hi=31),
]


# ---------------------------------------------------------------- checks
def check_widening(lib=None):
    """fp16 / bf16 decoding: a context of one token returns V exactly, for every finite
    bit pattern (eq. (4) with a single key gives weight 1)."""
    for dtype in (W.F16, W.BF16):
        bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
        want = W.from_bits(bits, dtype)           # numpy's own decoding
        D = 65536
        kc = np.zeros((1, 1, 1, D), dtype=np.uint16)
        vc = bits.reshape(1, 1, 1, D).copy()
        q = np.zeros((1, 1, D), dtype=np.uint16)
        out = O.paged_attention(q, kc, vc, np.zeros((1, 1), np.int32), np.ones(1, np.int32),
                                np.ones(1, np.float32), 1.0, dtype, lib=lib)[0, 0]
        fin = np.isfinite(want)
        assert np.array_equal(out[fin], want[fin]), f"{dtype} widening"
        assert np.all(np.isnan(out[np.isnan(want)]))


def check_brute_force(lib=None):
    for i, kw in enumerate(TINY):
        cfg = W.small_config(name=f"tiny{i}", seed=100 + i, **kw)
        case = W.make_case(cfg)
        kc, vc = numpy_cache_write(case)
        got = run_decode(case, kc, vc, lib)
        for b in range(cfg.batch):
            L = int(case.context_lens[b])
            want = dense_attention(W.from_bits(case.q[b:b + 1], case.dtype), unpage(case, kc, b, L),
                                   unpage(case, vc, b, L), case.slopes, case.scale, [L - 1])[0]
            np.testing.assert_allclose(got[b], want, rtol=0, atol=1e-12)


def check_library_sdpa(lib=None):
    """Un-paged tensors through torch's fp64 attention with an additive ALiBi mask and
    grouped heads must give the oracle's numbers."""
    import torch
    import torch.nn.functional as F
    for i, (dtype, Hq, Hkv, D, bs) in enumerate([(W.F16, 8, 2, 64, 16), (W.BF16, 12, 4, 32, 8),
                                                 (W.F16, 4, 4, 16, 16), (W.BF16, 8, 1, 64, 32)]):
        cfg = W.small_config(name=f"sdpa{i}", dtype=dtype, batch=3, num_heads=Hq, num_kv_heads=Hkv,
                             head_dim=D, block_size=bs, num_blocks=96, ctx_lo=1, ctx_hi=300,
                             seed=200 + i)
        case = W.make_case(cfg)
        kc, vc = numpy_cache_write(case)
        got = run_decode(case, kc, vc, lib)
        for b in range(cfg.batch):
            L = int(case.context_lens[b])
            qt = torch.from_numpy(W.from_bits(case.q[b], dtype))[None, :, None, :]        # [1,Hq,1,D]
            kt = torch.from_numpy(unpage(case, kc, b, L)).permute(1, 0, 2)[None]          # [1,Hkv,L,D]
            vt = torch.from_numpy(unpage(case, vc, b, L)).permute(1, 0, 2)[None]
            rel = torch.arange(L, dtype=torch.float64) - (L - 1)
            mask = (torch.from_numpy(case.slopes.astype(np.float64))[:, None] * rel[None, :])[None, :, None, :]
            want = F.scaled_dot_product_attention(qt, kt, vt, attn_mask=mask,
                                                  scale=float(case.scale), enable_gqa=True)
            np.testing.assert_allclose(got[b], want[0, :, 0, :].numpy(), rtol=0, atol=1e-11)


def check_zero_slopes_is_softmax_attention(lib=None):
    """With every slope 0 (or no slopes at all) eq. (3) has no bias left: plain softmax attention."""
    from scipy.special import softmax
    cfg = W.small_config(name="noslope", dtype=W.F16, batch=2, num_heads=4, num_kv_heads=2,
                         head_dim=16, block_size=8, ctx_hi=70, seed=7)
    case = W.make_case(cfg)
    kc, vc = numpy_cache_write(case)
    zero = np.zeros(cfg.num_heads, np.float32)
    got0 = run_decode(case, kc, vc, lib, slopes=zero)
    gotN = run_decode(case, kc, vc, lib, slopes=None)
    assert np.array_equal(got0, gotN)
    for b in range(cfg.batch):
        L = int(case.context_lens[b])
        K, V = unpage(case, kc, b, L), unpage(case, vc, b, L)
        qf = W.from_bits(case.q[b], case.dtype)
        for h in range(cfg.num_heads):
            g = h // (cfg.num_heads // cfg.num_kv_heads)
            w = softmax(K[:, g, :] @ qf[h] * np.float64(case.scale))
            np.testing.assert_allclose(got0[b, h], w @ V[:, g, :], rtol=0, atol=1e-12)


def check_single_token_returns_v(lib=None):
    cfg = W.small_config(name="L1", dtype=W.BF16, batch=3, num_heads=8, num_kv_heads=2,
                         head_dim=16, block_size=4, ctx_lo=1, ctx_hi=1, seed=11)
    case = W.make_case(cfg)
    kc, vc = numpy_cache_write(case)
    got = run_decode(case, kc, vc, lib)
    for b in range(cfg.batch):
        V = unpage(case, vc, b, 1)[0]                      # [Hkv, D]
        for h in range(cfg.num_heads):
            assert np.array_equal(got[b, h], V[h // 4])


def _const_case(L, dtype, slopes, Hq=2, Hkv=1, D=4, bs=16, seed=5):
    cfg = W.small_config(name="closed", dtype=dtype, batch=1, num_heads=Hq, num_kv_heads=Hkv,
                         head_dim=D, block_size=bs, num_blocks=(L + bs - 1) // bs + 3,
                         ctx_lo=L, ctx_hi=L, seed=seed)
    case = W.make_case(cfg, slopes=np.asarray(slopes, np.float32))
    kc, vc = numpy_cache_write(case)
    return cfg, case, kc, vc


def check_closed_form_geometric(lib=None):
    """q = 0 leaves only the ALiBi bias: w_j = r^(L-1-j) (1-r) / (1-r^L) with r = e^-slope
    (Section II: a bias linear in the relative position; recent keys weigh more)."""
    for L, dtype in [(7, W.F16), (300, W.BF16), (4096, W.F16), (32768, W.F16)]:
        slopes = [0.5, 2.0 ** -7]
        cfg, case, kc, vc = _const_case(L, dtype, slopes)
        case.q[:] = 0
        got = run_decode(case, kc, vc, lib)
        V = unpage(case, vc, 0, L)[:, 0, :]
        i = (L - 1 - np.arange(L)).astype(np.float64)
        for h, m in enumerate(np.asarray(slopes, np.float32).astype(np.float64)):
            r = np.exp(-m)
            w = r ** i * (1 - r) / (1 - r ** L)
            assert abs(w.sum() - 1) < 1e-12
            np.testing.assert_allclose(got[0, h], w @ V, rtol=0, atol=1e-11)


def check_closed_form_means_and_constants(lib=None):
    # slopes 0 and K = 0  ->  plain mean of V
    cfg, case, kc, vc = _const_case(37, W.F16, [0.0, 0.0])
    used = case.block_tables[0, : (37 + 15) // 16]
    kz = kc.copy()
    kz[used] = 0
    got = run_decode(case, kz, vc, lib)
    V = unpage(case, vc, 0, 37)[:, 0, :]
    np.testing.assert_allclose(got[0, 0], V.mean(axis=0), rtol=0, atol=1e-13)
    # V constant over tokens  ->  that constant, whatever the scores are
    cfg, case, kc, vc = _const_case(53, W.BF16, [0.3, 0.01])
    const = W.to_bits(np.array([1.5, -2.0, 0.25, 3.0], np.float32), W.BF16)
    vconst = vc.copy()
    vconst[case.block_tables[0, : (53 + 15) // 16]] = const
    got = run_decode(case, kc, vconst, lib)
    np.testing.assert_allclose(got[0], np.tile([1.5, -2.0, 0.25, 3.0], (2, 1)), rtol=0, atol=1e-14)


def check_one_hot_limits(lib=None):
    """A huge positive slope leaves only the newest key, a huge negative one only key 0:
    fixes the sign and the reference point of the relative position."""
    for L in (1, 5, 16, 17, 100):
        cfg, case, kc, vc = _const_case(L, W.F16, [200.0, -200.0], bs=16)
        kz = kc.copy()
        kz[case.block_tables[0, : (L + 15) // 16]] = 0
        got = run_decode(case, kz, vc, lib)
        V = unpage(case, vc, 0, L)[:, 0, :]
        assert np.array_equal(got[0, 0], V[L - 1]), L
        assert np.array_equal(got[0, 1], V[0]), L


def check_two_key_hand_case(lib=None):
    """Worked by hand from eq. (3)-(4): q = 1, k0 = 4, k1 = 2, scale = 1/2, slope = 1, L = 2.
    s0 = 0.5*4 + 1*(0-1) = 1, s1 = 0.5*2 + 0 = 1, so both weights are 1/2 and
    out = (v0 + v1)/2 = (3 + 5)/2 = 4.  (A scaled bias would give s0 = 1.5, s1 = 1.)
    Second head, slope ln 2 (fp32): s0 = 2 - ln 2, s1 = 1, w0 = e/(e+2)."""
    for dtype in (W.F16, W.BF16):
        one = lambda x: W.to_bits(np.array([x], np.float32), dtype)
        kc = np.zeros((1, 1, 2, 1), np.uint16)
        vc = np.zeros((1, 1, 2, 1), np.uint16)
        kc[0, 0, 0], kc[0, 0, 1] = one(4.0), one(2.0)
        vc[0, 0, 0], vc[0, 0, 1] = one(3.0), one(5.0)
        q = np.stack([one(1.0), one(1.0)])[None]            # [1, 2, 1]
        ln2 = np.float32(np.log(2.0))
        out = O.paged_attention(q, kc, vc, np.zeros((1, 1), np.int32), np.array([2], np.int32),
                                np.array([1.0, ln2], np.float32), 0.5, dtype, lib=lib)
        assert abs(out[0, 0, 0] - 4.0) < 1e-15
        w0 = np.e / (np.e + 2.0)
        assert abs(out[0, 1, 0] - (w0 * 3.0 + (1 - w0) * 5.0)) < 1e-7


def check_gqa_equals_mha_on_repeated_kv(lib=None):
    """Section II (a group shares one key-value pair): sharing one K/V per group is the same as every head of
    the group holding its own copy."""
    cfg = W.small_config(name="gqa", dtype=W.F16, batch=2, num_heads=8, num_kv_heads=2,
                         head_dim=8, block_size=4, ctx_hi=33, seed=21)
    case = W.make_case(cfg)
    kc, vc = numpy_cache_write(case)
    got = run_decode(case, kc, vc, lib)
    k_rep, v_rep = np.repeat(kc, 4, axis=1), np.repeat(vc, 4, axis=1)   # Hkv = Hq = 8
    mha = O.paged_attention(case.q, np.ascontiguousarray(k_rep), np.ascontiguousarray(v_rep),
                            case.block_tables, case.context_lens, case.slopes, case.scale,
                            case.dtype, lib=lib)
    assert np.array_equal(got, mha)
    # and MHA itself is per-head single-head attention on un-paged tensors
    for b in range(cfg.batch):
        L = int(case.context_lens[b])
        K, V = W.from_bits(k_rep, case.dtype), W.from_bits(v_rep, case.dtype)
        j = np.arange(L)
        blk = case.block_tables[b, j // 4]
        for h in range(8):
            s = K[blk, h, j % 4, :] @ W.from_bits(case.q[b, h], case.dtype) * np.float64(case.scale)
            s = s + np.float64(case.slopes[h]) * (j - (L - 1))
            p = np.exp(s - s.max())
            np.testing.assert_allclose(mha[b, h], (p / p.sum()) @ V[blk, h, j % 4, :], atol=1e-12, rtol=0)


def check_block_permutation_invariance(lib=None):
    cfg = W.small_config(name="perm", dtype=W.BF16, batch=3, num_heads=4, num_kv_heads=2,
                         head_dim=8, block_size=4, ctx_hi=45, seed=31)
    base = W.make_case(cfg)
    kc, vc = numpy_cache_write(base)
    ref = run_decode(base, kc, vc, lib)
    assert np.all(np.isfinite(ref))                       # NaN rows / blocks are never read
    for ps in (1, 2):
        other = W.make_case(cfg, perm_seed=ps)
        assert not np.array_equal(other.block_tables, base.block_tables)
        kc2, vc2 = numpy_cache_write(other)
        assert np.array_equal(run_decode(other, kc2, vc2, lib), ref)
    ident = W.make_case(cfg, identity_blocks=True)
    kc3, vc3 = numpy_cache_write(ident)
    assert np.array_equal(run_decode(ident, kc3, vc3, lib), ref)


def check_partition_invariance(lib=None):
    """Section III-A: per-partition results carried forward and combined equal the
    whole-context result, for any partition size including a ragged last partition."""
    cfg = W.small_config(name="part", dtype=W.F16, batch=3, num_heads=4, num_kv_heads=2,
                         head_dim=8, block_size=4, num_blocks=80, ctx_lo=1, ctx_hi=90, seed=41)
    case = W.make_case(cfg)
    kc, vc = numpy_cache_write(case)
    ref = run_decode(case, kc, vc, lib)
    for P in (4, 8, 20, 64, 512):
        got = O.paged_attention_partitioned(case.q, kc, vc, case.block_tables, case.context_lens,
                                            case.slopes, case.scale, case.dtype, P, lib=lib)
        np.testing.assert_allclose(got, ref, rtol=0, atol=1e-12)
    # steep slopes: early partitions underflow to weight 0 and must not disturb the result
    steep = np.array([30.0, 0.5, 3.0, 0.0], np.float32)
    ref = run_decode(case, kc, vc, lib, slopes=steep)
    got = O.paged_attention_partitioned(case.q, kc, vc, case.block_tables, case.context_lens,
                                        steep, case.scale, case.dtype, 8, lib=lib)
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-12)


def check_prefill(lib=None):
    """Prompt branch of Alg. 1: causal + ALiBi.  Row i equals (a) brute force with an explicit
    mask, (b) a decode call whose context is cut after that row's own position."""
    for i, (dtype, q_len) in enumerate([(W.F16, 5), (W.BF16, 9)]):
        cfg = W.small_config(name=f"pf{i}", kind="prefill", dtype=dtype, batch=3, num_heads=4,
                             num_kv_heads=2, head_dim=8, block_size=4, num_blocks=64, ctx_lo=3,
                             ctx_hi=40, q_len=q_len, seed=50 + i)
        case = W.make_case(cfg)
        kc, vc = numpy_cache_write(case)
        got = run_prefill(case, kc, vc, lib)
        assert got.shape[0] == int(case.cu_q_lens[-1])
        for b in range(cfg.batch):
            L, n = int(case.context_lens[b]), int(case.q_lens[b])
            t0 = int(case.cu_q_lens[b])
            pos = np.arange(L - n, L)
            want = dense_attention(W.from_bits(case.q[t0:t0 + n], dtype), unpage(case, kc, b, L),
                                   unpage(case, vc, b, L), case.slopes, case.scale, pos)
            np.testing.assert_allclose(got[t0:t0 + n], want, rtol=0, atol=1e-12)
            for r in range(n):                             # (b) stacked decodes
                cl = case.context_lens.copy()
                cl[b] = pos[r] + 1
                qd = np.zeros((cfg.batch, cfg.num_heads, cfg.head_dim), np.uint16)
                qd[b] = case.q[t0 + r]
                dec = O.paged_attention(qd, kc, vc, case.block_tables, cl, case.slopes, case.scale,
                                        dtype, lib=lib)
                assert np.array_equal(dec[b], got[t0 + r])
        # sampled-rows entry point agrees with the full one
        T = got.shape[0]
        rows = [(0, 0), (T - 1, 3), (T // 2, 1)]
        sub = run_prefill(case, kc, vc, lib, rows=rows)
        for r, (t, h) in enumerate(rows):
            assert np.array_equal(sub[r], got[t, h])


def check_prefill_library_sdpa(lib=None):
    import torch
    import torch.nn.functional as F
    cfg = W.small_config(name="pfsdpa", kind="prefill", dtype=W.BF16, batch=2, num_heads=8,
                         num_kv_heads=2, head_dim=32, block_size=16, num_blocks=40, ctx_lo=70,
                         ctx_hi=200, q_len=33, seed=61)
    case = W.make_case(cfg)
    kc, vc = numpy_cache_write(case)
    got = run_prefill(case, kc, vc, lib)
    for b in range(cfg.batch):
        L, n, t0 = int(case.context_lens[b]), int(case.q_lens[b]), int(case.cu_q_lens[b])
        qt = torch.from_numpy(W.from_bits(case.q[t0:t0 + n], case.dtype)).permute(1, 0, 2)[None]
        kt = torch.from_numpy(unpage(case, kc, b, L)).permute(1, 0, 2)[None]
        vt = torch.from_numpy(unpage(case, vc, b, L)).permute(1, 0, 2)[None]
        pos = torch.arange(L - n, L, dtype=torch.float64)
        rel = torch.arange(L, dtype=torch.float64)[None, :] - pos[:, None]          # [n, L]
        mask = torch.from_numpy(case.slopes.astype(np.float64))[:, None, None] * rel[None]
        mask = mask.masked_fill(rel[None] > 0, float("-inf"))[None]
        want = F.scaled_dot_product_attention(qt, kt, vt, attn_mask=mask, scale=float(case.scale),
                                              enable_gqa=True)[0].permute(1, 0, 2).numpy()
        np.testing.assert_allclose(got[t0:t0 + n], want, rtol=0, atol=1e-11)


def check_rows_entry_point(lib=None):
    cfg = W.small_config(name="rows", dtype=W.F16, batch=4, num_heads=4, num_kv_heads=1,
                         head_dim=8, block_size=4, ctx_hi=30, seed=71)
    case = W.make_case(cfg)
    kc, vc = numpy_cache_write(case)
    full = run_decode(case, kc, vc, lib)
    rows = [(3, 1), (0, 0), (2, 3)]
    sub = run_decode(case, kc, vc, lib, rows=rows)
    for r, (b, h) in enumerate(rows):
        assert np.array_equal(sub[r], full[b, h])


def check_empty_context(lib=None):
    cfg = W.small_config(name="empty", dtype=W.F16, batch=3, num_heads=2, num_kv_heads=1,
                         head_dim=8, block_size=4, ctx_lo=1, ctx_hi=9, seed=81)
    case = W.make_case(cfg, context_lens=np.array([5, 0, 9], np.int32))
    kc, vc = numpy_cache_write(case)
    qd = np.zeros((3, 2, 8), np.uint16)
    qd[0], qd[2] = case.q[0], case.q[1]
    out = O.paged_attention(qd, kc, vc, case.block_tables, case.context_lens, case.slopes,
                            case.scale, case.dtype, lib=lib)
    assert np.all(out[1] == 0) and np.all(np.isfinite(out))


def check_cache_write(lib=None):
    """eq. (2) / Alg. 1 cache store: bits land at [slot // bs, head, slot % bs, :], nothing
    else changes, negative slots are skipped, and appending token by token equals one bulk write."""
    cfg = W.small_config(name="cw", kind="prefill", dtype=W.BF16, batch=3, num_heads=4,
                         num_kv_heads=2, head_dim=8, block_size=4, num_blocks=40, ctx_lo=5,
                         ctx_hi=30, q_len=5, seed=91)
    case = W.make_case(cfg)
    kc, vc = filled(case, lib)
    kn, vn = numpy_cache_write(case)
    assert np.array_equal(kc, kn) and np.array_equal(vc, vn)
    # written rows hold the source bits, by direct element-wise reading of the layout
    for t in range(case.num_tokens):
        s = int(case.slot_mapping[t])
        for g in range(cfg.num_kv_heads):
            assert np.array_equal(kc[s // 4, g, s % 4], case.k_new[t, g])
            assert np.array_equal(vc[s // 4, g, s % 4], case.v_new[t, g])
    changed = (kc != case.k_cache).any(axis=(1, 3))       # [NB, bs]
    assert changed.sum() <= case.num_tokens
    # padding tokens
    slots = case.slot_mapping.copy()
    slots[::2] = -1
    k2, v2 = case.k_cache.copy(), case.v_cache.copy()
    O.reshape_and_cache(case.k_new, case.v_new, k2, v2, slots, lib=lib)
    for t in range(case.num_tokens):
        s = int(case.slot_mapping[t])
        if t % 2 == 0:
            assert np.array_equal(k2[s // 4, :, s % 4], case.k_cache[s // 4, :, s % 4])
        else:
            assert np.array_equal(v2[s // 4, :, s % 4], case.v_new[t])
    # token-by-token append == bulk
    k3, v3 = case.k_cache.copy(), case.v_cache.copy()
    for t in range(case.num_tokens):
        O.reshape_and_cache(case.k_new[t:t + 1], case.v_new[t:t + 1], k3, v3,
                            case.slot_mapping[t:t + 1], lib=lib)
    assert np.array_equal(k3, kc) and np.array_equal(v3, vc)


ALL_CHECKS = [
    check_widening, check_brute_force, check_library_sdpa, check_zero_slopes_is_softmax_attention,
    check_single_token_returns_v, check_closed_form_geometric,
    check_closed_form_means_and_constants, check_one_hot_limits, check_two_key_hand_case,
    check_gqa_equals_mha_on_repeated_kv, check_block_permutation_invariance,
    check_partition_invariance, check_prefill, check_prefill_library_sdpa,
    check_rows_entry_point, check_empty_context, check_cache_write,
]
