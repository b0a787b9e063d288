"""Pins for the oracle's 8-bit (E4M3) KV-cache clauses: every check compares the oracle with
something that is not the oracle - a library's float8 type, exact rational arithmetic, numpy
indexing, or the already pinned 2-byte oracle.  Each takes the library to test (None = the
committed oracle), so that the planted-mistake test can aim them at mutants."""
from fractions import Fraction

import numpy as np
import torch

import oracle as O
import workloads as W


def _library_values() -> np.ndarray:
    """The 256 code values according to torch's float8_e4m3fn (fp64, NaN where NaN)."""
    return torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float64).numpy()


def check_values_match_library_type(lib=None):
    got, want = O.e4m3_values(lib), _library_values()
    assert np.array_equal(np.isnan(got), np.isnan(want))
    ok = ~np.isnan(want)
    assert np.array_equal(got[ok], want[ok])
    assert np.array_equal(np.signbit(got[ok]), np.signbit(want[ok]))
    # what the format's definition fixes: two NaN codes, largest finite 448, smallest step 2^-9
    assert np.isnan(got[0x7F]) and np.isnan(got[0xFF]) and np.sum(np.isnan(got)) == 2
    assert got[0x7E] == 448.0 and got[0x01] == 2.0 ** -9 and got[0x08] == 2.0 ** -6 and got[0x38] == 1.0


def check_nearest_on_representable_values_and_midpoints(lib=None):
    vals = _library_values()
    pos = vals[:0x7F]                                   # 0 .. 448, increasing with the code
    assert np.all(np.diff(pos) > 0)
    # every representable value is its own nearest code (both signs; -0 keeps its sign bit)
    codes = np.arange(0x7F, dtype=np.uint8)
    assert np.array_equal(O.e4m3_nearest(pos.astype(np.float32), lib), codes)
    assert np.array_equal(O.e4m3_nearest((-pos).astype(np.float32), lib), codes | 0x80)
    # midpoints between neighbours are float32 numbers; exact rational arithmetic says which
    # neighbour is nearer for the floats just below and above, and ties go to the even code
    for c in range(0x7E):
        lo, hi = Fraction(float(pos[c])), Fraction(float(pos[c + 1]))
        mid = (lo + hi) / 2
        m32 = np.float32(float(mid))
        assert Fraction(float(m32)) == mid
        below, above = np.nextafter(m32, np.float32(0)), np.nextafter(m32, np.float32(1e9))
        want = [c if c % 2 == 0 else c + 1, c, c + 1]
        got = O.e4m3_nearest(np.array([m32, below, above], np.float32), lib)
        assert list(got) == want, (c, list(got), want)
        gotn = O.e4m3_nearest(-np.array([m32, below, above], np.float32), lib)
        assert list(gotn) == [w | 0x80 for w in want]


def check_nearest_matches_library_in_range(lib=None):
    rng = np.random.default_rng(8)
    x = np.concatenate([rng.normal(size=200000).astype(np.float32) * s for s in (0.01, 1.0, 30.0, 150.0)])
    x = x[np.abs(x) <= 448.0]
    want = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(O.e4m3_nearest(x, lib), want)
    # every fp16 and every bf16 number in range (the cache-write inputs are such numbers)
    for view in (np.float16, None):
        bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
        v = bits.view(np.float16).astype(np.float32) if view else W.from_bits(bits, W.BF16).astype(np.float32)
        v = v[np.isfinite(v) & (np.abs(v) <= 448.0)]
        want = torch.from_numpy(v).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
        assert np.array_equal(O.e4m3_nearest(v, lib), want)


def check_nearest_saturates_and_orders(lib=None):
    big = np.array([448.0, 448.00003, 464.0, 465.0, 1e6, 3e38, np.inf], np.float32)
    assert np.all(O.e4m3_nearest(big, lib) == 0x7E)
    assert np.all(O.e4m3_nearest(-big, lib) == 0xFE)
    assert O.e4m3_nearest(np.array([np.nan], np.float32), lib)[0] == 0x7F
    tiny = np.array([0.0, 1e-30, 2.0 ** -11, 2.0 ** -10, 1.5 * 2.0 ** -9], np.float32)
    assert list(O.e4m3_nearest(tiny, lib)) == [0, 0, 0, 0, 2]          # 2^-10 ties to the even code 0
    # monotone: a larger input never gets a smaller value
    x = np.sort(np.random.default_rng(9).uniform(-500, 500, size=100000).astype(np.float32))
    v = _library_values()[O.e4m3_nearest(x, lib)]
    assert np.all(np.diff(v) >= 0)
    # and the error is at most half a step of the format around the result
    inr = np.abs(x) <= 448
    assert np.all(np.abs(v[inr] - x[inr]) <= np.maximum(np.abs(x[inr]) * 2.0 ** -4, 2.0 ** -10))


def _small_case(dtype, seed=31):
    cfg = W.small_config(name="e4m3", dtype=dtype, batch=3, num_heads=8, num_kv_heads=2, head_dim=16,
                         block_size=4, num_blocks=64, ctx_lo=1, ctx_hi=37, seed=seed)
    return W.make_case(cfg)


def _all_tokens(case):
    """The 2-byte K/V rows of every token of the batch with the slot of each (the generator's own
    indexing helper)."""
    return W.all_token_rows(case)


def quantised_cache(case, k_scale, v_scale, lib=None):
    """E4M3 cache image of the whole batch, written by the oracle's quantising cache write."""
    cfg = case.cfg
    k_all, v_all, slots = _all_tokens(case)
    shape = (cfg.num_blocks, cfg.num_kv_heads, cfg.block_size, cfg.head_dim)
    kc8 = np.full(shape, 0x7F, np.uint8)                 # untouched rows stay NaN codes
    vc8 = np.full(shape, 0x7F, np.uint8)
    O.reshape_and_cache_e4m3(k_all, v_all, kc8, vc8, slots, k_scale, v_scale, case.dtype, lib)
    return kc8, vc8, (k_all, v_all, slots)


def check_cache_write_against_library_cast(lib=None):
    for dtype in (W.F16, W.BF16):
        case = _small_case(dtype)
        cfg = case.cfg
        k_scale, v_scale = np.float32(0.037), np.float32(1.7)
        kc8, vc8, (k_all, v_all, slots) = quantised_cache(case, k_scale, v_scale, lib)
        for arr8, src, sc in ((kc8, k_all, k_scale), (vc8, v_all, v_scale)):
            x = W.from_bits(src, dtype).astype(np.float32) * (np.float32(1.0) / sc)      # fp32 product
            x = np.clip(x, -448, 448)
            want_codes = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
            want = np.full(arr8.shape, 0x7F, np.uint8)
            want[slots // cfg.block_size, :, slots % cfg.block_size, :] = want_codes
            assert np.array_equal(arr8, want)
        # padding slots are skipped, saturation happens in the product (tiny scale)
        kc8b = np.full_like(kc8, 0x7F)
        vc8b = np.full_like(vc8, 0x7F)
        slots2 = slots.copy()
        slots2[::2] = -1
        O.reshape_and_cache_e4m3(k_all, v_all, kc8b, vc8b, slots2, np.float32(1e-4), np.float32(1e-4), dtype, lib)
        skipped = slots[::2]
        assert np.all(kc8b[skipped // cfg.block_size, :, skipped % cfg.block_size, :] == 0x7F)
        kept = slots[1::2]
        got = kc8b[kept // cfg.block_size, :, kept % cfg.block_size, :]
        src = W.from_bits(k_all[1::2], dtype)
        assert np.all(got[src > 0.05] == 0x7E) and np.all(got[src < -0.05] == 0xFE)


def check_attention_reduces_to_two_byte_oracle(lib=None):
    """Every E4M3 value is exactly a bf16 (and fp16) number, so attention over the 8-bit cache must
    equal the 2-byte oracle (pinned separately) run on a cache that holds the dequantised values,
    with k_scale folded into the score scale and v_scale applied to the result."""
    vals = _library_values()
    for dtype in (W.F16, W.BF16):
        case = _small_case(dtype, seed=33)
        k_scale, v_scale = np.float32(0.25), np.float32(3.0)       # powers of two / small integers:
        kc8, vc8, _ = quantised_cache(case, k_scale, v_scale, lib)  # scale * k_scale stays exact in fp32
        got = O.paged_attention_e4m3(case.q, kc8, vc8, case.block_tables, case.context_lens, case.slopes,
                                     case.scale, k_scale, v_scale, dtype, lib=lib)
        deq = lambda c8: W.to_bits(np.nan_to_num(vals[c8], nan=0.0).astype(np.float32), dtype)
        assert np.array_equal(W.from_bits(deq(kc8), dtype)[kc8 != 0x7F], vals[kc8][kc8 != 0x7F])
        ref = O.paged_attention(case.q, deq(kc8), deq(vc8), case.block_tables, case.context_lens, case.slopes,
                                np.float32(case.scale * k_scale), dtype)
        np.testing.assert_allclose(got, ref * float(v_scale), rtol=1e-12, atol=1e-12)
        # rows entry point, and an empty context
        rows = [(2, 7), (0, 0), (1, 3)]
        sub = O.paged_attention_e4m3(case.q, kc8, vc8, case.block_tables, case.context_lens, case.slopes,
                                     case.scale, k_scale, v_scale, dtype, rows=rows, lib=lib)
        np.testing.assert_allclose(sub, np.stack([got[b, h] for b, h in rows]), rtol=0, atol=0)
        lens0 = case.context_lens.copy()
        lens0[1] = 0
        z = O.paged_attention_e4m3(case.q, kc8, vc8, case.block_tables, lens0, case.slopes, case.scale,
                                   k_scale, v_scale, dtype, lib=lib)
        assert not z[1].any()


def check_scales_enter_where_the_definition_says(lib=None):
    case = _small_case(W.BF16, seed=35)
    kc8, vc8, _ = quantised_cache(case, np.float32(0.5), np.float32(0.5), lib)
    run = lambda scale, ks, vs: O.paged_attention_e4m3(case.q, kc8, vc8, case.block_tables, case.context_lens,
                                                       case.slopes, np.float32(scale), np.float32(ks),
                                                       np.float32(vs), W.BF16, lib=lib)
    base = run(case.scale, 0.5, 0.5)
    np.testing.assert_allclose(run(case.scale, 0.5, 1.0), 2.0 * base, rtol=1e-13)          # v_scale: linear in the output
    np.testing.assert_allclose(run(case.scale * 2, 0.25, 0.5), base, rtol=1e-12)           # k_scale: multiplies the score scale
    assert np.max(np.abs(run(case.scale, 1.0, 0.5) - base)) > 1e-3                          # and it matters
    # one token: softmax weight 1, output = v_scale * value(code) exactly
    lens1 = np.ones_like(case.context_lens)
    one = run(case.scale, 0.5, 0.5) if False else O.paged_attention_e4m3(
        case.q, kc8, vc8, case.block_tables, lens1, case.slopes, case.scale, np.float32(0.5), np.float32(0.5),
        W.BF16, lib=lib)
    vals = _library_values()
    for b in range(case.cfg.batch):
        blk = case.block_tables[b, 0]
        for h in range(case.cfg.num_heads):
            assert np.array_equal(one[b, h], 0.5 * vals[vc8[blk, h // 4, 0, :]])


def check_prefill_reduces_to_two_byte_oracle_and_to_decodes(lib=None):
    """Prefill over the 8-bit cache: equals the 2-byte prefill oracle (pinned separately) on the
    dequantised cache, and every row equals a decode call whose context ends at that row."""
    vals = _library_values()
    cfg = W.small_config(name="e4m3pf", kind="prefill", dtype=W.BF16, batch=3, num_heads=8, num_kv_heads=2,
                         head_dim=16, block_size=4, num_blocks=64, ctx_lo=9, ctx_hi=37, q_len=7, seed=37)
    case = W.make_case(cfg)
    k_scale, v_scale = np.float32(0.25), np.float32(3.0)
    kc8, vc8, _ = quantised_cache(case, k_scale, v_scale, lib)
    got = O.paged_prefill_e4m3(case.q, kc8, vc8, case.block_tables, case.context_lens, case.cu_q_lens,
                               case.slopes, case.scale, k_scale, v_scale, W.BF16, lib=lib)
    deq = lambda c8: W.to_bits(np.nan_to_num(vals[c8], nan=0.0).astype(np.float32), W.BF16)
    ref = O.paged_prefill(case.q, deq(kc8), deq(vc8), case.block_tables, case.context_lens, case.cu_q_lens,
                          case.slopes, np.float32(case.scale * k_scale), W.BF16)
    np.testing.assert_allclose(got, ref * float(v_scale), rtol=1e-12, atol=1e-12)
    # row t of sequence b == decode of that query with the context cut after its own position
    for b in range(cfg.batch):
        n_b = int(case.q_lens[b])
        for i in (0, n_b // 2, n_b - 1):
            t = int(case.cu_q_lens[b]) + i
            lens = case.context_lens.copy()
            lens[b] = int(case.context_lens[b]) - n_b + i + 1
            qd = np.zeros((cfg.batch, 8, 16), np.uint16)
            qd[b] = case.q[t]
            dec = O.paged_attention_e4m3(qd, kc8, vc8, case.block_tables, lens, case.slopes, case.scale,
                                         k_scale, v_scale, W.BF16, lib=lib)
            np.testing.assert_allclose(got[t], dec[b], rtol=1e-13, atol=1e-13)
    rows = [(5, 3), (0, 0), (int(case.cu_q_lens[-1]) - 1, 7)]
    sub = O.paged_prefill_e4m3(case.q, kc8, vc8, case.block_tables, case.context_lens, case.cu_q_lens,
                               case.slopes, case.scale, k_scale, v_scale, W.BF16, rows=rows, lib=lib)
    np.testing.assert_allclose(sub, np.stack([got[t, h] for t, h in rows]), rtol=0, atol=0)


def check_per_head_scales_reduce_to_per_tensor_clauses(lib=None):
    """One scale pair per KV head: KV head by KV head, the cache write, the decode clause and the prefill
    clause must give what the per-tensor clauses (pinned above; always the built oracle's here) give
    with that head's pair - on the codes of that head and on the rows of the query heads that read
    it.  Three KV heads with very different scales, so that a scale taken from the wrong head, from
    the query-head index or from the other tensor shows."""
    k_scales = np.array([0.5, 0.03125, 2.0], np.float32)
    v_scales = np.array([1.5, 0.25, 0.0078125], np.float32)
    for dtype in (W.F16, W.BF16):
        cfg = W.small_config(name="e4m3heads", kind="prefill", dtype=dtype, batch=3, num_heads=6, num_kv_heads=3,
                             head_dim=16, block_size=4, num_blocks=64, ctx_lo=9, ctx_hi=37, q_len=5, seed=41)
        case = W.make_case(cfg)
        k_all, v_all, slots = _all_tokens(case)
        shape = (cfg.num_blocks, cfg.num_kv_heads, cfg.block_size, cfg.head_dim)
        kc8, vc8 = np.full(shape, 0x7F, np.uint8), np.full(shape, 0x7F, np.uint8)
        O.reshape_and_cache_e4m3_heads(k_all, v_all, kc8, vc8, slots, k_scales, v_scales, dtype, lib=lib)
        for g in range(3):
            kt, vt = np.full(shape, 0x7F, np.uint8), np.full(shape, 0x7F, np.uint8)
            O.reshape_and_cache_e4m3(k_all, v_all, kt, vt, slots, k_scales[g], v_scales[g], dtype)
            assert np.array_equal(kc8[:, g], kt[:, g]) and np.array_equal(vc8[:, g], vt[:, g]), f"cache write, KV head {g}"
        assert len({kc8[:, g].tobytes() for g in range(3)}) == 3
        # decode: the last new token of every sequence as the query
        last = case.cu_q_lens[1:] - 1
        qd = case.q[last]
        got = O.paged_attention_e4m3_heads(qd, kc8, vc8, case.block_tables, case.context_lens, case.slopes, case.scale,
                                           k_scales, v_scales, dtype, lib=lib)
        pf = O.paged_prefill_e4m3_heads(case.q, kc8, vc8, case.block_tables, case.context_lens, case.cu_q_lens,
                                        case.slopes, case.scale, k_scales, v_scales, dtype, lib=lib)
        for g in range(3):
            ref = O.paged_attention_e4m3(qd, kc8, vc8, case.block_tables, case.context_lens, case.slopes, case.scale,
                                         k_scales[g], v_scales[g], dtype)
            refp = O.paged_prefill_e4m3(case.q, kc8, vc8, case.block_tables, case.context_lens, case.cu_q_lens,
                                        case.slopes, case.scale, k_scales[g], v_scales[g], dtype)
            for h in (2 * g, 2 * g + 1):
                np.testing.assert_allclose(got[:, h], ref[:, h], rtol=1e-13, atol=0, err_msg=f"decode, head {h}")
                np.testing.assert_allclose(pf[:, h], refp[:, h], rtol=1e-13, atol=0, err_msg=f"prefill, head {h}")
            other = (2 * g + 2) % 6
            assert np.max(np.abs(got[:, other] - ref[:, other])) > 1e-6          # the scales do differ in effect
        # row lists pick the same rows
        rows = [(0, 0), (2, 5), (1, 3)]
        sub = O.paged_attention_e4m3_heads(qd, kc8, vc8, case.block_tables, case.context_lens, case.slopes, case.scale,
                                           k_scales, v_scales, dtype, rows=rows, lib=lib)
        assert np.array_equal(sub, np.stack([got[b, h] for b, h in rows]))
        rows = [(0, 0), (case.num_tokens - 1, 5), (4, 2)]
        sub = O.paged_prefill_e4m3_heads(case.q, kc8, vc8, case.block_tables, case.context_lens, case.cu_q_lens,
                                         case.slopes, case.scale, k_scales, v_scales, dtype, rows=rows, lib=lib)
        assert np.array_equal(sub, np.stack([pf[t, h] for t, h in rows]))
        # the same pair for every head is the per-tensor clause
        u = np.full(3, 0.125, np.float32)
        a = O.paged_attention_e4m3_heads(qd, kc8, vc8, case.block_tables, case.context_lens, case.slopes, case.scale,
                                         u, 2 * u, dtype, lib=lib)
        b_ = O.paged_attention_e4m3(qd, kc8, vc8, case.block_tables, case.context_lens, case.slopes, case.scale,
                                    np.float32(0.125), np.float32(0.25), dtype)
        np.testing.assert_allclose(a, b_, rtol=1e-14, atol=0)


def check_two_byte_decoder_on_every_pattern(lib=None):
    """The 2-byte decoder of this file (queries and new-token rows) on all 65 536 fp16 and bf16
    patterns.  Two routes, both compared with numpy's own decoding of the pattern:

    * as a query: one sequence per pattern, head_dim 1, two cached tokens with codes K = (0, 1),
      V = (0, 1), no slopes, unit cache scales: the output is the weight of the second key,
      1 / (1 + exp(-scale * q)) - a logistic function, which resolves the last mantissa bit of q
      wherever |scale * k_scale * q| is of order 1.  scale * k_scale runs over the powers of two that bring
      every finite magnitude there once.  Infinite and NaN queries give NaN (inf * 0 in the first
      key's product), which a decoder that turned them into large finite numbers would not.
    * as a new-token row of the quantising cache write at scale 1: every finite pattern of
      magnitude <= 448 must land on the code the library cast gives its numpy-decoded value; larger
      ones (infinities included) saturate, NaN patterns give 0x7f."""
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    one = 0x38                                           # code of 1.0
    for dtype, e_lo, e_hi in ((W.F16, -24, 16), (W.BF16, -133, 128)):
        x = W.from_bits(bits, dtype)
        B = 65536
        q = bits.reshape(B, 1, 1).copy()
        kc8 = np.zeros((B, 1, 2, 1), np.uint8)
        kc8[:, 0, 1, 0] = one
        vc8 = kc8.copy()
        tables = np.arange(B, dtype=np.int32).reshape(B, 1)
        lens = np.full(B, 2, np.int32)
        seen = np.zeros(B, bool)
        fin = np.isfinite(x)
        with np.errstate(over="ignore", invalid="ignore"):
            for e in range(e_lo, e_hi + 1):
                a = int(np.clip(-e, -100, 100))              # 2^-e split over the score scale and k_scale
                scale, k_scale = np.float32(2.0 ** a), np.float32(2.0 ** (-e - a))
                sens = fin & (np.abs(x) >= 2.0 ** (e - 2)) & (np.abs(x) < 2.0 ** (e + 1))
                if not sens.any():
                    continue
                out = O.paged_attention_e4m3(q, kc8, vc8, tables, lens, None, scale, k_scale, 1.0, dtype, lib=lib)[:, 0, 0]
                want = 1.0 / (1.0 + np.exp(-(2.0 ** -e * x[sens])))
                np.testing.assert_allclose(out[sens], want, rtol=1e-13, atol=0, err_msg=f"{dtype} scale 2^{-e}")
                seen |= sens
                if e == 0:
                    assert np.all(np.isnan(out[~fin])) and np.count_nonzero(~fin) > 2
                    assert np.all(out[fin & (x == 0)] == 0.5)
        assert np.all(seen[fin & (x != 0)]), f"{dtype}: a finite pattern was never in the sensitive range"
        # the cache-write route
        rows = bits.reshape(4096, 1, 16)
        slots = np.arange(4096, dtype=np.int64)
        kc = np.full((256, 1, 16, 16), 0x7F, np.uint8)
        vc = np.full((256, 1, 16, 16), 0x7F, np.uint8)
        O.reshape_and_cache_e4m3(rows, rows, kc, vc, slots, 1.0, 1.0, dtype, lib)
        got = kc.reshape(-1)
        assert np.array_equal(got, vc.reshape(-1))
        inr = fin & (np.abs(x) <= 448)
        lib_codes = torch.from_numpy(x[inr].astype(np.float32)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
        assert np.array_equal(got[inr], lib_codes), f"{dtype}: cache write of in-range patterns"
        assert np.all(got[np.isnan(x)] == 0x7F)
        big = ~np.isnan(x) & (np.abs(x) > 448)
        assert np.array_equal(got[big], np.where(x[big] > 0, 0x7E, 0xFE).astype(np.uint8))


ALL_CHECKS = [
    check_prefill_reduces_to_two_byte_oracle_and_to_decodes,
    check_values_match_library_type,
    check_nearest_on_representable_values_and_midpoints,
    check_nearest_matches_library_in_range,
    check_nearest_saturates_and_orders,
    check_cache_write_against_library_cast,
    check_attention_reduces_to_two_byte_oracle,
    check_scales_enter_where_the_definition_says,
    check_two_byte_decoder_on_every_pattern,
    check_per_head_scales_reduce_to_per_tensor_clauses,
]
