"""GPU parity: the HIP path through the C ABI against the fp64 CPU oracle, element by element.

Bar: caches and index work bit-exact; attention outputs within 2e-3 (fp16) / 1e-2 (bf16)
max-abs of the oracle's fp64 result."""
import numpy as np
import pytest

import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def U():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    import paper_2505_02351_amd as G
    G.load_library()                       # fails loudly if the HIP library is not built
    import harness
    return harness


# Full-size workloads: the stated tolerance on every element of magnitude below 4.  Heads with a steep
# ALiBi slope (2^-0.25 per token for head 0) put most of their weight on the last one or two keys, so
# a handful of the millions of outputs are single N(0,1) V elements beyond 4, which the 2-byte output
# format itself rounds by more than the stated bar; harness.check_scaled bounds those by the format's
# half-ulp plus the unchanged compute budget, and at most this fraction of the elements may be such.
WORKLOAD_EXEMPT = 1e-4

_CASES = {}


def workload_case(name):
    """The full-size batches take seconds to draw; tests that do not modify them share one."""
    if name not in _CASES:
        _CASES.clear()                      # one at a time: each holds up to 1.3 GB of cache images
        _CASES[name] = W.make_case(W.CONFIGS[name])
    return _CASES[name]


def oracle_filled(O, case):
    kc, vc = case.k_cache.copy(), case.v_cache.copy()
    O.reshape_and_cache(case.k_new, case.v_new, kc, vc, case.slot_mapping)
    return kc, vc


def oracle_decode(O, case, kc, vc, rows=None, slopes="case"):
    sl = case.slopes if isinstance(slopes, str) else slopes
    return O.paged_attention(case.q, kc, vc, case.block_tables, case.context_lens, sl, case.scale,
                             case.dtype, rows=rows)


# ------------------------------------------------------------------ cache write (bit-exact)
CW = [
    dict(dtype=W.F16, batch=3, num_heads=8, num_kv_heads=2, head_dim=64, block_size=16, ctx_hi=90, q_len=1),
    dict(dtype=W.BF16, batch=5, num_heads=8, num_kv_heads=4, head_dim=128, block_size=32, ctx_hi=300, q_len=1),
    dict(dtype=W.BF16, batch=4, num_heads=4, num_kv_heads=1, head_dim=128, block_size=16, ctx_lo=40, ctx_hi=200,
         q_len=37, kind="prefill"),
    dict(dtype=W.F16, batch=2, num_heads=6, num_kv_heads=3, head_dim=64, block_size=64, ctx_lo=70, ctx_hi=500,
         q_len=70, kind="prefill"),
]


@pytest.mark.parametrize("i", range(len(CW)))
def test_cache_write_bit_exact(U, oracle, i):
    import torch
    import paper_2505_02351_amd as G
    cfg = W.small_config(name=f"cw{i}", num_blocks=128, seed=300 + i, **CW[i])
    case = W.make_case(cfg)
    dev = U.DevCase(case)
    dev.write_cache()
    torch.cuda.synchronize()
    kc, vc = oracle_filled(oracle, case)
    assert np.array_equal(U.to_host(dev.k_cache), kc)       # the ENTIRE buffers, NaN sentinels included
    assert np.array_equal(U.to_host(dev.v_cache), vc)

    # padding tokens (negative slots) and a strided source (token stride > Hkv*D)
    dev2 = U.DevCase(case)
    slots = case.slot_mapping.copy()
    slots[1::3] = -1
    T, Hkv, D = case.k_new.shape
    wide_k = torch.zeros((T, Hkv * D + 24), dtype=dev2.k_new.dtype, device="cuda")
    wide_v = torch.zeros((T, Hkv * D + 8), dtype=dev2.k_new.dtype, device="cuda")
    wide_k[:, : Hkv * D] = dev2.k_new.reshape(T, -1)
    wide_v[:, : Hkv * D] = dev2.v_new.reshape(T, -1)
    k_view = wide_k[:, : Hkv * D].view(T, Hkv, D)
    v_view = wide_v[:, : Hkv * D].view(T, Hkv, D)
    G.reshape_and_cache(k_view, v_view, dev2.k_cache, dev2.v_cache, torch.from_numpy(slots).cuda())
    torch.cuda.synchronize()
    kc2, vc2 = case.k_cache.copy(), case.v_cache.copy()
    oracle.reshape_and_cache(case.k_new, case.v_new, kc2, vc2, slots)
    assert np.array_equal(U.to_host(dev2.k_cache), kc2)
    assert np.array_equal(U.to_host(dev2.v_cache), vc2)

    # odd element stride -> the 2-byte copy path
    dev3 = U.DevCase(case)
    odd_k = torch.zeros((T, Hkv * D + 3), dtype=dev3.k_new.dtype, device="cuda")
    odd_k[:, : Hkv * D] = dev3.k_new.reshape(T, -1)
    G.reshape_and_cache(odd_k[:, : Hkv * D].view(T, Hkv, D), dev3.v_new, dev3.k_cache, dev3.v_cache,
                        dev3.slot_mapping)
    torch.cuda.synchronize()
    assert np.array_equal(U.to_host(dev3.k_cache), kc)
    assert np.array_equal(U.to_host(dev3.v_cache), vc)


def test_gather_kv_bit_exact(U, oracle):
    import torch
    import paper_2505_02351_amd as G
    cfg = W.small_config(name="gather", dtype=W.BF16, batch=4, num_heads=8, num_kv_heads=2, head_dim=128,
                         block_size=16, num_blocks=64, ctx_lo=1, ctx_hi=150, seed=310)
    case = W.make_case(cfg)
    dev = U.DevCase(case)
    dev.write_cache()
    Lmax = case.max_context_len
    k_out = torch.zeros((cfg.batch, Lmax, 2, 128), dtype=torch.bfloat16, device="cuda")
    v_out = torch.zeros_like(k_out)
    G.gather_kv(k_out, v_out, dev.k_cache, dev.v_cache, dev.block_tables, dev.context_lens)
    torch.cuda.synchronize()
    kc, vc = oracle_filled(oracle, case)
    kh, vh = U.to_host(k_out), U.to_host(v_out)
    for b in range(cfg.batch):
        L = int(case.context_lens[b])
        j = np.arange(L)
        blk = case.block_tables[b, j // 16]
        assert np.array_equal(kh[b, :L], kc[blk, :, j % 16, :])
        assert np.array_equal(vh[b, :L], vc[blk, :, j % 16, :])
        assert not kh[b, L:].any() and not vh[b, L:].any()


# ------------------------------------------------------------------ decode, small sweep
BALANCED = -2      # OPTGQA_SPLIT_BALANCED

SWEEP = [
    # dtype, Hq, Hkv, D, bs, batch, ctx_lo, ctx_hi
    (W.F16, 8, 2, 64, 16, 3, 1, 200),
    (W.BF16, 8, 2, 64, 16, 3, 1, 200),
    (W.F16, 32, 8, 128, 16, 5, 1, 700),
    (W.BF16, 32, 4, 128, 32, 4, 1, 900),
    (W.F16, 16, 16, 128, 16, 2, 30, 333),       # MHA, G = 1
    (W.BF16, 4, 2, 128, 64, 3, 1, 400),         # G = 2, block 64
    (W.F16, 12, 4, 64, 32, 3, 1, 300),          # G = 3 -> one head per workgroup
    (W.BF16, 12, 2, 128, 16, 2, 1, 300),        # G = 6 -> two heads per workgroup, three chunks
    (W.F16, 32, 2, 64, 16, 2, 1, 500),          # G = 16 -> two chunks of eight
    (W.BF16, 8, 1, 128, 16, 2, 1, 1500),        # multi-query
]


@pytest.mark.parametrize("i", range(len(SWEEP)))
@pytest.mark.parametrize("partition", [-1, 0, 64, 256, BALANCED])
def test_decode_sweep(U, oracle, i, partition):
    dtype, Hq, Hkv, D, bs, B, lo, hi = SWEEP[i]
    if partition > 0 and partition % bs:
        pytest.skip("partition size must be a multiple of the block size")
    cfg = W.small_config(name=f"sweep{i}", dtype=dtype, batch=B, num_heads=Hq, num_kv_heads=Hkv,
                         head_dim=D, block_size=bs, num_blocks=B * ((hi + bs - 1) // bs) + 7, ctx_lo=lo,
                         ctx_hi=hi, seed=400 + i)
    case = W.make_case(cfg)
    dev = U.DevCase(case)
    dev.write_cache()
    got = dev.decode(partition_size=partition)
    kc, vc = oracle_filled(oracle, case)
    ref = oracle_decode(oracle, case, kc, vc)
    err = U.max_abs_err(got, ref, dtype)
    assert err <= U.TOL[dtype], f"max abs err {err}"


@pytest.mark.parametrize("dtype", [W.F16, W.BF16])
def test_decode_edge_lengths(U, oracle, dtype):
    """Context lengths 0, 1, exactly one block, block +- 1, partition +- 1, in one batch."""
    lens = np.array([0, 1, 15, 16, 17, 31, 32, 33, 255, 256, 257, 512, 1], np.int32)
    cfg = W.small_config(name="edges", dtype=dtype, batch=len(lens), num_heads=8, num_kv_heads=2, head_dim=128,
                         block_size=16, num_blocks=160, ctx_lo=1, ctx_hi=512, seed=420)
    case = W.make_case(cfg, context_lens=lens)
    # q rows exist only for non-empty sequences in the generator; give every sequence a row
    q_full = np.zeros((len(lens), 8, 128), np.uint16)
    q_full[lens > 0] = case.q
    case.q = q_full
    kc, vc = oracle_filled(oracle, case)
    ref = oracle_decode(oracle, case, kc, vc)
    for partition in (-1, 0, 64, 256, BALANCED):
        dev = U.DevCase(case)
        dev.write_cache()
        got = dev.decode(partition_size=partition)
        assert not got[0].any(), "an empty context must give +0"
        assert U.max_abs_err(got, ref, dtype) <= U.TOL[dtype]
        # a one-token context returns V bit for bit (weight exactly 1)
        for b in (1, 12):
            pb = case.block_tables[b, 0]
            for h in range(8):
                assert np.array_equal(got[b, h], vc[pb, h // 4, 0, :])


@pytest.mark.parametrize("dtype", [W.F16, W.BF16])
def test_decode_one_hot_selects_row_bit_exact(U, oracle, dtype):
    """K = 0 and a slope of +-200: every weight but one underflows to exactly 0, so the output
    must be the selected V row bit for bit -- pins block-table, partial-block and partition
    indexing through the real kernels."""
    Hq = 8
    slopes = np.array([200.0, -200.0] * (Hq // 2), np.float32)
    cfg = W.small_config(name="onehot", dtype=dtype, batch=6, num_heads=Hq, num_kv_heads=2, head_dim=128,
                         block_size=16, num_blocks=300, ctx_lo=1, ctx_hi=700, seed=430)
    case = W.make_case(cfg, slopes=slopes)
    case.k_cache[:] = 0
    case.k_new[:] = 0
    kc, vc = oracle_filled(oracle, case)
    for partition in (-1, 64, 256, BALANCED):
        dev = U.DevCase(case)
        dev.write_cache()
        got = dev.decode(partition_size=partition)
        for b in range(cfg.batch):
            L = int(case.context_lens[b])
            newest = vc[case.block_tables[b, (L - 1) // 16], :, (L - 1) % 16, :]
            oldest = vc[case.block_tables[b, 0], :, 0, :]
            for h in range(Hq):
                want = newest if h % 2 == 0 else oldest
                assert np.array_equal(got[b, h], want[h // 4]), (partition, b, h)


def test_decode_block_permutation_bit_identical(U, oracle):
    cfg = W.small_config(name="permgpu", dtype=W.F16, batch=4, num_heads=16, num_kv_heads=4, head_dim=128,
                         block_size=16, num_blocks=256, ctx_lo=1, ctx_hi=800, seed=440)
    outs = []
    for ps in (None, 5, 6):
        case = W.make_case(cfg, perm_seed=ps)
        dev = U.DevCase(case)
        dev.write_cache()
        outs.append(dev.decode(partition_size=0))
    assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[0], outs[2])


def test_decode_no_slopes_and_steep_slopes(U, oracle):
    cfg = W.small_config(name="slopes", dtype=W.F16, batch=3, num_heads=8, num_kv_heads=2, head_dim=64,
                         block_size=16, num_blocks=200, ctx_lo=100, ctx_hi=900, seed=450)
    case = W.make_case(cfg)
    dev = U.DevCase(case)
    dev.write_cache()
    kc, vc = oracle_filled(oracle, case)
    got = dev.decode(slopes=None)
    ref = oracle_decode(oracle, case, kc, vc, slopes=None)
    assert U.max_abs_err(got, ref, W.F16) <= U.TOL[W.F16]
    import torch
    steep = np.array([30.0, 7.0, 1.0, 0.0, 0.25, 3.0, 12.0, 0.01], np.float32)
    for partition in (-1, 64):
        got = dev.decode(slopes=torch.from_numpy(steep).cuda(), partition_size=partition)
        ref = oracle_decode(oracle, case, kc, vc, slopes=steep)
        assert U.max_abs_err(got, ref, W.F16) <= U.TOL[W.F16]


def test_append_equals_bulk_fill(U, oracle):
    """Token-by-token (cache write of one token, then decode) reaches the same cache bits and the
    same output as one bulk fill followed by one decode (eq. (2))."""
    import torch
    import paper_2505_02351_amd as G
    steps = 20
    cfg = W.small_config(name="append", kind="prefill", dtype=W.BF16, batch=2, num_heads=8, num_kv_heads=2,
                         head_dim=128, block_size=16, num_blocks=32, ctx_lo=45, ctx_hi=60, q_len=steps, seed=460)
    case = W.make_case(cfg)
    bulk = U.DevCase(case)
    bulk.write_cache()
    inc = U.DevCase(case)
    out = torch.empty((2, 8, 128), dtype=torch.bfloat16, device="cuda")
    for s in range(steps):
        idx = torch.tensor([int(case.cu_q_lens[b]) + s for b in range(2)], device="cuda")
        G.reshape_and_cache(inc.k_new[idx], inc.v_new[idx], inc.k_cache, inc.v_cache, inc.slot_mapping[idx])
        lens = torch.from_numpy(case.context_lens - steps + s + 1).cuda()
        G.paged_attention(out, inc.q[idx].contiguous(), inc.k_cache, inc.v_cache, inc.block_tables, lens,
                          inc.slopes, float(case.scale), int(lens.max()), -1, None)
    torch.cuda.synchronize()
    assert np.array_equal(U.to_host(inc.k_cache), U.to_host(bulk.k_cache))
    assert np.array_equal(U.to_host(inc.v_cache), U.to_host(bulk.v_cache))
    last = torch.tensor([int(case.cu_q_lens[b]) + steps - 1 for b in range(2)], device="cuda")
    out2 = torch.empty_like(out)
    G.paged_attention(out2, bulk.q[last].contiguous(), bulk.k_cache, bulk.v_cache, bulk.block_tables,
                      bulk.context_lens, bulk.slopes, float(case.scale), case.max_context_len, -1, None)
    torch.cuda.synchronize()
    assert np.array_equal(U.to_host(out), U.to_host(out2))


@pytest.mark.parametrize("B,hi,zeros", [(300, 90, 40), (4200, 40, 900)])
def test_decode_balanced_many_sequences(U, oracle, B, hi, zeros):
    """Equal-work split with more sequences than lanes (every lane scans a run of sequences, then
    the run is searched), short and empty contexts mixed in, so that many units cross several
    sequence boundaries and some sequences are skipped altogether."""
    rng = np.random.default_rng(B)
    lens = rng.integers(1, hi + 1, size=B).astype(np.int32)
    lens[rng.choice(B, size=zeros, replace=False)] = 0
    lens[-1] = 0                      # the walk must also end on an empty sequence
    lens[B // 2] = hi * 8             # one long context among the short ones
    cfg = W.small_config(name="many", dtype=W.BF16, batch=B, num_heads=8, num_kv_heads=2, head_dim=128,
                         block_size=16, num_blocks=int(np.sum((lens + 15) // 16)) + 5, ctx_lo=1,
                         ctx_hi=hi * 8, seed=B)
    case = W.make_case(cfg, context_lens=lens)
    q_full = np.zeros((B, 8, 128), np.uint16)
    q_full[lens > 0] = case.q
    case.q = q_full
    dev = U.DevCase(case)
    dev.write_cache()
    got = dev.decode(partition_size=BALANCED)
    kc, vc = oracle_filled(oracle, case)
    ref = oracle_decode(oracle, case, kc, vc)
    assert not got[lens == 0].any(), "an empty context must give +0"
    assert U.max_abs_err(got, ref, W.BF16) <= U.TOL[W.BF16]


def test_decode_more_sequences_than_a_16_bit_grid(U, oracle):
    """70 000 one-block sequences in one call: the unsplit kernels run in slices of 65 535 rows, and
    the equal-work kernel with its two combine kernels takes the whole batch (sequences run along
    the x dimension of their grids)."""
    B = 70000
    rng = np.random.default_rng(70)
    lens = rng.integers(1, 17, size=B).astype(np.int32)
    lens[rng.choice(B, size=2000, replace=False)] = 0
    lens[B - 1] = 16
    cfg = W.small_config(name="grid16", dtype=W.F16, batch=B, num_heads=2, num_kv_heads=1, head_dim=64,
                         block_size=16, num_blocks=B + 3, ctx_lo=1, ctx_hi=16, seed=71)
    case = W.make_case(cfg, context_lens=lens)
    q_full = np.zeros((B, 2, 64), np.uint16)
    q_full[lens > 0] = case.q
    case.q = q_full
    kc, vc = oracle_filled(oracle, case)
    ref = oracle_decode(oracle, case, kc, vc)
    for partition in (-1, BALANCED, 16):
        dev = U.DevCase(case)
        dev.write_cache()
        got = dev.decode(partition_size=partition)
        assert not got[lens == 0].any(), partition
        assert U.max_abs_err(got, ref, W.F16) <= U.TOL[W.F16], partition


def test_decode_one_very_long_context(U, oracle):
    """A context of 2^20 tokens next to one of five tokens: 65 536 tiles in one segment, every
    unit of the equal-work split inside the same sequence, 256 fixed partitions of 4096 tokens,
    and the unsplit kernel walking it alone."""
    lens = np.array([1 << 20, 5], np.int32)
    cfg = W.small_config(name="long", dtype=W.BF16, batch=2, num_heads=4, num_kv_heads=1, head_dim=128,
                         block_size=64, num_blocks=(1 << 14) + 3, ctx_lo=1, ctx_hi=1 << 20, seed=4200)
    case = W.make_case(cfg, context_lens=lens)
    kc, vc = oracle_filled(oracle, case)
    ref = oracle_decode(oracle, case, kc, vc)
    dev = U.DevCase(case)
    got = dev.step()
    assert np.array_equal(U.to_host(dev.k_cache), kc) and np.array_equal(U.to_host(dev.v_cache), vc)
    assert U.max_abs_err(got, ref, W.BF16) <= U.TOL[W.BF16]
    for partition in (4096, BALANCED, -1):
        assert U.max_abs_err(dev.decode(partition_size=partition), ref, W.BF16) <= U.TOL[W.BF16], partition
    ref_w = __import__("oracle").paged_attention_window(case.q, kc, vc, case.block_tables, case.context_lens,
                                                        case.slopes, case.scale, 100000, W.BF16)
    assert U.max_abs_err(dev.decode_window(100000), ref_w, W.BF16) <= U.TOL[W.BF16]


def test_prefill_long_cached_context(U, oracle):
    """100 new tokens behind 150 000 cached ones: 4 700 key tiles per workgroup, nearly all of them
    far enough back for the steep-slope head to skip and none for the head without a slope."""
    cfg = W.small_config(name="longpf", kind="prefill", dtype=W.BF16, batch=1, num_heads=4, num_kv_heads=2,
                         head_dim=128, block_size=64, num_blocks=2400, ctx_lo=150100, ctx_hi=150100, q_len=100,
                         seed=4300)
    slopes = np.array([0.5, 0.0, 2.0 ** -10, 2.0 ** -16], np.float32)
    case = W.make_case(cfg, slopes=slopes)
    kc, vc = oracle_filled(oracle, case)
    ref = oracle.paged_prefill(case.q, kc, vc, case.block_tables, case.context_lens, case.cu_q_lens, case.slopes,
                               case.scale, case.dtype)
    dev = U.DevCase(case)
    dev.write_cache()
    U.check_scaled(dev.prefill(), ref, W.BF16, "prefill behind 150 000 cached tokens")


def lift_to_large_pool(dev, total_blocks):
    """Moves a DevCase's cache blocks to the top of a pool of ``total_blocks`` blocks (the rest is
    left uninitialised: no table names it), so that block offsets no longer fit 32 bits."""
    import torch
    n, bs = dev.k_cache.shape[0], dev.k_cache.shape[2]
    off = total_blocks - n
    for name in ("k_cache", "v_cache"):
        small = getattr(dev, name)
        big = torch.empty((total_blocks,) + tuple(small.shape[1:]), dtype=small.dtype, device="cuda")
        big[off:] = small
        setattr(dev, name, big)
    dev.block_tables = dev.block_tables + off
    dev.slot_mapping = torch.where(dev.slot_mapping >= 0, dev.slot_mapping + off * bs, dev.slot_mapping)
    return off


def test_pool_larger_than_4_gib(U, oracle):
    """Caches of 4.6 GB each with the batch's blocks at the top: element offsets beyond 2^31 and byte
    offsets beyond 2^32 in the cache write, every decode path and the prefill (the oracle sees the
    same blocks in a small pool: results do not depend on where a block lives)."""
    import torch
    total = 70000                                            # x 64 KiB per block and tensor
    cfg = W.small_config(name="bigpool", dtype=W.BF16, batch=6, num_heads=16, num_kv_heads=8, head_dim=128,
                         block_size=32, num_blocks=6 * 20 + 5, ctx_lo=30, ctx_hi=600, seed=4100)
    case = W.make_case(cfg)
    kc, vc = oracle_filled(oracle, case)
    ref = oracle_decode(oracle, case, kc, vc)
    dev = U.DevCase(case)
    off = lift_to_large_pool(dev, total)
    assert off * kc[0].size * 2 > 2 ** 32
    got = dev.step()                                         # fused cache write + equal-work split
    assert np.array_equal(U.to_host(dev.k_cache[off:]), kc) and np.array_equal(U.to_host(dev.v_cache[off:]), vc)
    assert U.max_abs_err(got, ref, W.BF16) <= U.TOL[W.BF16]
    for partition in (-1, 64, BALANCED):
        assert U.max_abs_err(dev.decode(partition_size=partition), ref, W.BF16) <= U.TOL[W.BF16], partition
    assert U.max_abs_err(dev.decode_window(10 ** 6), ref, W.BF16) <= U.TOL[W.BF16]
    dev2 = U.DevCase(case)
    lift_to_large_pool(dev2, total)
    dev2.write_cache()                                       # the separate cache-write kernel
    assert np.array_equal(U.to_host(dev2.k_cache[off:]), kc) and np.array_equal(U.to_host(dev2.v_cache[off:]), vc)
    del dev, dev2
    torch.cuda.empty_cache()
    pcfg = W.small_config(name="bigpool-pf", kind="prefill", dtype=W.F16, batch=3, num_heads=8, num_kv_heads=8,
                          head_dim=128, block_size=32, num_blocks=3 * 12 + 5, ctx_lo=100, ctx_hi=380, q_len=70,
                          seed=4101)
    pcase = W.make_case(pcfg)
    kc, vc = oracle_filled(oracle, pcase)
    pref = oracle.paged_prefill(pcase.q, kc, vc, pcase.block_tables, pcase.context_lens, pcase.cu_q_lens,
                                pcase.slopes, pcase.scale, pcase.dtype)
    pdev = U.DevCase(pcase)
    off = lift_to_large_pool(pdev, total)
    pdev.write_cache()
    assert np.array_equal(U.to_host(pdev.k_cache[off:]), kc)
    U.check_scaled(pdev.prefill(), pref, W.F16, "prefill, pool of 4.6 GB")
    del pdev
    torch.cuda.empty_cache()
    # 8-bit caches of 4.6 GB each (140 000 blocks of 32 KiB): quantising write, decode, prefill
    import oracle as O
    import paper_2505_02351_amd as G
    import pins_e4m3
    total8 = 140000
    k_scale, v_scale = 0.0125, 0.02
    kc8, vc8, (k_all, v_all, slots) = pins_e4m3.quantised_cache(pcase, k_scale, v_scale)
    off = total8 - kc8.shape[0]
    assert off * kc8[0].size > 2 ** 32
    dk = torch.empty((total8,) + kc8.shape[1:], dtype=torch.uint8, device="cuda")
    dv = torch.empty((total8,) + vc8.shape[1:], dtype=torch.uint8, device="cuda")
    dk[off:] = 0x7F
    dv[off:] = 0x7F
    G.reshape_and_cache_fp8(U.to_dev(k_all, pcase.dtype), U.to_dev(v_all, pcase.dtype), dk, dv,
                            torch.from_numpy(slots + off * pcfg.block_size).cuda(), k_scale, v_scale)
    torch.cuda.synchronize()
    assert np.array_equal(dk[off:].cpu().numpy(), kc8) and np.array_equal(dv[off:].cpu().numpy(), vc8)
    qd = U.to_dev(pcase.q, pcase.dtype)
    out = torch.full_like(qd, float("nan"))
    G.paged_prefill_fp8(out, qd, dk, dv, torch.from_numpy(pcase.block_tables + off).cuda(),
                        torch.from_numpy(pcase.context_lens).cuda(), torch.from_numpy(pcase.cu_q_lens).cuda(),
                        torch.from_numpy(pcase.slopes).cuda(), float(pcase.scale), k_scale, v_scale, pcase.max_q_len)
    ref8 = O.paged_prefill_e4m3(pcase.q, kc8, vc8, pcase.block_tables, pcase.context_lens, pcase.cu_q_lens,
                                pcase.slopes, pcase.scale, k_scale, v_scale, pcase.dtype)
    U.check_scaled(U.to_host(out), ref8, pcase.dtype, "prefill over E4M3 caches, pool of 4.6 GB")
    # decode over the same caches: the last new token of every sequence as the query
    last = pcase.cu_q_lens[1:] - 1
    q_dec = np.ascontiguousarray(pcase.q[last])
    n, _ = G.paged_attention_workspace_bytes(pcfg.batch, pcfg.num_heads, pcfg.num_kv_heads, 128, pcfg.block_size,
                                             pcase.max_context_len, G.SPLIT_BALANCED)
    ws = torch.empty(n // 4, dtype=torch.float32, device="cuda")
    qdd = U.to_dev(q_dec, pcase.dtype)
    outd = torch.full_like(qdd, float("nan"))
    G.paged_attention_fp8(outd, qdd, dk, dv, torch.from_numpy(pcase.block_tables + off).cuda(),
                          torch.from_numpy(pcase.context_lens).cuda(), torch.from_numpy(pcase.slopes).cuda(),
                          float(pcase.scale), k_scale, v_scale, pcase.max_context_len, ws)
    torch.cuda.synchronize()
    refd = O.paged_attention_e4m3(q_dec, kc8, vc8, pcase.block_tables, pcase.context_lens, pcase.slopes, pcase.scale,
                                  k_scale, v_scale, pcase.dtype)
    assert U.max_abs_err(U.to_host(outd), refd, pcase.dtype) <= U.TOL[pcase.dtype]
    del dk, dv
    torch.cuda.empty_cache()


def test_decode_balanced_and_fixed_partitions_against_the_oracle(U, oracle):
    """The two ways of splitting the context, on a ragged batch whose units start and end inside
    segments: each against the oracle at the stated tolerance, and against each other to well inside
    it (they differ only in fp32 combine order)."""
    cfg = W.small_config(name="bal", dtype=W.F16, batch=9, num_heads=16, num_kv_heads=4, head_dim=128,
                         block_size=32, num_blocks=9 * 40 + 3, ctx_lo=1, ctx_hi=1200, seed=77)
    case = W.make_case(cfg)
    dev = U.DevCase(case)
    dev.write_cache()
    kc, vc = oracle_filled(oracle, case)
    ref = oracle_decode(oracle, case, kc, vc)
    got_a, got_b = dev.decode(partition_size=BALANCED), dev.decode(partition_size=256)
    assert U.max_abs_err(got_a, ref, W.F16) <= U.TOL[W.F16]
    assert U.max_abs_err(got_b, ref, W.F16) <= U.TOL[W.F16]
    a, b = W.from_bits(got_a, W.F16), W.from_bits(got_b, W.F16)
    assert np.max(np.abs(a - b)) <= 2.0 ** -9          # one fp16 ulp in [1, 2): both sit on the same side of the oracle


@pytest.mark.parametrize("dtype", [W.F16, W.BF16])
def test_decode_edge_lengths_head_dim_64(U, oracle, dtype):
    """The edge lengths of the head_dim 128 test at head_dim 64 (a V tile is fetched 8 rows a load there,
    a K row is two MFMAs): every split mode, an empty context gives +0, a one-token context returns V."""
    lens = np.array([0, 1, 15, 16, 17, 31, 32, 33, 255, 256, 257, 512, 1], np.int32)
    cfg = W.small_config(name="edges64", dtype=dtype, batch=len(lens), num_heads=8, num_kv_heads=2, head_dim=64,
                         block_size=16, num_blocks=160, ctx_lo=1, ctx_hi=512, seed=421)
    case = W.make_case(cfg, context_lens=lens)
    q_full = np.zeros((len(lens), 8, 64), np.uint16)
    q_full[lens > 0] = case.q
    case.q = q_full
    kc, vc = oracle_filled(oracle, case)
    ref = oracle_decode(oracle, case, kc, vc)
    for partition in (-1, 0, 64, 256, BALANCED):
        dev = U.DevCase(case)
        dev.write_cache()
        got = dev.decode(partition_size=partition)
        assert not got[0].any(), "an empty context must give +0"
        assert U.max_abs_err(got, ref, dtype) <= U.TOL[dtype], partition
        for b in (1, 12):
            pb = case.block_tables[b, 0]
            for h in range(8):
                assert np.array_equal(got[b, h], vc[pb, h // 4, 0, :])


# ------------------------------------------------------------------ decode step in one call
@pytest.mark.parametrize("i", range(len(SWEEP)))
def test_decode_step_sweep(U, oracle, i):
    """optgqa_decode_step = cache write + attention: caches bit-exact, output within tolerance.
    Shapes with a long enough context take the fused kernel, the others the library's two-launch
    path."""
    dtype, Hq, Hkv, D, bs, B, lo, hi = SWEEP[i]
    cfg = W.small_config(name=f"step{i}", dtype=dtype, batch=B, num_heads=Hq, num_kv_heads=Hkv,
                         head_dim=D, block_size=bs, num_blocks=B * ((hi + bs - 1) // bs) + 7, ctx_lo=lo,
                         ctx_hi=hi, seed=700 + i)
    case = W.make_case(cfg)
    dev = U.DevCase(case)
    got = dev.step()
    kc, vc = oracle_filled(oracle, case)
    assert np.array_equal(U.to_host(dev.k_cache), kc) and np.array_equal(U.to_host(dev.v_cache), vc)
    ref = oracle_decode(oracle, case, kc, vc)
    assert U.max_abs_err(got, ref, dtype) <= U.TOL[dtype]
    # without a workspace the library must still do both halves (unsplit kernels)
    dev2 = U.DevCase(case)
    got2 = dev2.step(workspace=None)
    assert np.array_equal(U.to_host(dev2.k_cache), kc) and np.array_equal(U.to_host(dev2.v_cache), vc)
    assert U.max_abs_err(got2, ref, dtype) <= U.TOL[dtype]


@pytest.mark.parametrize("dtype", [W.F16, W.BF16])
def test_decode_step_edge_lengths(U, oracle, dtype):
    """The new token is the only one (L = 1), first / last row of a block, last token of a full
    tile, and absent (L = 0: nothing written, +0 out) - all in one fused launch."""
    lens = np.array([0, 1, 15, 16, 17, 31, 32, 33, 255, 256, 257, 512, 1, 0, 300], np.int32)
    cfg = W.small_config(name="step_edges", dtype=dtype, batch=len(lens), num_heads=8, num_kv_heads=2,
                         head_dim=128, block_size=16, num_blocks=200, ctx_lo=1, ctx_hi=512, seed=421)
    case = W.make_case(cfg, context_lens=lens)
    full = lambda a, shape: (lambda z: (z.__setitem__(lens > 0, a), z)[1])(np.zeros(shape, np.uint16))
    q_full = full(case.q, (len(lens), 8, 128))
    k_full = full(case.k_new, (len(lens), 2, 128))
    v_full = full(case.v_new, (len(lens), 2, 128))
    kc, vc = oracle_filled(oracle, case)
    case.q = q_full
    ref = oracle_decode(oracle, case, kc, vc)
    dev = U.DevCase(case)
    dev.k_new, dev.v_new = U.to_dev(k_full, dtype), U.to_dev(v_full, dtype)
    got = dev.step()
    assert np.array_equal(U.to_host(dev.k_cache), kc) and np.array_equal(U.to_host(dev.v_cache), vc)
    assert not got[lens == 0].any()
    assert U.max_abs_err(got, ref, dtype) <= U.TOL[dtype]
    for b in (1, 12):                       # one-token context: the new V row, bit for bit
        for h in range(8):
            assert np.array_equal(got[b, h], v_full[b, h // 4])


def test_decode_step_strided_new_rows(U, oracle):
    """k_new / v_new as slices of a wider buffer: a stride that keeps 16-byte pieces (fused) and an
    odd one (separate narrow cache write); both must land the same bits."""
    import torch
    cfg = W.small_config(name="step_stride", dtype=W.BF16, batch=6, num_heads=16, num_kv_heads=4, head_dim=128,
                         block_size=32, num_blocks=6 * 20 + 3, ctx_lo=200, ctx_hi=600, seed=43)
    case = W.make_case(cfg)
    kc, vc = oracle_filled(oracle, case)
    ref = oracle_decode(oracle, case, kc, vc)
    for pad in (64, 3):
        dev = U.DevCase(case)
        wide_k = torch.zeros(6, 4 * 128 + pad, dtype=torch.bfloat16, device="cuda")
        wide_v = torch.zeros(6, 4 * 128 + pad, dtype=torch.bfloat16, device="cuda")
        wide_k[:, :512] = dev.k_new.reshape(6, 512)
        wide_v[:, :512] = dev.v_new.reshape(6, 512)
        dev.k_new = wide_k[:, :512].unflatten(1, (4, 128))
        dev.v_new = wide_v[:, :512].unflatten(1, (4, 128))
        got = dev.step()
        assert np.array_equal(U.to_host(dev.k_cache), kc) and np.array_equal(U.to_host(dev.v_cache), vc), pad
        assert U.max_abs_err(got, ref, W.BF16) <= U.TOL[W.BF16]


# ------------------------------------------------------------------ 8-bit (E4M3) KV cache
def fp8_caches(U, case, k_scale, v_scale):
    """Quantise the whole batch into 8-bit caches on both sides (oracle: numpy image; GPU: uint8
    tensors through optgqa_reshape_and_cache_fp8) from the same 2-byte rows and slots."""
    import torch
    import pins_e4m3
    import paper_2505_02351_amd as G
    kc8, vc8, (k_all, v_all, slots) = pins_e4m3.quantised_cache(case, k_scale, v_scale)
    dk = torch.full(kc8.shape, 0x7F, dtype=torch.uint8, device="cuda")
    dv = torch.full(vc8.shape, 0x7F, dtype=torch.uint8, device="cuda")
    G.reshape_and_cache_fp8(U.to_dev(k_all, case.dtype), U.to_dev(v_all, case.dtype), dk, dv,
                            torch.from_numpy(slots).cuda(), k_scale, v_scale)
    torch.cuda.synchronize()
    return kc8, vc8, dk, dv


def fp8_decode(U, case, dk, dv, k_scale, v_scale, q=None):
    import torch
    import paper_2505_02351_amd as G
    c = case.cfg
    qd = U.to_dev(case.q if q is None else q, case.dtype)
    g_out = U.Guarded(qd.numel() * qd.element_size())
    out = g_out.view(qd.dtype, qd.shape)
    out.fill_(float("nan"))
    n, _ = G.paged_attention_workspace_bytes(qd.shape[0], c.num_heads, c.num_kv_heads, c.head_dim, c.block_size,
                                             max(case.max_context_len, 1), G.SPLIT_BALANCED)
    g_ws = U.Guarded(n)
    G.paged_attention_fp8(out, qd, dk, dv, torch.from_numpy(case.block_tables).cuda(),
                          torch.from_numpy(case.context_lens).cuda(), torch.from_numpy(case.slopes).cuda(),
                          float(case.scale), k_scale, v_scale, case.max_context_len, g_ws.view(torch.float32))
    torch.cuda.synchronize()
    assert g_out.intact() and g_ws.intact(), "a kernel wrote outside out or the workspace"
    return U.to_host(out)


@pytest.mark.parametrize("dtype", [W.F16, W.BF16])
def test_fp8_cache_write_every_input_pattern(U, oracle, dtype):
    """All 65 536 two-byte patterns (NaNs and infinities included) through the quantising cache
    write, at scales that exercise the subnormal codes, the normal range and saturation: the
    codes must equal the oracle's bit for bit."""
    import torch
    import oracle as O
    import paper_2505_02351_amd as G
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16).reshape(64, 8, 128)     # [T][Hkv][D]
    slots = np.random.default_rng(1).permutation(96)[:64].astype(np.int64)            # 6 blocks of 16
    slots[5] = -1                                                                       # one padding token
    for k_scale, v_scale in ((1.0, 0.013), (37.5, 2.0 ** -12), (3e-3, 1e4)):
        kc8 = np.full((6, 8, 16, 128), 0x7F, np.uint8)
        vc8 = np.full((6, 8, 16, 128), 0x7F, np.uint8)
        O.reshape_and_cache_e4m3(bits, bits, kc8, vc8, slots, k_scale, v_scale, dtype)
        dk = torch.full(kc8.shape, 0x7F, dtype=torch.uint8, device="cuda")
        dv = torch.full(vc8.shape, 0x7F, dtype=torch.uint8, device="cuda")
        G.reshape_and_cache_fp8(U.to_dev(bits, dtype), U.to_dev(bits, dtype), dk, dv, torch.from_numpy(slots).cuda(),
                                k_scale, v_scale)
        torch.cuda.synchronize()
        assert np.array_equal(dk.cpu().numpy(), kc8), (dtype, k_scale)
        assert np.array_equal(dv.cpu().numpy(), vc8), (dtype, v_scale)


FP8_SWEEP = list(range(len(SWEEP)))


@pytest.mark.parametrize("i", FP8_SWEEP)
def test_fp8_decode_sweep(U, oracle, i):
    import oracle as O
    dtype, Hq, Hkv, D, bs, B, lo, hi = SWEEP[i]
    cfg = W.small_config(name=f"fp8_{i}", dtype=dtype, batch=B, num_heads=Hq, num_kv_heads=Hkv,
                         head_dim=D, block_size=bs, num_blocks=B * ((hi + bs - 1) // bs) + 7, ctx_lo=lo,
                         ctx_hi=hi, seed=900 + i)
    case = W.make_case(cfg)
    k_scale, v_scale = 0.0125, 0.02                     # N(0,1) data: the format's range covers +-5.6 / +-9 sigma
    kc8, vc8, dk, dv = fp8_caches(U, case, k_scale, v_scale)
    assert np.array_equal(dk.cpu().numpy(), kc8) and np.array_equal(dv.cpu().numpy(), vc8)
    got = fp8_decode(U, case, dk, dv, k_scale, v_scale)
    ref = O.paged_attention_e4m3(case.q, kc8, vc8, case.block_tables, case.context_lens, case.slopes, case.scale,
                                 k_scale, v_scale, dtype)
    err = U.max_abs_err(got, ref, dtype)
    assert err <= U.TOL[dtype], f"max abs err {err}"


@pytest.mark.parametrize("dtype", [W.F16, W.BF16])
def test_fp8_every_code_through_decode_and_prefill(U, oracle, dtype):
    """Caches of uniformly random bytes (every finite E4M3 code, subnormals and +-448 included, many
    times in K and in V; the two NaN codes replaced) read by the decode and the prefill kernels: the
    widening of codes on the device must agree with the oracle's decoder for all of them."""
    import torch
    import oracle as O
    import paper_2505_02351_amd as G
    cfg = W.small_config(name="fp8_codes", kind="prefill", dtype=dtype, batch=3, num_heads=8, num_kv_heads=2,
                         head_dim=128, block_size=16, num_blocks=60, ctx_lo=40, ctx_hi=300, q_len=37, seed=431)
    case = W.make_case(cfg)
    rng = np.random.default_rng(432)
    shape = (cfg.num_blocks, cfg.num_kv_heads, cfg.block_size, cfg.head_dim)
    kc8 = rng.integers(0, 256, size=shape, dtype=np.uint8)
    vc8 = rng.integers(0, 256, size=shape, dtype=np.uint8)
    kc8[(kc8 & 0x7F) == 0x7F] = 0x7E
    vc8[(vc8 & 0x7F) == 0x7F] = 0x7E
    for c in (kc8, vc8):
        assert len(np.unique(c)) == 254
    k_scale, v_scale = 0.002, 0.004                      # scores of a few units, outputs below 2
    dk, dv = torch.from_numpy(kc8).cuda(), torch.from_numpy(vc8).cuda()
    tables, lens = torch.from_numpy(case.block_tables).cuda(), torch.from_numpy(case.context_lens).cuda()
    slopes = torch.from_numpy(case.slopes).cuda()
    # prefill: every new token against its causal context
    qd = U.to_dev(case.q, dtype)
    out = torch.full_like(qd, float("nan"))
    G.paged_prefill_fp8(out, qd, dk, dv, tables, lens, torch.from_numpy(case.cu_q_lens).cuda(), slopes,
                        float(case.scale), k_scale, v_scale, case.max_q_len)
    torch.cuda.synchronize()
    ref = O.paged_prefill_e4m3(case.q, kc8, vc8, case.block_tables, case.context_lens, case.cu_q_lens,
                               case.slopes, case.scale, k_scale, v_scale, dtype)
    U.check_scaled(U.to_host(out), ref, dtype, "prefill over random codes")
    # decode: the last new token of every sequence as the query of a decode call
    last = case.cu_q_lens[1:] - 1
    q_dec = case.q[last]
    qd = U.to_dev(q_dec, dtype)
    out = torch.full_like(qd, float("nan"))
    n, _ = G.paged_attention_workspace_bytes(cfg.batch, cfg.num_heads, cfg.num_kv_heads, cfg.head_dim, cfg.block_size,
                                             case.max_context_len, G.SPLIT_BALANCED)
    ws = torch.empty(n // 4, dtype=torch.float32, device="cuda")
    G.paged_attention_fp8(out, qd, dk, dv, tables, lens, slopes, float(case.scale), k_scale, v_scale,
                          case.max_context_len, ws)
    torch.cuda.synchronize()
    ref_dec = O.paged_attention_e4m3(q_dec, kc8, vc8, case.block_tables, case.context_lens, case.slopes, case.scale,
                                     k_scale, v_scale, dtype)
    U.check_scaled(U.to_host(out), ref_dec, dtype, "decode over random codes")
    # the two clauses agree on those rows (same keys, same position)
    np.testing.assert_allclose(ref_dec, ref[last], rtol=1e-9, atol=1e-12)


@pytest.mark.parametrize("dtype", [W.F16, W.BF16])
def test_fp8_decode_edge_lengths(U, oracle, dtype):
    import oracle as O
    lens = np.array([0, 1, 15, 16, 17, 31, 32, 33, 255, 256, 257, 512, 1, 0], np.int32)
    cfg = W.small_config(name="fp8_edges", dtype=dtype, batch=len(lens), num_heads=8, num_kv_heads=2,
                         head_dim=128, block_size=16, num_blocks=180, ctx_lo=1, ctx_hi=512, seed=422)
    case = W.make_case(cfg, context_lens=lens)
    q_full = np.zeros((len(lens), 8, 128), np.uint16)
    q_full[lens > 0] = case.q
    # the generator's new-token rows exist for non-empty sequences only; rebuild the case's views
    case.q = q_full
    k_scale, v_scale = 0.02, 0.5
    kc8, vc8, dk, dv = fp8_caches(U, case, k_scale, v_scale)
    assert np.array_equal(dk.cpu().numpy(), kc8) and np.array_equal(dv.cpu().numpy(), vc8)
    got = fp8_decode(U, case, dk, dv, k_scale, v_scale)
    ref = O.paged_attention_e4m3(case.q, kc8, vc8, case.block_tables, case.context_lens, case.slopes, case.scale,
                                 k_scale, v_scale, dtype)
    assert not got[lens == 0].any()
    assert U.max_abs_err(got, ref, dtype) <= U.TOL[dtype]
    # one-token contexts: weight exactly 1, so the output is v_scale * value(code), rounded once
    vals = O.e4m3_values()
    for b in (1, 12):
        blk = case.block_tables[b, 0]
        for h in range(8):
            want = W.to_bits((v_scale * vals[vc8[blk, h // 4, 0, :]]).astype(np.float32), dtype)
            assert np.array_equal(got[b, h], want)


def test_fp8_decode_workload_full(U, oracle):
    """The bench's batch (C3 shapes) with 8-bit caches, every output row against the oracle."""
    import oracle as O
    case = workload_case("C3")
    k_scale, v_scale = 0.0125, 0.0125
    kc8, vc8, dk, dv = fp8_caches(U, case, k_scale, v_scale)
    assert np.array_equal(dk.cpu().numpy(), kc8) and np.array_equal(dv.cpu().numpy(), vc8)
    got = fp8_decode(U, case, dk, dv, k_scale, v_scale)
    ref = O.paged_attention_e4m3(case.q, kc8, vc8, case.block_tables, case.context_lens, case.slopes, case.scale,
                                 k_scale, v_scale, case.dtype)
    U.check_scaled(got, ref, case.dtype, "C3, E4M3 caches", max_exempt=WORKLOAD_EXEMPT)


@pytest.mark.parametrize("i", [0, 1, 2, 3, 4, 6, 8, 9, 10, 11, 12])
def test_fp8_prefill(U, oracle, i):
    """Tiled prefill over 8-bit caches against the oracle's clause (the caches are filled by the
    quantising cache write on both sides, codes compared bit for bit first)."""
    import torch
    import oracle as O
    import paper_2505_02351_amd as G
    dtype, Hq, Hkv, D, bs, B, lo, hi, qlen = PF[i]
    cfg = W.small_config(name=f"fp8pf{i}", kind="prefill", dtype=dtype, batch=B, num_heads=Hq, num_kv_heads=Hkv,
                         head_dim=D, block_size=bs, num_blocks=B * ((hi + bs - 1) // bs) + 5, ctx_lo=lo,
                         ctx_hi=hi, q_len=qlen, seed=950 + i)
    case = W.make_case(cfg)
    k_scale, v_scale = 0.0125, 0.02
    kc8, vc8, dk, dv = fp8_caches(U, case, k_scale, v_scale)
    assert np.array_equal(dk.cpu().numpy(), kc8) and np.array_equal(dv.cpu().numpy(), vc8)
    qd = U.to_dev(case.q, dtype)
    out = torch.full_like(qd, float("nan"))
    G.paged_prefill_fp8(out, qd, dk, dv, torch.from_numpy(case.block_tables).cuda(),
                        torch.from_numpy(case.context_lens).cuda(), torch.from_numpy(case.cu_q_lens).cuda(),
                        torch.from_numpy(case.slopes).cuda(), float(case.scale), k_scale, v_scale, case.max_q_len)
    torch.cuda.synchronize()
    ref = O.paged_prefill_e4m3(case.q, kc8, vc8, case.block_tables, case.context_lens, case.cu_q_lens,
                               case.slopes, case.scale, k_scale, v_scale, dtype)
    # (v_scale 0.02 puts V elements up to 9: rows that see one or two keys can land in [4, 8), where
    # the output's own rounding is twice the budget of the stated tolerance)
    U.check_scaled(U.to_host(out), ref, dtype, f"fp8 prefill {i}")


def test_fp8_prefill_workload_full(U, oracle):
    """The prefill workload (8 sequences, 512 new tokens after 2048 cached ones) over 8-bit caches,
    every output row against the oracle."""
    import torch
    import oracle as O
    import paper_2505_02351_amd as G
    case = workload_case("C5")
    k_scale, v_scale = 0.0125, 0.0125
    kc8, vc8, dk, dv = fp8_caches(U, case, k_scale, v_scale)
    assert np.array_equal(dk.cpu().numpy(), kc8) and np.array_equal(dv.cpu().numpy(), vc8)
    qd = U.to_dev(case.q, case.dtype)
    out = torch.full_like(qd, float("nan"))
    G.paged_prefill_fp8(out, qd, dk, dv, torch.from_numpy(case.block_tables).cuda(),
                        torch.from_numpy(case.context_lens).cuda(), torch.from_numpy(case.cu_q_lens).cuda(),
                        torch.from_numpy(case.slopes).cuda(), float(case.scale), k_scale, v_scale, case.max_q_len)
    torch.cuda.synchronize()
    ref = O.paged_prefill_e4m3(case.q, kc8, vc8, case.block_tables, case.context_lens, case.cu_q_lens,
                               case.slopes, case.scale, k_scale, v_scale, case.dtype)
    U.check_scaled(U.to_host(out), ref, case.dtype, "C5, E4M3 caches", max_exempt=WORKLOAD_EXEMPT)


@pytest.mark.parametrize("i", range(len(SWEEP)))
def test_fp8_decode_step_sweep(U, oracle, i):
    """optgqa_decode_step_fp8 on the sweep shapes: caches holding every token but the
    step's are quantised first; after the call the caches must equal the oracle's quantised image
    of the whole batch bit for bit and the output its E4M3 attention clause."""
    import torch
    import oracle as O
    import paper_2505_02351_amd as G
    dtype, Hq, Hkv, D, bs, B, lo, hi = SWEEP[i]
    cfg = W.small_config(name=f"fp8step{i}", dtype=dtype, batch=B, num_heads=Hq, num_kv_heads=Hkv, head_dim=D,
                         block_size=bs, num_blocks=B * ((hi + bs - 1) // bs) + 7, ctx_lo=lo, ctx_hi=hi, seed=1900 + i)
    case = W.make_case(cfg)
    k_scale, v_scale = 0.0125, 0.03
    kc8, vc8, _ = __import__("pins_e4m3").quantised_cache(case, k_scale, v_scale)       # all tokens, oracle side
    k_old, v_old, slots_old = W.all_token_rows(case, include_new=False)
    dk = torch.full(kc8.shape, 0x7F, dtype=torch.uint8, device="cuda")
    dv = torch.full(vc8.shape, 0x7F, dtype=torch.uint8, device="cuda")
    if len(slots_old):
        G.reshape_and_cache_fp8(U.to_dev(k_old, dtype), U.to_dev(v_old, dtype), dk, dv,
                                torch.from_numpy(slots_old).cuda(), k_scale, v_scale)
    dev = U.DevCase(case)
    ws = dev.workspace(BALANCED)[0]
    for window_free in (True,):
        dev.out.fill_(float("nan"))
        G.decode_step_fp8(dev.out, dev.q, dev.k_new, dev.v_new, dk, dv, dev.block_tables, dev.context_lens, dev.slopes,
                          float(case.scale), k_scale, v_scale, case.max_context_len, ws)
        torch.cuda.synchronize()
        dev.check_canaries()
    assert np.array_equal(dk.cpu().numpy(), kc8) and np.array_equal(dv.cpu().numpy(), vc8)
    ref = O.paged_attention_e4m3(case.q, kc8, vc8, case.block_tables, case.context_lens, case.slopes, case.scale,
                                 k_scale, v_scale, dtype)
    err = U.max_abs_err(U.to_host(dev.out), ref, dtype)
    assert err <= U.TOL[dtype], err


@pytest.mark.parametrize("dtype", [W.F16, W.BF16])
def test_fp8_decode_step_edge_lengths(U, oracle, dtype):
    """The new token alone (L = 1: nothing is streamed, the combine kernel does it all), first / last
    row of a block, absent sequences (L = 0), more than 64 sequences."""
    import torch
    import oracle as O
    import paper_2505_02351_amd as G
    import pins_e4m3
    lens = np.array([0, 1, 15, 16, 17, 31, 32, 33, 255, 256, 257, 512, 1, 0, 300, 1, 1, 2] * 4, np.int32)
    cfg = W.small_config(name="fp8step_edges", dtype=dtype, batch=len(lens), num_heads=8, num_kv_heads=2,
                         head_dim=128, block_size=16, num_blocks=len(lens) * 33, ctx_lo=1, ctx_hi=512, seed=1921)
    case = W.make_case(cfg, context_lens=lens)
    full = lambda a, shape: (lambda z: (z.__setitem__(lens > 0, a), z)[1])(np.zeros(shape, np.uint16))
    q_full = full(case.q, (len(lens), 8, 128))
    k_full = full(case.k_new, (len(lens), 2, 128))
    v_full = full(case.v_new, (len(lens), 2, 128))
    k_scale, v_scale = 0.02, 0.0125
    kc8, vc8, _ = pins_e4m3.quantised_cache(case, k_scale, v_scale)
    k_old, v_old, slots_old = W.all_token_rows(case, include_new=False)
    dk = torch.full(kc8.shape, 0x7F, dtype=torch.uint8, device="cuda")
    dv = torch.full(vc8.shape, 0x7F, dtype=torch.uint8, device="cuda")
    G.reshape_and_cache_fp8(U.to_dev(k_old, dtype), U.to_dev(v_old, dtype), dk, dv, torch.from_numpy(slots_old).cuda(),
                            k_scale, v_scale)
    case.q = q_full
    dev = U.DevCase(case)
    dev.k_new, dev.v_new = U.to_dev(k_full, dtype), U.to_dev(v_full, dtype)
    ws = dev.workspace(BALANCED)[0]
    dev.out.fill_(float("nan"))
    G.decode_step_fp8(dev.out, dev.q, dev.k_new, dev.v_new, dk, dv, dev.block_tables, dev.context_lens, dev.slopes,
                      float(case.scale), k_scale, v_scale, case.max_context_len, ws)
    torch.cuda.synchronize()
    dev.check_canaries()
    assert np.array_equal(dk.cpu().numpy(), kc8) and np.array_equal(dv.cpu().numpy(), vc8)
    ref = O.paged_attention_e4m3(case.q, kc8, vc8, case.block_tables, case.context_lens, case.slopes, case.scale,
                                 k_scale, v_scale, dtype)
    got = U.to_host(dev.out)
    assert U.max_abs_err(got, ref, dtype) <= U.TOL[dtype]
    assert not got[lens == 0].any()


HEAD_SCALES = [
    # dtype, Hq, Hkv, bs, batch, ctx_lo, ctx_hi, new tokens per sequence, head_dim
    (W.BF16, 32, 4, 32, 5, 40, 900, 1, 128),
    (W.F16, 12, 3, 16, 4, 1, 500, 1, 128),           # G = 4, three KV heads
    (W.BF16, 8, 8, 16, 3, 100, 400, 37, 128),        # MHA, a prefill chunk
    (W.F16, 16, 2, 64, 2, 200, 700, 130, 128),       # G = 8, prefill
    (W.F16, 8, 2, 16, 4, 1, 600, 1, 64),             # head_dim 64, G = 4
    (W.BF16, 16, 4, 32, 3, 100, 500, 70, 64),        # head_dim 64, prefill
]


@pytest.mark.parametrize("i", range(len(HEAD_SCALES)))
def test_fp8_per_head_scales(U, oracle, i):
    """8-bit caches with one scale pair per KV head (scales spread over four orders of magnitude):
    quantising cache write bit for bit, then - one new token per sequence - the decode call and the
    one-call decode step (caches bit for bit again), or - a chunk of new tokens - the prefill, each
    against the oracle's per-head clause."""
    import torch
    import oracle as O
    import paper_2505_02351_amd as G
    dtype, Hq, Hkv, bs, B, lo, hi, q_len, D = HEAD_SCALES[i]
    kind = "decode" if q_len == 1 else "prefill"
    cfg = W.small_config(name=f"fp8heads{i}", kind=kind, dtype=dtype, batch=B, num_heads=Hq, num_kv_heads=Hkv,
                         head_dim=D, block_size=bs, num_blocks=B * ((hi + bs - 1) // bs) + 7, ctx_lo=lo, ctx_hi=hi,
                         q_len=q_len, seed=2700 + i)
    case = W.make_case(cfg)
    rng = np.random.default_rng(2800 + i)
    k_scales = (0.0125 * np.exp2(rng.integers(-3, 4, size=Hkv))).astype(np.float32)
    v_scales = (0.02 * np.exp2(rng.uniform(-6, 6, size=Hkv))).astype(np.float32)       # not powers of two
    shape = (cfg.num_blocks, Hkv, bs, D)
    k_all, v_all, slots = W.all_token_rows(case)
    kc8, vc8 = np.full(shape, 0x7F, np.uint8), np.full(shape, 0x7F, np.uint8)
    O.reshape_and_cache_e4m3_heads(k_all, v_all, kc8, vc8, slots, k_scales, v_scales, dtype)
    ks_d, vs_d = torch.from_numpy(k_scales).cuda(), torch.from_numpy(v_scales).cuda()
    dk = torch.full(shape, 0x7F, dtype=torch.uint8, device="cuda")
    dv = torch.full(shape, 0x7F, dtype=torch.uint8, device="cuda")
    G.reshape_and_cache_fp8_heads(U.to_dev(k_all, dtype), U.to_dev(v_all, dtype), dk, dv, torch.from_numpy(slots).cuda(),
                                  ks_d, vs_d)
    torch.cuda.synchronize()
    assert np.array_equal(dk.cpu().numpy(), kc8) and np.array_equal(dv.cpu().numpy(), vc8)
    dev = U.DevCase(case)
    if kind == "decode":
        ref = O.paged_attention_e4m3_heads(case.q, kc8, vc8, case.block_tables, case.context_lens, case.slopes,
                                           case.scale, k_scales, v_scales, dtype)
        ws = dev.workspace(BALANCED)[0]
        dev.out.fill_(float("nan"))
        G.paged_attention_fp8_heads(dev.out, dev.q, dk, dv, dev.block_tables, dev.context_lens, dev.slopes,
                                    float(case.scale), ks_d, vs_d, case.max_context_len, ws)
        torch.cuda.synchronize()
        dev.check_canaries()
        U.check_scaled(U.to_host(dev.out), ref, dtype, f"per-head scales {i}, decode")
        # the one-call step: wipe the new tokens' rows, the step has to put the same codes back
        s_ = torch.from_numpy(case.slot_mapping).cuda()
        dk[s_ // bs, :, s_ % bs, :] = 0x7F
        dv[s_ // bs, :, s_ % bs, :] = 0x7F
        ws = dev.workspace(BALANCED)[0]
        dev.out.fill_(float("nan"))
        G.decode_step_fp8_heads(dev.out, dev.q, dev.k_new, dev.v_new, dk, dv, dev.block_tables, dev.context_lens,
                                dev.slopes, float(case.scale), ks_d, vs_d, case.max_context_len, ws)
        torch.cuda.synchronize()
        dev.check_canaries()
        assert np.array_equal(dk.cpu().numpy(), kc8) and np.array_equal(dv.cpu().numpy(), vc8)
        U.check_scaled(U.to_host(dev.out), ref, dtype, f"per-head scales {i}, decode step")
    else:
        ref = O.paged_prefill_e4m3_heads(case.q, kc8, vc8, case.block_tables, case.context_lens, case.cu_q_lens,
                                         case.slopes, case.scale, k_scales, v_scales, dtype)
        dev.out.fill_(float("nan"))
        G.paged_prefill_fp8_heads(dev.out, dev.q, dk, dv, dev.block_tables, dev.context_lens, dev.cu_q_lens,
                                  dev.slopes, float(case.scale), ks_d, vs_d, case.max_q_len)
        torch.cuda.synchronize()
        dev.check_canaries()
        U.check_scaled(U.to_host(dev.out), ref, dtype, f"per-head scales {i}, prefill")


@pytest.mark.parametrize("dtype", [W.F16, W.BF16])
def test_fp8_per_head_cache_write_every_input_pattern(U, oracle, dtype):
    """All 65 536 two-byte patterns through the quantising cache write with a different scale per KV
    head (eight heads: subnormal codes, the normal range, saturation): codes bit for bit."""
    import torch
    import oracle as O
    import paper_2505_02351_amd as G
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16).reshape(64, 8, 128)     # [T][Hkv][D]
    slots = np.random.default_rng(2).permutation(96)[:64].astype(np.int64)
    k_scales = np.array([1.0, 37.5, 3e-3, 0.013, 2.0 ** -12, 1e4, 0.7, 5.0], np.float32)
    v_scales = k_scales[::-1].copy()
    kc8 = np.full((6, 8, 16, 128), 0x7F, np.uint8)
    vc8 = np.full((6, 8, 16, 128), 0x7F, np.uint8)
    O.reshape_and_cache_e4m3_heads(bits, bits, kc8, vc8, slots, k_scales, v_scales, dtype)
    dk = torch.full(kc8.shape, 0x7F, dtype=torch.uint8, device="cuda")
    dv = torch.full(vc8.shape, 0x7F, dtype=torch.uint8, device="cuda")
    G.reshape_and_cache_fp8_heads(U.to_dev(bits, dtype), U.to_dev(bits, dtype), dk, dv, torch.from_numpy(slots).cuda(),
                                  torch.from_numpy(k_scales).cuda(), torch.from_numpy(v_scales).cuda())
    torch.cuda.synchronize()
    assert np.array_equal(dk.cpu().numpy(), kc8)
    assert np.array_equal(dv.cpu().numpy(), vc8)


def test_fp8_rejects_what_it_cannot_do(U):
    import torch
    import paper_2505_02351_amd as G
    q = torch.zeros(2, 8, 64, dtype=torch.float16, device="cuda")
    c8 = torch.zeros(4, 2, 16, 64, dtype=torch.uint8, device="cuda")
    bt = torch.zeros(2, 2, dtype=torch.int32, device="cuda")
    cl = torch.ones(2, dtype=torch.int32, device="cuda")
    ws = torch.empty(1 << 20, dtype=torch.float32, device="cuda")
    cu = torch.tensor([0, 1, 2], dtype=torch.int32, device="cuda")
    q96 = torch.zeros(2, 8, 96, dtype=torch.float16, device="cuda")
    c96 = torch.zeros(4, 2, 16, 96, dtype=torch.uint8, device="cuda")
    with pytest.raises(RuntimeError):                    # head_dim 96
        G.paged_attention_fp8(torch.empty_like(q96), q96, c96, c96, bt, cl, None, 0.1, 1.0, 1.0, 32, ws)
    with pytest.raises(RuntimeError):                    # head_dim 96, prefill
        G.paged_prefill_fp8(torch.empty_like(q96), q96, c96, c96, bt, cl, cu, None, 0.1, 1.0, 1.0, 1)
    q = torch.zeros(2, 8, 128, dtype=torch.float16, device="cuda")
    c8 = torch.zeros(4, 2, 16, 128, dtype=torch.uint8, device="cuda")
    with pytest.raises(RuntimeError):                    # no workspace
        G.paged_attention_fp8(torch.empty_like(q), q, c8, c8, bt, cl, None, 0.1, 1.0, 1.0, 32, None)
    with pytest.raises(RuntimeError):                    # scale must be positive
        G.paged_attention_fp8(torch.empty_like(q), q, c8, c8, bt, cl, None, 0.1, 0.0, 1.0, 32, ws)


# ------------------------------------------------------------------ sliding window (local mask)
WINDOWS = [1, 2, 15, 16, 17, 33, 100, 257, 10 ** 6]


@pytest.mark.parametrize("i", range(len(SWEEP)))
def test_decode_window_sweep(U, oracle, i):
    """Windowed decode against the oracle's local-mask clause, every window of WINDOWS on the sweep
    shapes, both over filled caches and
    with the cache write in the same call (caches bit-exact); without slopes on one pass (Alg. 1
    builds the local mask when there are none)."""
    import oracle as O
    dtype, Hq, Hkv, D, bs, B, lo, hi = SWEEP[i]
    cfg = W.small_config(name=f"win{i}", dtype=dtype, batch=B, num_heads=Hq, num_kv_heads=Hkv,
                         head_dim=D, block_size=bs, num_blocks=B * ((hi + bs - 1) // bs) + 7, ctx_lo=lo,
                         ctx_hi=hi, seed=1400 + i)
    case = W.make_case(cfg)
    kc, vc = oracle_filled(oracle, case)
    dev = U.DevCase(case)
    dev.write_cache()
    for window in WINDOWS:
        ref = O.paged_attention_window(case.q, kc, vc, case.block_tables, case.context_lens, case.slopes, case.scale,
                                       window, dtype)
        err = U.max_abs_err(dev.decode_window(window), ref, dtype)
        assert err <= U.TOL[dtype], f"window {window}: {err}"
        fresh = U.DevCase(case)
        err = U.max_abs_err(fresh.decode_window(window, fused=True), ref, dtype)
        assert err <= U.TOL[dtype], f"window {window}, fused step: {err}"
        assert np.array_equal(U.to_host(fresh.k_cache), kc) and np.array_equal(U.to_host(fresh.v_cache), vc)
    ref = O.paged_attention_window(case.q, kc, vc, case.block_tables, case.context_lens, None, case.scale, 40, dtype)
    assert U.max_abs_err(dev.decode_window(40, slopes=None), ref, dtype) <= U.TOL[dtype]


@pytest.mark.parametrize("dtype", [W.F16, W.BF16])
def test_decode_window_edge_lengths(U, oracle, dtype):
    """Windows that start on / next to tile and block boundaries, contexts shorter than the window,
    empty sequences, and a batch of more than 64 sequences (two-level scan) in one launch."""
    import oracle as O
    lens = np.array([0, 1, 15, 16, 17, 31, 32, 33, 48, 49, 63, 64, 65, 255, 256, 257, 512, 1, 0, 300] * 4, np.int32)
    cfg = W.small_config(name="win_edges", dtype=dtype, batch=len(lens), num_heads=8, num_kv_heads=2,
                         head_dim=128, block_size=16, num_blocks=len(lens) * 33, ctx_lo=1, ctx_hi=512, seed=1421)
    case = W.make_case(cfg, context_lens=lens)
    full = lambda a, shape: (lambda z: (z.__setitem__(lens > 0, a), z)[1])(np.zeros(shape, np.uint16))
    q_full = full(case.q, (len(lens), 8, 128))
    k_full = full(case.k_new, (len(lens), 2, 128))
    v_full = full(case.v_new, (len(lens), 2, 128))
    kc, vc = oracle_filled(oracle, case)
    case.q = q_full
    for window in (1, 16, 17, 32, 48, 250):
        ref = O.paged_attention_window(case.q, kc, vc, case.block_tables, case.context_lens, case.slopes, case.scale,
                                       window, dtype)
        dev = U.DevCase(case)
        dev.k_new, dev.v_new = U.to_dev(k_full, dtype), U.to_dev(v_full, dtype)
        got = dev.decode_window(window, fused=True)
        assert np.array_equal(U.to_host(dev.k_cache), kc) and np.array_equal(U.to_host(dev.v_cache), vc)
        assert U.max_abs_err(got, ref, dtype) <= U.TOL[dtype], window
        assert not got[lens == 0].any()
        got = dev.decode_window(window)                      # caches now filled: the plain windowed call
        assert U.max_abs_err(got, ref, dtype) <= U.TOL[dtype], window


@pytest.mark.parametrize("window", [1024, 4096])
def test_decode_window_workload_full(U, oracle, window):
    """The decode workload (batch 64, contexts 1k..8k) with a sliding window, cache write in the
    same call: caches bit-exact, every output row against the oracle."""
    import oracle as O
    case = workload_case("C3")
    dev = U.DevCase(case)
    got = dev.decode_window(window, fused=True)
    kc, vc = oracle_filled(oracle, case)
    assert np.array_equal(U.to_host(dev.k_cache), kc) and np.array_equal(U.to_host(dev.v_cache), vc)
    ref = O.paged_attention_window(case.q, kc, vc, case.block_tables, case.context_lens, case.slopes, case.scale,
                                   window, case.dtype)
    U.check_scaled(got, ref, case.dtype, f"C3, window {window}", max_exempt=WORKLOAD_EXEMPT)


@pytest.mark.parametrize("i", range(10))
def test_prefill_window_sweep(U, oracle, i):
    import oracle as O
    dtype, Hq, Hkv, D, bs, B, lo, hi, q_len = PF[i]
    cfg = W.small_config(name=f"pfwin{i}", kind="prefill", dtype=dtype, batch=B, num_heads=Hq, num_kv_heads=Hkv,
                         head_dim=D, block_size=bs, num_blocks=B * ((hi + bs - 1) // bs) + 5, ctx_lo=lo,
                         ctx_hi=hi, q_len=q_len, seed=1500 + i)
    case = W.make_case(cfg)
    dev = U.DevCase(case)
    dev.write_cache()
    kc, vc = oracle_filled(oracle, case)
    for window in (1, 7, 31, 32, 33, 64, 150, 10 ** 6):
        ref = O.paged_prefill_window(case.q, kc, vc, case.block_tables, case.context_lens, case.cu_q_lens,
                                     case.slopes, case.scale, window, dtype)
        err = U.max_abs_err(dev.prefill_window(window), ref, dtype)
        assert err <= U.TOL[dtype], f"window {window}: {err}"
    ref = O.paged_prefill_window(case.q, kc, vc, case.block_tables, case.context_lens, case.cu_q_lens, None,
                                 case.scale, 20, dtype)
    assert U.max_abs_err(dev.prefill_window(20, slopes=None), ref, dtype) <= U.TOL[dtype]


def test_prefill_window_workload_full(U, oracle):
    """The prefill workload with a 512-key window, every output row against the oracle."""
    import oracle as O
    case = workload_case("C5")
    dev = U.DevCase(case)
    dev.write_cache()
    kc, vc = oracle_filled(oracle, case)
    got = dev.prefill_window(512)
    ref = O.paged_prefill_window(case.q, kc, vc, case.block_tables, case.context_lens, case.cu_q_lens,
                                 case.slopes, case.scale, 512, case.dtype)
    U.check_scaled(got, ref, case.dtype, "C5, window 512", max_exempt=WORKLOAD_EXEMPT)


@pytest.mark.parametrize("dtype", [W.F16, W.BF16])
def test_prefill_with_scores_far_below_zero(U, oracle, dtype):
    """Every score of every row strongly negative (queries opposed to all keys): the softmax
    reference has to follow the first visible keys down, or the 16-bit weights underflow."""
    cfg = W.small_config(name="pfneg", kind="prefill", dtype=dtype, batch=2, num_heads=8, num_kv_heads=2,
                         head_dim=128, block_size=16, num_blocks=64, ctx_lo=100, ctx_hi=300, q_len=70, seed=1600)
    case = W.make_case(cfg)
    kc, vc = oracle_filled(oracle, case)
    # keys share a strong common component c; queries point along -c
    rng = np.random.default_rng(5)
    c = rng.standard_normal(128).astype(np.float32)
    kf = W.from_bits(kc, dtype).astype(np.float32)
    kf = np.nan_to_num(kf) * 0.3 + c
    kc = W.to_bits(kf, dtype)
    q = W.to_bits((W.from_bits(case.q, dtype).astype(np.float32) * 0.3 - 3.0 * c).astype(np.float32), dtype)
    import torch
    dev = U.DevCase(case)
    dev.k_cache = U.to_dev(kc, dtype)
    dev.v_cache = U.to_dev(vc, dtype)
    dev.q = U.to_dev(q, dtype)
    ref = oracle.paged_prefill(q, kc, vc, case.block_tables, case.context_lens, case.cu_q_lens, case.slopes,
                               case.scale, dtype)
    assert U.max_abs_err(dev.prefill(), ref, dtype) <= U.TOL[dtype]
    import oracle as O
    ref = O.paged_prefill_window(q, kc, vc, case.block_tables, case.context_lens, case.cu_q_lens, case.slopes,
                                 case.scale, 50, dtype)
    assert U.max_abs_err(dev.prefill_window(50), ref, dtype) <= U.TOL[dtype]


def test_window_rejects_what_it_cannot_do(U):
    import torch
    import paper_2505_02351_amd as G
    bt = torch.zeros(2, 2, dtype=torch.int32, device="cuda")
    cl = torch.ones(2, dtype=torch.int32, device="cuda")
    cu = torch.tensor([0, 1, 2], dtype=torch.int32, device="cuda")
    ws = torch.empty(1 << 20, dtype=torch.float32, device="cuda")
    q = torch.zeros(2, 8, 128, dtype=torch.float16, device="cuda")
    c = torch.zeros(4, 2, 16, 128, dtype=torch.float16, device="cuda")
    with pytest.raises(RuntimeError):                    # head_dim 128 without a workspace
        G.paged_attention_window(torch.empty_like(q), q, c, c, bt, cl, None, 0.1, 8, 32, None)
    with pytest.raises(RuntimeError):                    # window must be positive
        G.paged_attention_window(torch.empty_like(q), q, c, c, bt, cl, None, 0.1, 0, 32, ws)
    with pytest.raises(RuntimeError):
        G.paged_prefill_window(torch.empty_like(q), q, c, c, bt, cl, cu, None, 0.1, 0, 1)


# ------------------------------------------------------------------ whole prompt, caches empty
PROMPT = [
    # dtype, Hq, Hkv, bs, batch, len_lo, len_hi[, head_dim]
    (W.BF16, 8, 2, 16, 3, 1, 300),
    (W.F16, 8, 2, 16, 3, 1, 300, 64),
    (W.BF16, 12, 4, 32, 2, 40, 500, 64),   # G = 3, head_dim 64
    (W.F16, 32, 8, 16, 2, 100, 700),
    (W.F16, 4, 4, 32, 3, 1, 400),          # MHA: 128 tokens per workgroup
    (W.BF16, 6, 2, 16, 2, 5, 100),         # G = 3
    (W.F16, 32, 2, 64, 2, 30, 260),        # G = 16: 8 tokens per workgroup
    (W.BF16, 40, 2, 16, 1, 200, 200),      # G = 20 -> two head chunks; only the first stores the rows
    # enough workgroups for the 8-wave form of the kernel:
    (W.BF16, 16, 8, 16, 32, 100, 300),     # G = 2: 128 tokens per workgroup
    (W.F16, 8, 8, 32, 64, 1, 300, 64),     # MHA, head_dim 64: 256 tokens per workgroup
]


@pytest.mark.parametrize("i", range(len(PROMPT)))
def test_prompt_prefill_sweep(U, oracle, i):
    """optgqa_prompt_prefill against the oracle's whole-prompt clause; the caches it fills must equal
    the cache-write oracle's bit for bit (untouched rows keep their fill pattern); K / V given as
    strided views of one fused [T, (Hq + 2 Hkv) D] tensor on one pass."""
    import torch
    import oracle as O
    import paper_2505_02351_amd as G
    dtype, Hq, Hkv, bs, B, lo, hi = PROMPT[i][:7]
    D = PROMPT[i][7] if len(PROMPT[i]) > 7 else 128
    cfg = W.small_config(name=f"prompt{i}", kind="prefill", dtype=dtype, batch=B, num_heads=Hq, num_kv_heads=Hkv,
                         head_dim=D, block_size=bs, num_blocks=B * ((hi + bs - 1) // bs) + 5, ctx_lo=lo,
                         ctx_hi=hi, q_len=hi, seed=1700 + i)
    case = W.make_case(cfg)
    assert np.array_equal(case.q_lens, case.context_lens)
    ref = O.prompt_attention(case.q, case.k_new, case.v_new, case.cu_q_lens, case.slopes, case.scale, dtype)
    kc, vc = oracle_filled(oracle, case)
    dev = U.DevCase(case)
    # dense inputs, caches stored
    dev.out.fill_(float("nan"))
    G.prompt_prefill(dev.out, dev.q, dev.k_new, dev.v_new, dev.k_cache, dev.v_cache, dev.block_tables, dev.cu_q_lens,
                     dev.slopes, float(case.scale), case.max_q_len)
    torch.cuda.synchronize()
    dev.check_canaries()
    # (binade-aware bound: the larger cases have tens of millions of V elements, a few of them beyond
    # 4, and a row that sees one or two keys can return such a value, rounded at twice the budget)
    U.check_scaled(U.to_host(dev.out), ref, dtype, f"prompt {i}")
    assert np.array_equal(U.to_host(dev.k_cache), kc) and np.array_equal(U.to_host(dev.v_cache), vc)
    # fused QKV tensor: k and v are strided views; no caches
    T = case.num_tokens
    fused = torch.zeros(T, (Hq + 2 * Hkv) * D, dtype=dev.q.dtype, device="cuda")
    fused[:, Hq * D:(Hq + Hkv) * D] = dev.k_new.reshape(T, Hkv * D)
    fused[:, (Hq + Hkv) * D:] = dev.v_new.reshape(T, Hkv * D)
    k_view = fused[:, Hq * D:(Hq + Hkv) * D].unflatten(1, (Hkv, D))
    v_view = fused[:, (Hq + Hkv) * D:].unflatten(1, (Hkv, D))
    dev.out.fill_(float("nan"))
    G.prompt_prefill(dev.out, dev.q, k_view, v_view, None, None, None, dev.cu_q_lens, None, float(case.scale),
                     case.max_q_len)
    torch.cuda.synchronize()
    ref = O.prompt_attention(case.q, case.k_new, case.v_new, case.cu_q_lens, None, case.scale, dtype)
    U.check_scaled(U.to_host(dev.out), ref, dtype, f"prompt {i}, fused input")


def test_prompt_prefill_then_decode(U, oracle):
    """A prompt processed by optgqa_prompt_prefill, then one decode step over the caches it filled:
    the step's output equals the oracle's decode over the oracle's caches."""
    import torch
    import paper_2505_02351_amd as G
    cfg = W.small_config(name="prompt_then_decode", dtype=W.BF16, batch=4, num_heads=16, num_kv_heads=4, head_dim=128,
                         block_size=16, num_blocks=4 * 40 + 3, ctx_lo=50, ctx_hi=600, seed=1750)
    case = W.make_case(cfg)                                        # decode case: last token is the step's
    k_all, v_all, slots = W.all_token_rows(case, include_new=False)
    lens = case.context_lens.astype(np.int64) - 1
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    dev = U.DevCase(case)
    dev.k_cache.fill_(float("nan")), dev.v_cache.fill_(float("nan"))
    T = int(cu[-1])
    qp = torch.zeros(T, 16, 128, dtype=dev.q.dtype, device="cuda")
    G.prompt_prefill(torch.empty_like(qp), qp, U.to_dev(k_all, W.BF16), U.to_dev(v_all, W.BF16), dev.k_cache,
                     dev.v_cache, dev.block_tables, torch.from_numpy(cu).cuda(), dev.slopes, float(case.scale),
                     int(lens.max()))
    got = dev.step()
    kc, vc = oracle_filled(oracle, case)
    ref = oracle_decode(oracle, case, kc, vc)
    assert U.max_abs_err(got, ref, W.BF16) <= U.TOL[W.BF16]


def test_prompt_prefill_workload_full(U, oracle):
    """Eight prompts of 2560 tokens at the prefill workload's head shapes: caches bit-exact, every
    output row against the oracle.  (Rows 1 and 2 of a prompt see two or three keys, so an output can
    exceed magnitude 4: the bound follows the output type's own rounding there and only there.)"""
    import torch
    import oracle as O
    import paper_2505_02351_amd as G
    case = workload_case("C5-prompt")
    dev = U.DevCase(case)
    dev.out.fill_(float("nan"))
    G.prompt_prefill(dev.out, dev.q, dev.k_new, dev.v_new, dev.k_cache, dev.v_cache, dev.block_tables, dev.cu_q_lens,
                     dev.slopes, float(case.scale), case.max_q_len)
    torch.cuda.synchronize()
    dev.check_canaries()
    got = U.to_host(dev.out)
    kc, vc = oracle_filled(oracle, case)
    assert np.array_equal(U.to_host(dev.k_cache), kc) and np.array_equal(U.to_host(dev.v_cache), vc)
    ref = O.prompt_attention(case.q, case.k_new, case.v_new, case.cu_q_lens, case.slopes, case.scale, case.dtype)
    U.check_scaled(got, ref, case.dtype, "C5-prompt", max_exempt=WORKLOAD_EXEMPT)


def test_prompt_prefill_rejects_what_it_cannot_do(U):
    import torch
    import paper_2505_02351_amd as G
    cu = torch.tensor([0, 2], dtype=torch.int32, device="cuda")
    q = torch.zeros(2, 8, 128, dtype=torch.float16, device="cuda")
    wide = torch.zeros(2, 2 * 128 + 4, dtype=torch.float16, device="cuda")
    kv = wide[:, :256].unflatten(1, (2, 128))            # token stride 260: not a multiple of 8
    with pytest.raises(RuntimeError):
        G.prompt_prefill(torch.empty_like(q), q, kv, kv, None, None, None, cu, None, 0.1, 2)


def test_decode_with_shared_prefix_blocks(U, oracle):
    """Block tables that alias each other (groups of sequences served from the same physical
    prefix blocks; Section III-B speaks of sharing and reusing cached blocks): nothing in the path assumes blocks are
    private, so the step must still match the oracle, which walks the same tables."""
    cfg = W.small_config(name="shared", dtype=W.BF16, batch=12, num_heads=16, num_kv_heads=4, head_dim=128,
                         block_size=16, num_blocks=12 * 64 + 7, ctx_lo=300, ctx_hi=1000, seed=2100)
    case = W.make_case(cfg)
    shared = W.share_prefix_blocks(case, group=4, fraction=0.9)
    assert shared > 0
    kc, vc = oracle_filled(oracle, case)
    ref = oracle_decode(oracle, case, kc, vc)
    dev = U.DevCase(case)
    got = dev.step()
    assert np.array_equal(U.to_host(dev.k_cache), kc) and np.array_equal(U.to_host(dev.v_cache), vc)
    assert U.max_abs_err(got, ref, W.BF16) <= U.TOL[W.BF16]
    assert U.max_abs_err(dev.decode(partition_size=256), ref, W.BF16) <= U.TOL[W.BF16]


SHARED = [
    # dtype, Hq, Hkv, bs, batch, ctx_lo, ctx_hi, head_dim   heads per pass -> bundle
    (W.BF16, 32, 4, 32, 10, 40, 900, 128),      # G = 8  -> pairs
    (W.F16, 32, 8, 16, 13, 20, 700, 128),       # G = 4  -> bundles of 4, last bundle incomplete
    (W.BF16, 8, 8, 16, 35, 1, 300, 128),        # G = 1  -> bundles of 16; 70 virtual sequences: two-level scan
    (W.F16, 12, 2, 16, 7, 30, 500, 128),        # G = 6  -> pairs, 12 of the 16 columns in use
    (W.BF16, 6, 2, 64, 11, 64, 700, 128),       # G = 3  -> bundles of 5 (15 columns), block 64
    (W.F16, 32, 2, 16, 4, 50, 400, 128),        # G = 16 -> bundle of 1: nothing can be shared
    (W.BF16, 16, 2, 16, 80, 1, 120, 128),       # G = 8, 80 sequences: 160 virtual sequences, many short
    (W.F16, 8, 2, 16, 9, 20, 600, 64),          # head_dim 64, G = 4 -> bundles of 4
    (W.BF16, 16, 2, 32, 6, 40, 500, 64),        # head_dim 64, G = 8 -> pairs
]


@pytest.mark.parametrize("i", range(len(SHARED)))
def test_decode_shared_prefix_sweep(U, oracle, i):
    """Shared prefixes read once per bundle (Section III-B): ragged numbers of shared blocks per
    member, members that share nothing, members whose whole cached context is shared, sequences of
    length 0 and 1.  The oracle knows nothing of sharing - it walks the aliased tables - and the
    plain and fused calls must both match it; the fused call's caches bit for bit."""
    import paper_2505_02351_amd as G
    dtype, Hq, Hkv, bs, B, lo, hi, D = SHARED[i]
    cfg = W.small_config(name=f"shared{i}", dtype=dtype, batch=B, num_heads=Hq, num_kv_heads=Hkv, head_dim=D,
                         block_size=bs, num_blocks=B * ((hi + bs - 1) // bs) + 7, ctx_lo=lo, ctx_hi=hi, seed=2400 + i)
    rng = np.random.default_rng(2500 + i)
    lens = rng.integers(lo, hi + 1, size=B).astype(np.int32)
    lens[rng.choice(B, size=max(B // 6, 1), replace=False)] = rng.choice([0, 1, bs, bs + 1, 2 * bs + 1])
    case = W.make_case(cfg, context_lens=lens)
    bundle = G.shared_prefix_bundle(Hq, Hkv, D)
    assert bundle == 16 // max(d for d in range(1, 17) if (Hq // Hkv) % d == 0)
    shared = W.share_prefix_in_bundles(case, bundle, seed=2600 + i)
    assert bundle == 1 or shared.any()
    assert G.validate_shared_prefix_host(case.block_tables, case.context_lens, shared, bs, bundle, 1) == 0
    full = lambda a, shape: (lambda z: (z.__setitem__(lens > 0, a), z)[1])(np.zeros(shape, np.uint16))
    q_full = full(case.q, (B, Hq, D))
    k_full, v_full = full(case.k_new, (B, Hkv, D)), full(case.v_new, (B, Hkv, D))
    kc, vc = oracle_filled(oracle, case)
    case.q = q_full
    ref = oracle_decode(oracle, case, kc, vc)
    dev = U.DevCase(case)
    dev.k_new, dev.v_new = U.to_dev(k_full, dtype), U.to_dev(v_full, dtype)
    got = dev.decode_shared(shared, fused=True)
    assert np.array_equal(U.to_host(dev.k_cache), kc) and np.array_equal(U.to_host(dev.v_cache), vc)
    assert not got[lens == 0].any()
    U.check_scaled(got, ref, dtype, f"shared prefixes {i}, fused step")
    got = dev.decode_shared(shared)                         # caches now filled: the plain call
    assert not got[lens == 0].any()
    U.check_scaled(got, ref, dtype, f"shared prefixes {i}, plain")
    # no sharing declared at all: the same kernel degenerates to the plain equal-work split
    got = dev.decode_shared(np.zeros(B, np.int32))
    U.check_scaled(got, ref, dtype, f"shared prefixes {i}, nothing declared")


@pytest.mark.parametrize("group", [2, 4, 16])
def test_decode_shared_prefix_workload_full(U, oracle, group):
    """The bench's batch (C3 shapes) with runs of `group` sequences sharing 90 % of their common cached
    length, through optgqa_decode_step_shared in bundles of two: every row against the oracle."""
    import paper_2505_02351_amd as G
    case = W.make_case(W.CONFIGS["C3"])
    cfg = case.cfg
    W.share_prefix_blocks(case, group, 0.9)
    bundle = G.shared_prefix_bundle(cfg.num_heads, cfg.num_kv_heads, cfg.head_dim)
    shared = W.bundle_shared_blocks(case, bundle)
    assert bundle == 2 and np.count_nonzero(shared) == cfg.batch // 2
    assert G.validate_shared_prefix_host(case.block_tables, case.context_lens, shared, cfg.block_size, bundle, 1) == 0
    kc, vc = oracle_filled(oracle, case)
    ref = oracle_decode(oracle, case, kc, vc)
    dev = U.DevCase(case)
    got = dev.decode_shared(shared, fused=True)
    assert np.array_equal(U.to_host(dev.k_cache), kc) and np.array_equal(U.to_host(dev.v_cache), vc)
    U.check_scaled(got, ref, case.dtype, f"C3, groups of {group} share a prefix", max_exempt=WORKLOAD_EXEMPT)


def test_shared_prefix_rejects_what_it_cannot_do(U):
    import torch
    import paper_2505_02351_amd as G
    bt = torch.zeros(2, 2, dtype=torch.int32, device="cuda")
    cl = torch.ones(2, dtype=torch.int32, device="cuda")
    sb = torch.zeros(2, dtype=torch.int32, device="cuda")
    ws = torch.empty(1 << 20, dtype=torch.float32, device="cuda")
    q = torch.zeros(2, 8, 128, dtype=torch.float16, device="cuda")
    c = torch.zeros(4, 2, 16, 128, dtype=torch.float16, device="cuda")
    with pytest.raises(RuntimeError):                    # no workspace
        G.paged_attention_shared(torch.empty_like(q), q, c, c, bt, cl, sb, None, 0.1, 32, None)
    q96 = torch.zeros(2, 8, 96, dtype=torch.float16, device="cuda")
    c96 = torch.zeros(4, 2, 16, 96, dtype=torch.float16, device="cuda")
    with pytest.raises(RuntimeError):                    # head_dim 96
        G.paged_attention_shared(torch.empty_like(q96), q96, c96, c96, bt, cl, sb, None, 0.1, 32, ws)
    with pytest.raises(TypeError):                       # int64 sharing table
        G.paged_attention_shared(torch.empty_like(q), q, c, c, bt, cl, sb.long(), None, 0.1, 32, ws)


def test_prefill_with_a_sequence_without_new_tokens(U, oracle):
    """A batch in which one sequence contributes no query token (cu_q_lens repeats a value): its
    workgroups have nothing to do, the others are unaffected."""
    import torch
    import paper_2505_02351_amd as G
    cfg = W.small_config(name="pf_empty", kind="prefill", dtype=W.F16, batch=3, num_heads=8, num_kv_heads=2,
                         head_dim=128, block_size=16, num_blocks=3 * 20 + 5, ctx_lo=40, ctx_hi=300, q_len=37, seed=2200)
    case = W.make_case(cfg)
    kc, vc = oracle_filled(oracle, case)
    # insert an extra sequence (a copy of sequence 0's table and length) with zero new tokens after sequence 0
    bt = np.insert(case.block_tables, 1, case.block_tables[0], axis=0)
    cl = np.insert(case.context_lens, 1, case.context_lens[0]).astype(np.int32)
    cu = np.insert(case.cu_q_lens, 1, case.cu_q_lens[1]).astype(np.int32)
    ref = oracle.paged_prefill(case.q, kc, vc, bt, cl, cu, case.slopes, case.scale, W.F16)
    ref0 = oracle.paged_prefill(case.q, kc, vc, case.block_tables, case.context_lens, case.cu_q_lens, case.slopes,
                                case.scale, W.F16)
    assert np.array_equal(ref, ref0)
    dev = U.DevCase(case)
    dev.write_cache()
    out = torch.full_like(dev.q, float("nan"))
    G.paged_prefill(out, dev.q, dev.k_cache, dev.v_cache, torch.from_numpy(bt).cuda(), torch.from_numpy(cl).cuda(),
                    torch.from_numpy(cu).cuda(), dev.slopes, float(case.scale), case.max_q_len)
    torch.cuda.synchronize()
    assert U.max_abs_err(U.to_host(out), ref, W.F16) <= U.TOL[W.F16]


# ------------------------------------------------------------------ seeded random mixes
def test_random_mix_of_decode_calls(U, oracle):
    """Forty seeded random decode batches (head counts, group sizes, block sizes, ragged lengths incl.
    empty sequences) through a randomly chosen entry point each: plain attention with a random split,
    the one-call step, a sliding window (plain / fused), the 8-bit caches.  Every output against
    the oracle clause that defines it; caches bit-exact where the call writes them."""
    import torch
    import oracle as O
    import paper_2505_02351_amd as G
    rng = np.random.default_rng(20251)
    for it in range(40):
        D = int(rng.choice([64, 128, 128, 128]))
        Hkv = int(rng.choice([1, 2, 4, 8]))
        Gq = int(rng.choice([1, 2, 3, 4, 6, 8, 16]))
        bs = int(rng.choice([16, 32, 64]))
        B = int(rng.integers(1, 12))
        hi = int(rng.choice([40, 200, 700, 1500]))
        dtype = W.F16 if rng.integers(2) else W.BF16
        cfg = W.small_config(name=f"mix{it}", dtype=dtype, batch=B, num_heads=Hkv * Gq, num_kv_heads=Hkv, head_dim=D,
                             block_size=bs, num_blocks=B * ((hi + bs - 1) // bs) + 9, ctx_lo=1, ctx_hi=hi,
                             seed=3000 + it)
        lens = rng.integers(1, hi + 1, size=B).astype(np.int32)
        case = W.make_case(cfg, context_lens=lens)
        kc, vc = oracle_filled(oracle, case)
        mode = ["plain", "step", "window", "window_step", "fp8", "fp8_step"][int(rng.integers(6))]
        tag = f"case {it}: {mode} D={D} Hkv={Hkv} G={Gq} bs={bs} B={B} {dtype}"
        dev = U.DevCase(case)
        if mode == "plain":
            dev.write_cache()
            P = int(rng.choice([-1, 0, 64, 256, BALANCED]))
            if P > 0 and P % bs:
                P = 0
            got = dev.decode(partition_size=P)
            ref = oracle_decode(oracle, case, kc, vc)
        elif mode == "step":
            got = dev.step()
            assert np.array_equal(U.to_host(dev.k_cache), kc) and np.array_equal(U.to_host(dev.v_cache), vc), tag
            ref = oracle_decode(oracle, case, kc, vc)
        elif mode in ("window", "window_step"):
            window = int(rng.choice([1, 3, 16, 31, 100, 500]))
            if mode == "window":
                dev.write_cache()
            got = dev.decode_window(window, fused=(mode == "window_step"))
            assert np.array_equal(U.to_host(dev.k_cache), kc) and np.array_equal(U.to_host(dev.v_cache), vc), tag
            ref = O.paged_attention_window(case.q, kc, vc, case.block_tables, case.context_lens, case.slopes,
                                           case.scale, window, dtype)
        else:
            k_scale, v_scale = float(rng.choice([0.01, 0.05, 1.0])), float(rng.choice([0.02, 0.5]))
            kc8, vc8, dk, dv = fp8_caches(U, case, k_scale, v_scale)
            assert np.array_equal(dk.cpu().numpy(), kc8) and np.array_equal(dv.cpu().numpy(), vc8), tag
            if mode == "fp8_step":
                # wipe the new tokens' rows again: the step has to put them back
                s_ = torch.from_numpy(case.slot_mapping).cuda()
                dk[s_ // bs, :, s_ % bs, :] = 0x7F
                dv[s_ // bs, :, s_ % bs, :] = 0x7F
                ws = dev.workspace(BALANCED)[0]
                dev.out.fill_(float("nan"))
                G.decode_step_fp8(dev.out, dev.q, dev.k_new, dev.v_new, dk, dv, dev.block_tables, dev.context_lens,
                                  dev.slopes, float(case.scale), k_scale, v_scale, case.max_context_len, ws)
                torch.cuda.synchronize()
                dev.check_canaries()
                assert np.array_equal(dk.cpu().numpy(), kc8) and np.array_equal(dv.cpu().numpy(), vc8), tag
                got = U.to_host(dev.out)
            else:
                got = fp8_decode(U, case, dk, dv, k_scale, v_scale)
            ref = O.paged_attention_e4m3(case.q, kc8, vc8, case.block_tables, case.context_lens, case.slopes,
                                         case.scale, k_scale, v_scale, dtype)
        U.check_scaled(got, ref, dtype, tag)


def test_random_mix_of_prefill_calls(U, oracle):
    """Twenty-four seeded random prefill batches (chunk lengths from 1 token to the whole prompt)
    through the paged kernel, its windowed and 8-bit variants and the whole-prompt call."""
    import torch
    import oracle as O
    import paper_2505_02351_amd as G
    rng = np.random.default_rng(20252)
    for it in range(24):
        D = int(rng.choice([64, 128, 128, 128]))
        Hkv = int(rng.choice([1, 2, 4]))
        Gq = int(rng.choice([1, 2, 3, 4, 8, 16]))
        bs = int(rng.choice([16, 32, 64]))
        B = int(rng.integers(1, 5))
        hi = int(rng.choice([60, 300, 900]))
        q_len = int(rng.choice([1, 7, 33, 130, hi]))
        dtype = W.F16 if rng.integers(2) else W.BF16
        cfg = W.small_config(name=f"pmix{it}", kind="prefill", dtype=dtype, batch=B, num_heads=Hkv * Gq,
                             num_kv_heads=Hkv, head_dim=D, block_size=bs, num_blocks=B * ((hi + bs - 1) // bs) + 5,
                             ctx_lo=1, ctx_hi=hi, q_len=q_len, seed=3100 + it)
        case = W.make_case(cfg)
        kc, vc = oracle_filled(oracle, case)
        mode = ["plain", "window", "fp8", "prompt"][int(rng.integers(4))]
        if mode == "prompt" and not np.array_equal(case.q_lens, case.context_lens):
            mode = "window"
        tag = f"case {it}: {mode} D={D} Hkv={Hkv} G={Gq} bs={bs} B={B} q_len={q_len} {dtype}"
        dev = U.DevCase(case)
        if mode == "plain":
            dev.write_cache()
            got = dev.prefill()
            ref = oracle.paged_prefill(case.q, kc, vc, case.block_tables, case.context_lens, case.cu_q_lens,
                                       case.slopes, case.scale, dtype)
        elif mode == "window":
            window = int(rng.choice([1, 5, 32, 77, 400]))
            dev.write_cache()
            got = dev.prefill_window(window)
            ref = O.paged_prefill_window(case.q, kc, vc, case.block_tables, case.context_lens, case.cu_q_lens,
                                         case.slopes, case.scale, window, dtype)
        elif mode == "fp8":
            k_scale, v_scale = float(rng.choice([0.0125, 0.1])), float(rng.choice([0.02, 1.0]))
            kc8, vc8, dk, dv = fp8_caches(U, case, k_scale, v_scale)
            out = torch.full_like(dev.q, float("nan"))
            G.paged_prefill_fp8(out, dev.q, dk, dv, dev.block_tables, dev.context_lens, dev.cu_q_lens, dev.slopes,
                                float(case.scale), k_scale, v_scale, case.max_q_len)
            torch.cuda.synchronize()
            got = U.to_host(out)
            ref = O.paged_prefill_e4m3(case.q, kc8, vc8, case.block_tables, case.context_lens, case.cu_q_lens,
                                       case.slopes, case.scale, k_scale, v_scale, dtype)
        else:
            dev.out.fill_(float("nan"))
            G.prompt_prefill(dev.out, dev.q, dev.k_new, dev.v_new, dev.k_cache, dev.v_cache, dev.block_tables,
                             dev.cu_q_lens, dev.slopes, float(case.scale), case.max_q_len)
            torch.cuda.synchronize()
            got = U.to_host(dev.out)
            assert np.array_equal(U.to_host(dev.k_cache), kc) and np.array_equal(U.to_host(dev.v_cache), vc), tag
            ref = O.prompt_attention(case.q, case.k_new, case.v_new, case.cu_q_lens, case.slopes, case.scale, dtype)
        U.check_scaled(got, ref, dtype, tag)


def test_random_mix_of_shared_prefix_calls(U, oracle):
    """Forty seeded random batches whose runs of sequences share a prefix of random length (runs that
    match the kernel's bundles, shorter ones, longer ones), through both shared-prefix entry points."""
    import paper_2505_02351_amd as G
    rng = np.random.default_rng(20254)
    for it in range(40):
        D = int(rng.choice([64, 128, 128]))
        Hkv = int(rng.choice([1, 2, 4, 8]))
        Gq = int(rng.choice([1, 2, 3, 4, 6, 8, 16, 20]))
        bs = int(rng.choice([16, 32, 64]))
        B = int(rng.integers(1, 40))
        hi = int(rng.choice([40, 200, 700, 1500]))
        lo = int(rng.integers(1, hi + 1))
        dtype = W.F16 if rng.integers(2) else W.BF16
        frac = float(rng.choice([0.2, 0.5, 0.9, 1.0]))
        Hq = Hkv * Gq
        bundle = G.shared_prefix_bundle(Hq, Hkv, D)
        group = max(int(rng.choice([2, 3, bundle, 2 * bundle])) if rng.integers(2) else bundle, 2)
        tag = f"case {it}: D={D} Hkv={Hkv} G={Gq} bs={bs} B={B} lens {lo}..{hi} {dtype} bundle={bundle} runs of {group}"
        cfg = W.small_config(name=f"spmix{it}", dtype=dtype, batch=B, num_heads=Hq, num_kv_heads=Hkv, head_dim=D,
                             block_size=bs, num_blocks=B * ((hi + bs - 1) // bs) + 7, ctx_lo=lo, ctx_hi=hi,
                             seed=3400 + it)
        case = W.make_case(cfg)
        W.share_prefix_blocks(case, group, frac)
        shared = W.bundle_shared_blocks(case, bundle)
        assert G.validate_shared_prefix_host(case.block_tables, case.context_lens, shared, bs, bundle, 1) == 0, tag
        kc, vc = oracle_filled(oracle, case)
        ref = oracle_decode(oracle, case, kc, vc)
        dev = U.DevCase(case)
        got = dev.decode_shared(shared, fused=True)
        assert np.array_equal(U.to_host(dev.k_cache), kc) and np.array_equal(U.to_host(dev.v_cache), vc), tag
        U.check_scaled(got, ref, dtype, tag + ", fused step")
        U.check_scaled(dev.decode_shared(shared), ref, dtype, tag + ", plain")


def test_random_mix_of_prefill_steps(U, oracle):
    """Thirty seeded random prefill batches (chunk lengths from 1 token to the whole prompt, every
    group size and block size) through the one-call step: caches and output bit for bit those of
    cache write + prefill, and the output against the oracle."""
    rng = np.random.default_rng(20253)
    for it in range(30):
        D = int(rng.choice([64, 128, 128, 128]))
        Hkv = int(rng.choice([1, 2, 4]))
        Gq = int(rng.choice([1, 2, 3, 4, 8, 16, 20]))
        bs = int(rng.choice([16, 32, 64]))
        B = int(rng.integers(1, 6))
        hi = int(rng.choice([60, 300, 900]))
        q_len = int(rng.choice([1, 2, 7, 33, 130, 257, hi]))
        dtype = W.F16 if rng.integers(2) else W.BF16
        cfg = W.small_config(name=f"psmix{it}", kind="prefill", dtype=dtype, batch=B, num_heads=Hkv * Gq,
                             num_kv_heads=Hkv, head_dim=D, block_size=bs, num_blocks=B * ((hi + bs - 1) // bs) + 5,
                             ctx_lo=1, ctx_hi=hi, q_len=q_len, seed=3300 + it)
        case = W.make_case(cfg)
        tag = f"case {it}: D={D} Hkv={Hkv} G={Gq} bs={bs} B={B} q_len={q_len} {dtype}"
        kc, vc = oracle_filled(oracle, case)
        two = U.DevCase(case)
        two.write_cache()
        want = two.prefill()
        one = U.DevCase(case)
        got = one.prefill_step()
        assert np.array_equal(U.to_host(one.k_cache), kc) and np.array_equal(U.to_host(one.v_cache), vc), tag
        assert np.array_equal(got, want), tag
        ref = oracle.paged_prefill(case.q, kc, vc, case.block_tables, case.context_lens, case.cu_q_lens,
                                   case.slopes, case.scale, dtype)
        U.check_scaled(got, ref, dtype, tag)


def test_decode_step_replays_from_a_hip_graph(U, oracle):
    """The one-call step allocates nothing, synchronises nothing and records no memset, so it can be
    captured: every replay (with eager steps and synchronisations in between) must reproduce the
    eager output bit for bit and leave the caches as the oracle's cache write does."""
    import torch
    import paper_2505_02351_amd as G
    cfg = W.small_config(name="graph", dtype=W.BF16, batch=7, num_heads=16, num_kv_heads=4, head_dim=128,
                         block_size=32, num_blocks=7 * 30 + 3, ctx_lo=100, ctx_hi=900, seed=17)
    case = W.make_case(cfg)
    dev = U.DevCase(case)
    ws, _ = dev.workspace(0)
    def step():
        G.decode_step(dev.out, dev.q, dev.k_new, dev.v_new, dev.k_cache, dev.v_cache, dev.block_tables,
                      dev.context_lens, dev.slopes, float(case.scale), case.max_context_len, ws)
    step()                                   # also does the library's one-off occupancy query
    torch.cuda.synchronize()
    eager = dev.out.clone()
    kc, vc = oracle_filled(oracle, case)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(4):
        dev.out.fill_(float("nan"))
        dev.k_cache.copy_(U.to_dev(case.k_cache, case.dtype))      # back to the image before the step
        dev.v_cache.copy_(U.to_dev(case.v_cache, case.dtype))
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(dev.out, eager), rep
        assert np.array_equal(U.to_host(dev.k_cache), kc) and np.array_equal(U.to_host(dev.v_cache), vc), rep
        step()                               # eager work between the replays
        torch.cuda.synchronize()
        assert torch.equal(dev.out, eager), rep


def test_prefill_step_replays_from_a_hip_graph(U, oracle):
    """The same for the one-call prefill step (one launch, nothing allocated): every replay gives
    the eager output bit for bit and the caches the oracle's cache write leaves."""
    import torch
    import paper_2505_02351_amd as G
    cfg = W.small_config(name="graph-pf", kind="prefill", dtype=W.BF16, batch=3, num_heads=16, num_kv_heads=4,
                         head_dim=128, block_size=16, num_blocks=3 * 40 + 3, ctx_lo=150, ctx_hi=600, q_len=97, seed=18)
    case = W.make_case(cfg)
    dev = U.DevCase(case)
    def step():
        G.prefill_step(dev.out, dev.q, dev.k_new, dev.v_new, dev.k_cache, dev.v_cache, dev.block_tables,
                       dev.context_lens, dev.cu_q_lens, dev.slopes, float(case.scale), case.max_q_len)
    step()                                   # also raises the kernel's dynamic LDS limit, once per process
    torch.cuda.synchronize()
    eager = dev.out.clone()
    kc, vc = oracle_filled(oracle, case)
    ref = oracle.paged_prefill(case.q, kc, vc, case.block_tables, case.context_lens, case.cu_q_lens,
                               case.slopes, case.scale, case.dtype)
    U.check_scaled(U.to_host(eager), ref, case.dtype, "prefill step before capture")
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(4):
        dev.out.fill_(float("nan"))
        dev.k_cache.copy_(U.to_dev(case.k_cache, case.dtype))      # back to the image before the step
        dev.v_cache.copy_(U.to_dev(case.v_cache, case.dtype))
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(dev.out, eager), rep
        assert np.array_equal(U.to_host(dev.k_cache), kc) and np.array_equal(U.to_host(dev.v_cache), vc), rep
        step()                               # eager work between the replays
        torch.cuda.synchronize()
        assert torch.equal(dev.out, eager), rep


def test_stream_probe_runs_and_checks_its_list(U):
    import torch
    import paper_2505_02351_amd as G
    pool = torch.zeros(64 * 4096, dtype=torch.uint8, device="cuda")
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    lst = np.random.default_rng(0).integers(0, 64, size=2 * 4 * 5).astype(np.int32)
    G.stream_probe(pool, pool, lst, 2, 5, sink)
    torch.cuda.synchronize()
    assert not sink.any()
    lst[7] = 64
    with pytest.raises(RuntimeError):
        G.stream_probe(pool, pool, lst, 2, 5, sink)


# ------------------------------------------------------------------ the workloads themselves
@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4", "C5"])
def test_workload_block_permutation_bit_identical(U, name):
    """Every configuration under three different assignments of physical blocks (same logical
    content, tables permuted consistently - Section III-A: pages only re-arrange the sequence): the
    outputs must be the same bits, through the call the bench times."""
    cfg = W.CONFIGS[name]
    outs = []
    for perm_seed in (None, 101, 102):
        case = W.make_case(cfg, perm_seed=perm_seed)
        dev = U.DevCase(case)
        if cfg.kind == "decode":
            outs.append(dev.step() if cfg.partition_size == 0 else
                        (dev.write_cache(), dev.decode(partition_size=cfg.partition_size))[1])
        else:
            dev.write_cache()
            outs.append(dev.prefill())
        del dev, case
    assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[0], outs[2])


WORKLOAD_RUNS = [
    ("C1", 0), ("C1", -1), ("C2", 0), ("C2", -1), ("C2", "step"),
    ("C3", 0), ("C3", 1024), ("C3", "step"),          # "step": optgqa_decode_step, the call the bench times
    ("C3-all8k", "step"),                              # the "batch 64 / 8k" upper case of the target
    ("C4", 512), ("C4", BALANCED), ("C4", "step"),     # 512: the configuration's own partition size
]


@pytest.mark.parametrize("name,mode", WORKLOAD_RUNS)
def test_decode_workload_full(U, oracle, name, mode):
    """Every decode workload at full size, in the launch configuration the bench times and in the
    other split modes: the ENTIRE caches bit for bit after the cache write, and every output row
    against the oracle at the stated tolerance."""
    case = workload_case(name)
    cfg = case.cfg
    if mode == 512:
        assert cfg.partition_size == 512
    dev = U.DevCase(case)
    if mode == "step":
        got = dev.step()
    else:
        dev.write_cache()
        got = dev.decode(partition_size=mode)
    kc, vc = oracle_filled(oracle, case)
    assert np.array_equal(U.to_host(dev.k_cache), kc) and np.array_equal(U.to_host(dev.v_cache), vc)
    ref = oracle_decode(oracle, case, kc, vc)
    U.check_scaled(got, ref, case.dtype, f"{name}, mode {mode}", max_exempt=WORKLOAD_EXEMPT)


# ------------------------------------------------------------------ prefill
PF = [
    (W.BF16, 8, 2, 128, 16, 3, 40, 300, 33),
    (W.F16, 8, 2, 64, 16, 2, 20, 200, 20),
    (W.BF16, 32, 8, 128, 16, 2, 300, 700, 130),
    (W.F16, 4, 4, 128, 32, 2, 64, 400, 64),
    (W.BF16, 6, 2, 128, 16, 2, 5, 100, 100),        # q_len > some contexts: whole prompt is new; G = 3
    (W.F16, 16, 2, 128, 32, 2, 100, 500, 77),       # G = 8, block 32, ragged tiles
    (W.BF16, 4, 4, 128, 16, 3, 1, 260, 260),        # MHA (G = 1), prompts from scratch incl. length 1
    (W.F16, 32, 2, 128, 16, 1, 300, 300, 40),       # G = 16
    (W.BF16, 40, 2, 128, 64, 1, 200, 200, 33),      # G = 20 -> two chunks of 10 heads (padded to 16)
    (W.BF16, 8, 2, 128, 16, 2, 700, 1500, 1),       # one new token per sequence through the prefill path
    # enough workgroups for the 8-wave form of the kernel (256 rows per workgroup, 512+ workgroups):
    (W.BF16, 16, 8, 128, 16, 32, 150, 300, 140),    # G = 2: 128 tokens per workgroup, ragged second query tile
    (W.F16, 8, 8, 64, 32, 64, 50, 400, 400),        # MHA, head_dim 64: 256 tokens per workgroup, whole prompts new
    (W.F16, 32, 8, 128, 16, 8, 600, 900, 520),      # G = 4 (the bench's shape class): 64 tokens per workgroup
]


@pytest.mark.parametrize("i", range(len(PF)))
def test_prefill_sweep(U, oracle, i):
    dtype, Hq, Hkv, D, bs, B, lo, hi, q_len = PF[i]
    cfg = W.small_config(name=f"pf{i}", kind="prefill", dtype=dtype, batch=B, num_heads=Hq, num_kv_heads=Hkv,
                         head_dim=D, block_size=bs, num_blocks=B * ((hi + bs - 1) // bs) + 5, ctx_lo=lo,
                         ctx_hi=hi, q_len=q_len, seed=500 + i)
    case = W.make_case(cfg)
    dev = U.DevCase(case)
    dev.write_cache()
    got = dev.prefill()
    kc, vc = oracle_filled(oracle, case)
    ref = oracle.paged_prefill(case.q, kc, vc, case.block_tables, case.context_lens, case.cu_q_lens,
                               case.slopes, case.scale, dtype)
    U.check_scaled(got, ref, dtype, f"prefill {i}")


@pytest.mark.parametrize("i", range(len(PF)))
def test_prefill_step_sweep(U, oracle, i):
    """Cache write + prefill in one launch: caches and output bit for bit what the two calls give
    (the new tokens' rows are NaN patterns in the cache until the call stores them, so a key read
    from the wrong place would show), and both against the oracle."""
    dtype, Hq, Hkv, D, bs, B, lo, hi, q_len = PF[i]
    cfg = W.small_config(name=f"pfs{i}", kind="prefill", dtype=dtype, batch=B, num_heads=Hq, num_kv_heads=Hkv,
                         head_dim=D, block_size=bs, num_blocks=B * ((hi + bs - 1) // bs) + 5, ctx_lo=lo,
                         ctx_hi=hi, q_len=q_len, seed=500 + i)
    case = W.make_case(cfg)
    two = U.DevCase(case)
    two.write_cache()
    want = two.prefill()
    one = U.DevCase(case)
    got = one.prefill_step()
    kc, vc = oracle_filled(oracle, case)
    assert np.array_equal(U.to_host(one.k_cache), kc) and np.array_equal(U.to_host(one.v_cache), vc)
    assert np.array_equal(U.to_host(two.k_cache), kc) and np.array_equal(U.to_host(two.v_cache), vc)
    assert np.array_equal(got, want), f"prefill step {i}: output differs from write + prefill"
    ref = oracle.paged_prefill(case.q, kc, vc, case.block_tables, case.context_lens, case.cu_q_lens,
                               case.slopes, case.scale, dtype)
    U.check_scaled(got, ref, dtype, f"prefill step {i}")


def test_prefill_step_strided_rows_and_chunks(U, oracle):
    """New rows handed over with a token stride, and a prompt fed in three chunks of uneven size
    (each step reads what the earlier ones stored): the caches end up as the oracle fills them and
    every chunk's output matches the oracle's for the same positions."""
    import torch
    import paper_2505_02351_amd as G
    for dtype, D in ((W.BF16, 128), (W.F16, 64)):
        Hq, Hkv, bs, B = 8, 2, 16, 3
        cfg = W.small_config(name="pfs_chunks", kind="prefill", dtype=dtype, batch=B, num_heads=Hq, num_kv_heads=Hkv,
                             head_dim=D, block_size=bs, num_blocks=B * 25 + 3, ctx_lo=150, ctx_hi=390, q_len=390,
                             seed=911)
        case = W.make_case(cfg)                       # whole prompts new: lengths L_b, positions 0 .. L_b - 1
        kc, vc = oracle_filled(oracle, case)
        ref = oracle.paged_prefill(case.q, kc, vc, case.block_tables, case.context_lens, case.cu_q_lens,
                                   case.slopes, case.scale, dtype)
        dev = U.DevCase(case)
        L = case.context_lens.astype(np.int64)
        cu = case.cu_q_lens.astype(np.int64)
        assert np.array_equal(cu[1:] - cu[:-1], L)
        # strided copies of the new rows (token stride 1.5 rows)
        row = Hkv * D
        kbig = torch.zeros((int(cu[-1]), row + row // 2), dtype=dev.k_new.dtype, device="cuda")
        vbig = torch.zeros_like(kbig)
        kbig[:, :row] = dev.k_new.view(-1, row)
        vbig[:, :row] = dev.v_new.view(-1, row)
        done = np.zeros(B, dtype=np.int64)
        out_all = np.zeros_like(U.to_host(dev.out))
        for frac in (0.37, 0.8, 1.0):
            upto = np.maximum(np.minimum((L * frac).astype(np.int64) | 1, L), done)   # odd chunk ends, except the last
            if frac == 1.0:
                upto = L
            n = upto - done
            idx = np.concatenate([np.arange(cu[b] + done[b], cu[b] + upto[b]) for b in range(B)]).astype(np.int64)
            sel = torch.from_numpy(idx).cuda()
            cu_chunk = torch.from_numpy(np.concatenate([[0], np.cumsum(n)]).astype(np.int32)).cuda()
            ctx = torch.from_numpy(upto.astype(np.int32)).cuda()
            q = dev.q[sel].contiguous()
            out = torch.full_like(q, float("nan"))
            kn = kbig[sel].contiguous()[:, :row].view(-1, Hkv, D)       # rows with a token stride of 1.5 rows
            vn = vbig[sel].contiguous()[:, :row].view(-1, Hkv, D)
            assert kn.stride(0) == row + row // 2
            G.prefill_step(out, q, kn, vn, dev.k_cache, dev.v_cache, dev.block_tables, ctx, cu_chunk, dev.slopes,
                           float(case.scale), int(n.max()))
            torch.cuda.synchronize()
            out_all[idx] = U.to_host(out)
            done = upto
        assert np.array_equal(U.to_host(dev.k_cache), kc) and np.array_equal(U.to_host(dev.v_cache), vc)
        U.check_scaled(out_all, ref, dtype, f"chunked prefill steps, head_dim {D}")


def test_prefill_step_workload_full(U, oracle):
    """C5 at full size through the one-call step: caches bit-exact, output bit for bit the two-call
    path's and every row against the oracle."""
    case = workload_case("C5")
    two = U.DevCase(case)
    two.write_cache()
    want = two.prefill()
    del two
    dev = U.DevCase(case)
    got = dev.prefill_step()
    kc, vc = oracle_filled(oracle, case)
    assert np.array_equal(U.to_host(dev.k_cache), kc) and np.array_equal(U.to_host(dev.v_cache), vc)
    assert np.array_equal(got, want)
    ref = oracle.paged_prefill(case.q, kc, vc, case.block_tables, case.context_lens, case.cu_q_lens,
                               case.slopes, case.scale, case.dtype)
    U.check_scaled(got, ref, case.dtype, "C5, one-call step", max_exempt=WORKLOAD_EXEMPT)


def test_prefill_step_rejects_what_it_cannot_do(U):
    import torch
    import paper_2505_02351_amd as G
    cfg = W.small_config(name="pfs_rej", kind="prefill", dtype=W.BF16, batch=2, num_heads=8, num_kv_heads=2,
                         head_dim=128, block_size=16, num_blocks=40, ctx_lo=40, ctx_hi=100, q_len=20, seed=77)
    case = W.make_case(cfg)
    dev = U.DevCase(case)
    lib = G.load_library()
    args = lambda **kw: [kw.get(k, v) for k, v in dict(
        out=dev.out.data_ptr(), q=dev.q.data_ptr(), k_new=dev.k_new.data_ptr(), v_new=dev.v_new.data_ptr(),
        k_cache=dev.k_cache.data_ptr(), v_cache=dev.v_cache.data_ptr(), bt=dev.block_tables.data_ptr(),
        cl=dev.context_lens.data_ptr(), cu=dev.cu_q_lens.data_ptr(), sl=dev.slopes.data_ptr(), scale=0.1, B=2, Hq=8,
        Hkv=2, D=128, bs=16, mb=int(dev.block_tables.shape[1]), mq=20, ks=256, vs=256, dt=1, st=None).items()]
    assert lib.optgqa_prefill_step(*args(k_new=None)) == -1
    assert lib.optgqa_prefill_step(*args(k_cache=None)) == -1
    assert lib.optgqa_prefill_step(*args(ks=255)) == -2          # rows overlap
    assert lib.optgqa_prefill_step(*args(ks=260)) == -3          # not a multiple of 8 elements
    assert lib.optgqa_prefill_step(*args(vs=(1 << 30) + 8)) == -2
    assert lib.optgqa_prefill_step(*args(D=96)) == -3
    assert lib.optgqa_prefill_step(*args(scale=float("inf"))) == -2
    assert lib.optgqa_prefill_step(*args(k_new=dev.k_new.data_ptr() + 2)) == -3
    assert lib.optgqa_prefill_step(*args(mq=0)) == 0             # nothing to do
    torch.cuda.synchronize()
    assert np.array_equal(U.to_host(dev.k_cache), case.k_cache)  # nothing was stored by any of them


@pytest.mark.parametrize("scale", [0.0, 1e-30, -0.05])
def test_prefill_with_zero_tiny_and_negative_scale(U, oracle, scale):
    """The tiled kernel carries part of the ALiBi term inside the score accumulator as slope / scale;
    a score scale of zero (bias-only softmax), a vanishing one and a negative one must still give
    what eq. (3), (4) give, through the paged, windowed and whole-prompt entry points."""
    import torch
    import oracle as O
    import paper_2505_02351_amd as G
    for dtype in (W.F16, W.BF16):
        cfg = W.small_config(name="pf_scale", kind="prefill", dtype=dtype, batch=2, num_heads=8, num_kv_heads=2,
                             head_dim=128, block_size=16, num_blocks=50, ctx_lo=100, ctx_hi=300, q_len=300,
                             seed=2300)
        case = W.make_case(cfg)
        kc, vc = oracle_filled(oracle, case)
        dev = U.DevCase(case)
        dev.write_cache()
        ref = oracle.paged_prefill(case.q, kc, vc, case.block_tables, case.context_lens, case.cu_q_lens,
                                   case.slopes, scale, dtype)
        dev.out.fill_(float("nan"))
        G.paged_prefill(dev.out, dev.q, dev.k_cache, dev.v_cache, dev.block_tables, dev.context_lens, dev.cu_q_lens,
                        dev.slopes, scale, case.max_q_len)
        torch.cuda.synchronize()
        U.check_scaled(U.to_host(dev.out), ref, dtype, f"paged prefill, scale {scale}")
        dev.out.fill_(float("nan"))
        G.prompt_prefill(dev.out, dev.q, dev.k_new, dev.v_new, None, None, None, dev.cu_q_lens, dev.slopes, scale,
                         case.max_q_len)
        torch.cuda.synchronize()
        ref = O.prompt_attention(case.q, case.k_new, case.v_new, case.cu_q_lens, case.slopes, scale, dtype)
        U.check_scaled(U.to_host(dev.out), ref, dtype, f"whole prompt, scale {scale}")
        dev.out.fill_(float("nan"))
        G.paged_prefill_window(dev.out, dev.q, dev.k_cache, dev.v_cache, dev.block_tables, dev.context_lens,
                               dev.cu_q_lens, dev.slopes, scale, 40, case.max_q_len)
        torch.cuda.synchronize()
        ref = O.paged_prefill_window(case.q, kc, vc, case.block_tables, case.context_lens, case.cu_q_lens,
                                     case.slopes, scale, 40, dtype)
        U.check_scaled(U.to_host(dev.out), ref, dtype, f"windowed prefill, scale {scale}")
        dev.check_canaries()
        # decode takes the same scales
        last = case.cu_q_lens[1:] - 1
        qd = dev.q[torch.from_numpy(last.astype(np.int64)).cuda()].contiguous()
        out = torch.full_like(qd, float("nan"))
        G.paged_attention(out, qd, dev.k_cache, dev.v_cache, dev.block_tables, dev.context_lens, dev.slopes, scale,
                          case.max_context_len, -1, None)
        torch.cuda.synchronize()
        ref = oracle.paged_attention(case.q[last], kc, vc, case.block_tables, case.context_lens, case.slopes, scale,
                                     dtype)
        U.check_scaled(U.to_host(out), ref, dtype, f"decode, scale {scale}")


def test_prefill_workload_full(U, oracle):
    """C5 at full size: caches bit-exact, all 4096 x 32 output rows against the oracle."""
    case = workload_case("C5")
    dev = U.DevCase(case)
    dev.write_cache()
    kc, vc = oracle_filled(oracle, case)
    assert np.array_equal(U.to_host(dev.k_cache), kc) and np.array_equal(U.to_host(dev.v_cache), vc)
    got = dev.prefill()
    ref = oracle.paged_prefill(case.q, kc, vc, case.block_tables, case.context_lens, case.cu_q_lens,
                               case.slopes, case.scale, case.dtype)
    U.check_scaled(got, ref, case.dtype, "C5", max_exempt=WORKLOAD_EXEMPT)
