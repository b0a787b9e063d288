"""optgqa_paged_attention_static (the entry point for callers that cannot allocate: its
split-context scratch is a static device array of the library) against optgqa_paged_attention
with a caller-owned workspace, on two calls in a row, the second with a smaller input, then a
head_dim 64 batch (fixed partitions in the same scratch)."""
import numpy as np
import pytest

import workloads as W

pytestmark = pytest.mark.gpu


def test_static_scratch_entry_point_matches_workspace_entry_point(oracle):
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    import paper_2505_02351_amd as G
    G.load_library()
    import harness as U

    shapes = [
        # dtype, Hq, Hkv, D, bs, batch, ctx_lo, ctx_hi
        (W.BF16, 32, 4, 128, 32, 24, 200, 3000),     # equal-work split, 24 x 4 segments
        (W.BF16, 32, 4, 128, 32, 5, 1, 700),         # smaller input right after: stale slots must not leak
        (W.F16, 16, 4, 64, 16, 6, 300, 1500),        # head_dim 64: fixed partitions in the same scratch
    ]
    for i, (dtype, Hq, Hkv, D, bs, B, lo, hi) in enumerate(shapes):
        cfg = W.small_config(name=f"static{i}", dtype=dtype, batch=B, num_heads=Hq, num_kv_heads=Hkv, head_dim=D,
                             block_size=bs, num_blocks=B * ((hi + bs - 1) // bs) + 7, ctx_lo=lo, ctx_hi=hi,
                             seed=5100 + i)
        case = W.make_case(cfg)
        print(f"static scratch case {i}: B={B} Hq={Hq} Hkv={Hkv} D={D} bs={bs} max L={case.max_context_len}", flush=True)
        dev = U.DevCase(case)
        dev.write_cache()
        n, chosen = G.paged_attention_workspace_bytes(B, Hq, Hkv, D, bs, case.max_context_len, 0)
        assert n > 0 and chosen != 0, "the case is meant to take the split path"
        assert n <= G.STATIC_SCRATCH_BYTES
        want = dev.decode(partition_size=0)                      # caller-owned workspace
        out = torch.full_like(dev.q, float("nan"))
        G.paged_attention_static(out, dev.q, dev.k_cache, dev.v_cache, dev.block_tables, dev.context_lens,
                                 dev.slopes, float(case.scale), case.max_context_len)
        torch.cuda.synchronize()
        got = U.to_host(out)
        # same kernels, same launch shapes, same order of operations: the same bits
        assert np.array_equal(got, want), f"case {i}"
        kc, vc = case.k_cache.copy(), case.v_cache.copy()
        oracle.reshape_and_cache(case.k_new, case.v_new, kc, vc, case.slot_mapping)
        ref = oracle.paged_attention(case.q, kc, vc, case.block_tables, case.context_lens, case.slopes, case.scale,
                                     dtype)
        assert U.max_abs_err(got, ref, dtype) <= U.TOL[dtype]

    # a shape whose split needs more than the static array: refused, nothing launched
    B = 500
    q = torch.zeros(B, 32, 128, dtype=torch.bfloat16, device="cuda")
    cache = torch.zeros(4, 2, 16, 128, dtype=torch.bfloat16, device="cuda")
    bt = torch.zeros(B, 256, dtype=torch.int32, device="cuda")
    cl = torch.ones(B, dtype=torch.int32, device="cuda")
    n, _ = G.paged_attention_workspace_bytes(B, 32, 2, 128, 16, 4096, 0)
    assert n > G.STATIC_SCRATCH_BYTES
    with pytest.raises(G.OptGqaError) as e:
        G.paged_attention_static(torch.empty_like(q), q, cache, cache, bt, cl, None, 0.1, 4096)
    assert e.value.status == -4
