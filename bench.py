#!/usr/bin/env python3
"""Benchmark of the paged GQA + ALiBi decode hot path on one MI355X.

One "step" = one pass of the whole path over one synthetic batch that is already resident in
HBM: the KV-cache write of the step's new tokens and decode attention over the paged cache
(block-table lookup, group scores, ALiBi, softmax, weighted sum, split-context partition +
combine).  Decode workloads whose partition size is left to the library run the step as ONE
call, optgqa_decode_step; with --partition-size (or a workload that fixes it) the step is
optgqa_reshape_and_cache followed by optgqa_paged_attention.  Prefill workloads (C5) run
optgqa_reshape_and_cache + optgqa_paged_prefill.

Prints ONE JSON line.  `value` is the KV-read rate: algorithmic KV bytes of the batch
(2 * sum(context_lens) * Hkv * D * 2 bytes: every K and V element once per KV-head group)
divided by the wall-clock time of a step, over K steps timed without any event in the stream.
`roofline` prices the dominant kernel alone - the one that streams the KV cache - from HIP
events that the library records around that kernel's launch (optgqa_set_kernel_events) in a
second pass of K steps: HBM-bound for decode (8 TB/s peak), MFMA-bound for the tiled prefill
(2.5 PFLOP/s dense bf16/fp16).  `cpu_baseline` times the fp64 CPU oracle on a bounded sample
of the same batch.  With the default workload (C3, drawn context lengths) a `target_check`
object adds the same measurement for C3-all8k - the batch with every context at 8192 tokens,
which is how the target ("batch 64 / 8k context") is worded.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C3] [--partition-size P]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(1, os.path.join(ROOT, "tests"))      # harness.py: device copies of a generated batch

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_PEAK_TFLOPS = 2500.0      # MI355X dense bf16 / fp16 MFMA, published
KV_SCALE = 0.0125              # --kv-cache e4m3: N(0,1) data, the format's +-448 covers +-5.6 sigma
# HBM bytes per launch of the dominant kernel, from two rocprofv3 --pmc runs per workload (FETCH_SIZE,
# then WRITE_SIZE, KiB per dispatch, mean of 12 dispatches), each scaled by what the same counter
# reads for a plain device copy of 1 GiB (FETCH_SIZE reads 524 301 KiB per GiB copied: x 2.000;
# WRITE_SIZE 1 048 576 KiB: x 1.000).  Keyed by what was run; the summary each entry comes from is
# named next to it.  Not measured in this run: an entry goes stale when its kernel changes, and a
# workload / variant without an entry reports null.
MEASURED_TRAFFIC_BYTES = {
    # key: (bytes, profile summary)                                                    # FETCH_SIZE KiB, WRITE_SIZE KiB
    "C1":              (100_352, "profiles/paged_decode_C1_C2_C4.md"),                # 48.5, 1.0
    "C2":              (83_445_555, "profiles/paged_decode_C1_C2_C4.md"),             # 39 634.0, 2 221.8
    "C3":              (644_162_765, "profiles/paged_decode_C3.md"),                  # 311 871.7, 5 321.8
    "C3-all8k":        (1_089_124_045, "profiles/paged_decode_C3_all8k.md"),          # 529 144.4, 5 308.9
    "C4":              (550_505_882, "profiles/paged_decode_C1_C2_C4.md"),            # 264 641.4, 8 320.6 (P = 512)
    "C4|partition=0":  (551_163_494, "profiles/paged_decode_C1_C2_C4.md"),            # 267 002.1, 4 241.4
    "C5":              (170_643_047, "profiles/paged_prefill_C5.md"),                 # 58 733.6, 49 176.4 (one-call step)
    "C5|two-call":     (151_277_670, "profiles/paged_prefill_C5.md"),                 # 57 481.5, 32 769.1
    "C5-prompt":       (505_036_083, "profiles/paged_prefill_C5_variants.md"),        # 123 718.5, 245 762.3
    "C3|e4m3":         (331_807_642, "profiles/paged_decode_C3_e4m3.md"),             # 157 346.7, 9 337.5
    "C5|e4m3":         (109_350_093, "profiles/paged_prefill_C5_variants.md"),        # 37 009.6, 32 768.0
    "C3|window=1024":  (148_694_733, "profiles/paged_decode_C3_window.md"),           # 70 019.7, 5 170.3
    "C3|window=4096":  (475_426_816, "profiles/paged_decode_C3_window.md"),           # 229 492.9, 5 298.2
    "C5|window=512":   (100_962_509, "profiles/paged_prefill_C5_variants.md"),        # 32 916.8, 32 768.0
    "C3|shared=2":     (429_063_475, "profiles/paged_decode_C3_shared_prefix.md"),    # 205 238.6, 8 530.1
    "C3|shared=4":     (476_824_166, "profiles/paged_decode_C3_shared_prefix.md"),    # 228 907.5, 7 833.6
    "C3-d64":          (321_057_690, "profiles/paged_decode_C3.md"),                  # 155 409.8, 2 713.3 (C3 shapes at head_dim 64)
}


def traffic_key(args, workload: str) -> str:
    """Key of MEASURED_TRAFFIC_BYTES for this run."""
    parts = [workload]
    if args.partition_size is not None:
        parts.append(f"partition={args.partition_size}")
    if args.kv_cache == "e4m3":
        parts.append("e4m3")
    if args.window > 0:
        parts.append(f"window={args.window}")
    if args.shared_prefix > 1:
        parts.append(f"shared={args.shared_prefix}" + ("" if args.shared_prefix_kernel == "bundled" else ",plain"))
    if args.prefill_calls == "two" and workload in ("C5", "C5-d64", "C5-noalibi") and args.kv_cache != "e4m3" \
            and args.window <= 0:
        parts.append("two-call")
    return "|".join(parts)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="C3")
    ap.add_argument("--partition-size", type=int, default=None,
                    help="override the workload's partition size (0 = library chooses, -1 = never split)")
    ap.add_argument("--prefill-calls", choices=["one", "two"], default="one",
                    help="prefill workloads over 2-byte caches without a window: 'one' = optgqa_prefill_step (cache "
                         "write inside the prefill kernel), 'two' = optgqa_reshape_and_cache + optgqa_paged_prefill")
    ap.add_argument("--no-alibi", action="store_true",
                    help="run the workload without ALiBi slopes (plain causal attention; the workload is then named "
                         "<workload>-noalibi: a variant - the prefill kernel can then drop no key tile)")
    ap.add_argument("--head-dim", type=int, choices=[64, 128], default=None,
                    help="run the workload's shapes at this head_dim instead of its own (the workload is then "
                         "named <workload>-d<head_dim>: a variant, not one of the configured workloads)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--lib", default=None, help="load this build of liboptgqa.so instead of the in-tree one")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MIB",
                    help="instead of the benchmark, run a plain device copy of MIB MiB five times "
                         "(known traffic, for scaling the rocprofv3 FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--kv-cache", choices=["native", "e4m3"], default="native",
                    help="e4m3: the same decode workload over 8-bit (E4M3) KV caches with per-tensor scales - "
                         "quantising cache write + optgqa_paged_attention_fp8; KV bytes are then 1 per element")
    ap.add_argument("--no-stream-probe", action="store_true",
                    help="skip the no-arithmetic streaming measurement over the same caches")
    ap.add_argument("--no-target-check", action="store_true",
                    help="skip the extra C3-all8k measurement (every context 8192: the 'batch 64 / 8k' case)")
    ap.add_argument("--window", type=int, default=0,
                    help="> 0: the same workload with a sliding window of this many tokens (local mask of "
                         "Alg. 1), 2-byte caches; KV bytes and flops count the visible keys only")
    ap.add_argument("--shared-prefix", type=int, default=0, metavar="GROUP",
                    help="> 1: runs of GROUP consecutive sequences share 90 %% of their common cached length "
                         "through the same physical blocks (decode workloads); rates still count every "
                         "sequence's logical KV bytes")
    ap.add_argument("--shared-prefix-kernel", choices=["bundled", "plain"], default="bundled",
                    help="with --shared-prefix: bundled = optgqa_decode_step_shared (a bundle of sequences reads "
                         "its shared blocks once); plain = optgqa_decode_step on the same aliased tables")
    ap.add_argument("--no-cold", action="store_true", help="skip the cold-cache pass (evict, then time each step)")
    ap.add_argument("--cpu-sample-seqs", type=int, default=0,
                    help="sequences of the batch the CPU oracle is timed on (0 = all)")
    return ap.parse_args()


def cpu_baseline_e4m3(case, W, n_seqs: int, min_seconds: float = 10.0):
    """The oracle's 8-bit clause on the first n_seqs sequences (0 = all): its own quantising cache
    write of the whole batch once (not timed), then dequantise-then-attend, repeated ~min_seconds."""
    import oracle as O
    cfg = case.cfg
    k_all, v_all, slots = W.all_token_rows(case)
    shape = (cfg.num_blocks, cfg.num_kv_heads, cfg.block_size, cfg.head_dim)
    kc8, vc8 = np.full(shape, 0x7F, np.uint8), np.full(shape, 0x7F, np.uint8)
    O.reshape_and_cache_e4m3(k_all, v_all, kc8, vc8, slots, KV_SCALE, KV_SCALE, case.dtype)
    n_seqs = n_seqs if n_seqs > 0 else cfg.batch
    if cfg.kind != "decode":
        # as for the 2-byte caches: every 16th (token, head) pair of the first sequence
        T0 = int(case.cu_q_lens[1])
        rows = [(t, h) for t in range(T0) for h in range(cfg.num_heads)][::16]
        reps, t0 = 0, time.perf_counter()
        while True:
            O.paged_prefill_e4m3(case.q, kc8, vc8, case.block_tables, case.context_lens, case.cu_q_lens,
                                 case.slopes, case.scale, KV_SCALE, KV_SCALE, case.dtype, rows=rows)
            reps += 1
            dt = time.perf_counter() - t0
            if dt >= min_seconds or reps >= 1000:
                break
        per = dt / reps
        kv_bytes = 2 * int(case.context_lens[0]) * cfg.num_kv_heads * cfg.head_dim // 16
        return {"value": kv_bytes / per / 1e9, "unit": "GB/s", "cores": O.num_threads(), "kind": "oracle",
                "sample": f"every 16th (query token, head) row of sequence 0 ({len(rows)} rows), E4M3 caches "
                          f"({kv_bytes / 1e6:.1f} MB of KV per pass, {reps} passes in {dt:.1f} s)",
                "query_tokens_per_s": T0 / 16.0 / per}
    rows = [(b, h) for b in range(n_seqs) for h in range(cfg.num_heads)]
    reps, t0 = 0, time.perf_counter()
    while True:
        O.paged_attention_e4m3(case.q, kc8, vc8, case.block_tables, case.context_lens, case.slopes, case.scale,
                               KV_SCALE, KV_SCALE, case.dtype, rows=rows)
        reps += 1
        dt = time.perf_counter() - t0
        if dt >= min_seconds or reps >= 1000:
            break
    per = dt / reps
    kv_bytes = 2 * int(case.context_lens[:n_seqs].astype(np.int64).sum()) * cfg.num_kv_heads * cfg.head_dim
    return {"value": kv_bytes / per / 1e9, "unit": "GB/s", "cores": O.num_threads(), "kind": "oracle",
            "sample": f"first {n_seqs} of {cfg.batch} sequences, all {cfg.num_heads} query heads, E4M3 caches "
                      f"({kv_bytes / 1e6:.1f} MB of KV per pass, {reps} passes in {dt:.1f} s)",
            "query_tokens_per_s": n_seqs / per}


def cpu_baseline(case, W, n_seqs: int, min_seconds: float = 10.0, window: int = 0):
    """The oracle as it stands on the first n_seqs sequences of the batch (all their heads; 0 = the
    whole batch), repeated until about min_seconds of CPU work has been timed.  window > 0: the
    oracle's local-mask clause (which scores every key and masks afterwards, as the definition says)."""
    import oracle as O
    cfg = case.cfg
    kc, vc = case.k_cache.copy(), case.v_cache.copy()
    O.reshape_and_cache(case.k_new, case.v_new, kc, vc, case.slot_mapping)
    lens = case.context_lens.astype(np.int64)
    if n_seqs <= 0:
        n_seqs = cfg.batch
    if cfg.kind == "decode":
        rows = [(b, h) for b in range(n_seqs) for h in range(cfg.num_heads)]
        what = f"first {n_seqs} of {cfg.batch} sequences, all {cfg.num_heads} query heads"

        def run():
            if window > 0:
                O.paged_attention_window(case.q, kc, vc, case.block_tables, case.context_lens, case.slopes,
                                         case.scale, window, case.dtype, rows=rows)
            else:
                O.paged_attention(case.q, kc, vc, case.block_tables, case.context_lens, case.slopes, case.scale,
                                  case.dtype, rows=rows)
        seen = np.minimum(lens[:n_seqs], window) if window > 0 else lens[:n_seqs]
        kv_bytes = 2 * int(seen.sum()) * cfg.num_kv_heads * cfg.head_dim * 2
        n_q = n_seqs
    else:
        # every 16th (token, head) pair of the first sequence: the oracle re-reads K/V per row
        T0 = int(case.cu_q_lens[1])
        rows = [(t, h) for t in range(T0) for h in range(cfg.num_heads)][::16]
        what = f"every 16th (query token, head) row of sequence 0 ({len(rows)} rows)"

        def run():
            if "-prompt" in cfg.name:
                O.prompt_attention(case.q, case.k_new, case.v_new, case.cu_q_lens, case.slopes, case.scale,
                                   case.dtype, rows=rows)
            elif window > 0:
                O.paged_prefill_window(case.q, kc, vc, case.block_tables, case.context_lens, case.cu_q_lens,
                                       case.slopes, case.scale, window, case.dtype, rows=rows)
            else:
                O.paged_prefill(case.q, kc, vc, case.block_tables, case.context_lens, case.cu_q_lens, case.slopes,
                                case.scale, case.dtype, rows=rows)
        kv_bytes = 2 * int(lens[0]) * cfg.num_kv_heads * cfg.head_dim * 2 // 16
        n_q = T0 / 16.0
    reps, t0 = 0, time.perf_counter()
    while True:
        run()
        reps += 1
        dt = time.perf_counter() - t0
        if dt >= min_seconds or reps >= 1000:
            break
    per = dt / reps
    single = None
    if cfg.name in ("C1", "C2"):
        # the small configs once more on one thread (a few passes)
        nthreads = O.num_threads()
        O.set_num_threads(1)
        t1 = time.perf_counter()
        n1 = 0
        while n1 < 3 and time.perf_counter() - t1 < 10.0:
            run()
            n1 += 1
        single = {"value": kv_bytes / ((time.perf_counter() - t1) / n1) / 1e9, "unit": "GB/s", "cores": 1, "passes": n1}
        O.set_num_threads(nthreads)
    return {
        **({"single_thread": single} if single else {}),
        "value": kv_bytes / per / 1e9, "unit": "GB/s", "cores": O.num_threads(), "kind": "oracle",
        "sample": f"{what}{f', window {window}' if window > 0 else ''} ({kv_bytes / 1e6:.1f} MB of KV per pass, "
                  f"{reps} passes in {dt:.1f} s)",
        "query_tokens_per_s": n_q / per,
    }


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(units of work are independent per sequence and KV head; nothing is sharded here)", file=sys.stderr)
        sys.exit(2)
    import torch
    if args.copy_calibration:
        n = args.copy_calibration << 20
        src = torch.ones(n, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": {"bytes_read_per_copy": n, "bytes_written_per_copy": n, "copies": 5}}))
        return
    import paper_2505_02351_amd as G
    import workloads as W

    G.load_library(args.lib) if args.lib else G.load_library()      # no library, no benchmark
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    def measure(workload: str, steps: int, warmup: int):
        """Runs one workload; returns (result dict, case)."""
        cfg = W.CONFIGS[workload]
        if args.head_dim is not None and args.head_dim != cfg.head_dim:
            import dataclasses
            cfg = dataclasses.replace(cfg, head_dim=args.head_dim, name=f"{cfg.name}-d{args.head_dim}")
        if args.no_alibi:
            import dataclasses
            cfg = dataclasses.replace(cfg, name=f"{cfg.name}-noalibi")
        case = W.make_case(cfg)
        if args.no_alibi:
            case.slopes = None
        shared_tokens = 0
        if args.shared_prefix > 1:
            assert cfg.kind == "decode", "--shared-prefix applies to decode workloads"
            shared_tokens = W.share_prefix_blocks(case, args.shared_prefix, 0.9)
        bundled = shared_tokens > 0 and args.shared_prefix_kernel == "bundled"
        from harness import DevCase
        dev = DevCase(case)
        P = cfg.partition_size if args.partition_size is None else args.partition_size
        decode = cfg.kind == "decode"
        ws, chosen_P = dev.workspace(P) if decode else (None, 0)
        max_ctx = case.max_context_len
        scale = float(case.scale)
        stream = torch.cuda.current_stream()

        e4m3 = args.kv_cache == "e4m3"
        window = max(args.window, 0)
        assert not (e4m3 and window), "--window runs over 2-byte caches"
        if window and decode:
            ws, chosen_P = dev.workspace(G.SPLIT_BALANCED)
        if e4m3:
            # 8-bit caches of the same logical content, quantised on the GPU from the 2-byte rows of
            # every token but the step's new ones (those are written by the timed step)
            k_old, v_old, slots_old = W.all_token_rows(case, include_new=False)
            shape = (cfg.num_blocks, cfg.num_kv_heads, cfg.block_size, cfg.head_dim)
            k8 = torch.full(shape, 0x7F, dtype=torch.uint8, device="cuda")
            v8 = torch.full(shape, 0x7F, dtype=torch.uint8, device="cuda")
            from harness import to_dev
            if len(slots_old):
                G.reshape_and_cache_fp8(to_dev(k_old, case.dtype), to_dev(v_old, case.dtype), k8, v8,
                                        torch.from_numpy(slots_old).cuda(), KV_SCALE, KV_SCALE)
            torch.cuda.synchronize()
            del k_old, v_old
            if decode:
                ws, chosen_P = dev.workspace(G.SPLIT_BALANCED)
        one_call = decode and (P == 0 or window or e4m3)
        bundle_read_tokens = 0
        if bundled:
            assert not (e4m3 or window) and P == 0, "--shared-prefix-kernel bundled: 2-byte caches, no window, library's split"
            bundle = G.shared_prefix_bundle(cfg.num_heads, cfg.num_kv_heads, cfg.head_dim)
            shared_host = W.bundle_shared_blocks(case, bundle)
            assert G.validate_shared_prefix_host(case.block_tables, case.context_lens, shared_host, cfg.block_size,
                                                 bundle, 1) == 0
            shared_dev = torch.from_numpy(shared_host).cuda()
            ws = dev.shared_workspace()
            chosen_P = G.SPLIT_BALANCED
            # tokens a bundle reads once instead of once per sharing member
            for b0 in range(0, cfg.batch, bundle):
                members = [b for b in range(b0 + 1, min(b0 + bundle, cfg.batch)) if shared_host[b] > 0]
                if members:
                    bundle_read_tokens += len(members) * int(min(shared_host[b] for b in members)) * cfg.block_size

        prompt = "-prompt" in cfg.name       # whole prompts, caches empty: one call stores K/V and attends
        assert not (prompt and (e4m3 or window)), "the whole-prompt workload runs over 2-byte inputs, full causal mask"

        # prefill over cached context, 2-byte caches, full causal mask: one call stores the new rows and attends
        pf_one_call = not decode and not prompt and not e4m3 and not window and args.prefill_calls == "one"

        def step():
            if prompt:
                G.prompt_prefill(dev.out, dev.q, dev.k_new, dev.v_new, dev.k_cache, dev.v_cache, dev.block_tables,
                                 dev.cu_q_lens, dev.slopes, scale, case.max_q_len, stream)
                return
            if e4m3 and decode:
                G.decode_step_fp8(dev.out, dev.q, dev.k_new, dev.v_new, k8, v8, dev.block_tables, dev.context_lens,
                                  dev.slopes, scale, KV_SCALE, KV_SCALE, max_ctx, ws, stream)
                return
            if e4m3:
                G.reshape_and_cache_fp8(dev.k_new, dev.v_new, k8, v8, dev.slot_mapping, KV_SCALE, KV_SCALE, stream)
                G.paged_prefill_fp8(dev.out, dev.q, k8, v8, dev.block_tables, dev.context_lens, dev.cu_q_lens,
                                    dev.slopes, scale, KV_SCALE, KV_SCALE, case.max_q_len, stream)
                return
            if bundled:
                G.decode_step_shared(dev.out, dev.q, dev.k_new, dev.v_new, dev.k_cache, dev.v_cache, dev.block_tables,
                                     dev.context_lens, shared_dev, dev.slopes, scale, max_ctx, ws, stream)
                return
            if one_call and window:
                G.decode_step_window(dev.out, dev.q, dev.k_new, dev.v_new, dev.k_cache, dev.v_cache,
                                     dev.block_tables, dev.context_lens, dev.slopes, scale, window, max_ctx, ws, stream)
                return
            if one_call:
                G.decode_step(dev.out, dev.q, dev.k_new, dev.v_new, dev.k_cache, dev.v_cache, dev.block_tables,
                              dev.context_lens, dev.slopes, scale, max_ctx, ws, stream)
                return
            if pf_one_call:
                G.prefill_step(dev.out, dev.q, dev.k_new, dev.v_new, dev.k_cache, dev.v_cache, dev.block_tables,
                               dev.context_lens, dev.cu_q_lens, dev.slopes, scale, case.max_q_len, stream)
                return
            G.reshape_and_cache(dev.k_new, dev.v_new, dev.k_cache, dev.v_cache, dev.slot_mapping, stream)
            if decode:
                G.paged_attention(dev.out, dev.q, dev.k_cache, dev.v_cache, dev.block_tables, dev.context_lens,
                                  dev.slopes, scale, max_ctx, P, ws, stream)
            elif window:
                G.paged_prefill_window(dev.out, dev.q, dev.k_cache, dev.v_cache, dev.block_tables, dev.context_lens,
                                       dev.cu_q_lens, dev.slopes, scale, window, case.max_q_len, stream)
            else:
                G.paged_prefill(dev.out, dev.q, dev.k_cache, dev.v_cache, dev.block_tables, dev.context_lens,
                                dev.cu_q_lens, dev.slopes, scale, case.max_q_len, stream)

        for _ in range(warmup):
            step()
        torch.cuda.synchronize()

        # ---- pass 1: K steps, wall clock, nothing but the step's own launches in the stream -------
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            step()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0

        # ---- pass 2: the same K steps with an event pair around the dominant kernel of each --------
        starts = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
        stops = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
        for e in starts + stops:
            e.record(stream)                      # makes torch create the HIP event behind it
        torch.cuda.synchronize()
        for i in range(steps):
            G.set_kernel_events(starts[i], stops[i])
            step()
        G.set_kernel_events(None, None)
        torch.cuda.synchronize()
        kernel_ms = np.array([s.elapsed_time(e) for s, e in zip(starts, stops)])

        # ---- pass 3: cold steps - the last-level cache (256 MiB) is evicted before every step by
        # READING a 1 GiB scratch buffer (a written one leaves dirty lines whose write-back then runs
        # under the timed step: measured +60 us on the decode workload), and each whole step is timed
        # by its own event pair --
        cold = None
        if not args.no_cold:
            n_cold = min(steps, 50)
            scratch = torch.zeros(1 << 28, dtype=torch.int32, device="cuda")
            c0 = [torch.cuda.Event(enable_timing=True) for _ in range(n_cold)]
            c1 = [torch.cuda.Event(enable_timing=True) for _ in range(n_cold)]
            for i in range(n_cold):
                scratch.sum()
                c0[i].record(stream)
                step()
                c1[i].record(stream)
            torch.cuda.synchronize()
            del scratch
            cold_ms = np.array([a.elapsed_time(b) for a, b in zip(c0, c1)])
            cold = {"steps": n_cold, "median_ms": float(np.median(cold_ms)), "min_ms": float(cold_ms.min()),
                    "p90_ms": float(np.percentile(cold_ms, 90)),
                    "what": "whole step, event pair per step (includes ~3 us of event overhead), 1 GiB "
                            "read between steps to evict the last-level cache"}

        ms_per_step = wall * 1e3 / steps
        kv_bytes = case.kv_bytes() // (2 if e4m3 else 1)
        if window and decode:                      # a query reads min(L, window) tokens of each KV head
            seen = np.minimum(case.context_lens.astype(np.int64), window)
            kv_bytes = int(2 * int(seen.sum()) * cfg.num_kv_heads * cfg.head_dim * 2)
        value = kv_bytes / (ms_per_step * 1e-3) / 1e9
        n_q = case.num_tokens
        launch_ms = {"mean": float(kernel_ms.mean()), "median": float(np.median(kernel_ms)),
                     "min": float(kernel_ms.min()), "p90": float(np.percentile(kernel_ms, 90))}
        traffic = MEASURED_TRAFFIC_BYTES.get(traffic_key(args, cfg.name), (None, None))
        # bytes the kernel has to read: with the bundled shared-prefix kernel a bundle's shared blocks count once
        unique_kv_bytes = kv_bytes - 2 * bundle_read_tokens * cfg.num_kv_heads * cfg.head_dim * 2
        if decode:
            achieved = unique_kv_bytes / (kernel_ms.mean() * 1e-3) / 1e9
            if chosen_P == G.SPLIT_BALANCED:
                kname = "paged_decode_flat_kernel (equal-work split%s%s%s)" % (
                    ", E4M3 caches, new token merged by the combine kernel" if e4m3 else ", cache write fused" if one_call else "",
                    f", window {window}" if window else "", ", shared prefixes read once per bundle" if bundled else "")
            elif cfg.head_dim == 128 and chosen_P > 0:
                kname = f"paged_decode_flat_kernel (fixed partitions of {chosen_P} tokens on the equal-work kernel)"
            else:
                kname = "paged_decode_mma_kernel / paged_decode_mc_kernel (unsplit or fixed partitions)"
            roofline = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                        "frac": achieved / HBM_PEAK_GBS,
                        "traffic": traffic[0], "traffic_source": traffic[1],
                        "kernel": kname, "algorithmic_bytes_per_launch": unique_kv_bytes, "launch_ms": launch_ms}
        else:
            # causal prefill: query i of sequence b sees pos_i + 1 keys; QK^T and PV are 2 * D flops per
            # (query, key, head) each
            flops = 0
            for b in range(cfg.batch):
                n_b = int(case.q_lens[b])
                first = int(case.context_lens[b]) - n_b
                if window:
                    visible = np.minimum(np.arange(first, first + n_b, dtype=np.int64) + 1, window).sum()
                else:
                    visible = n_b * first + n_b * (n_b + 1) // 2
                flops += 4 * cfg.num_heads * cfg.head_dim * int(visible)
            achieved = flops / (kernel_ms.mean() * 1e-3) / 1e12
            roofline = {"bound": "mfma", "achieved": achieved, "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                        "frac": achieved / MFMA_PEAK_TFLOPS, "traffic": traffic[0], "traffic_source": traffic[1],
                        "kernel": ("paged_prefill_step_kernel (cache write inside)" if pf_one_call else "paged_prefill_mma_kernel")
                                  + (" (E4M3 caches)" if e4m3 else "")
                                  + (" (K/V from the contiguous inputs, cache write fused)" if prompt else "")
                                  + (f" (window {window})" if window else ""),
                        "algorithmic_flops_per_launch": flops,
                        "launch_ms": launch_ms}

        # the cache write on its own (it is part of every step above; inside the kernel for one-call steps)
        cw = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(40)]
        for a, b in cw:
            a.record(stream)
            if e4m3:
                G.reshape_and_cache_fp8(dev.k_new, dev.v_new, k8, v8, dev.slot_mapping, KV_SCALE, KV_SCALE, stream)
            else:
                G.reshape_and_cache(dev.k_new, dev.v_new, dev.k_cache, dev.v_cache, dev.slot_mapping, stream)
            b.record(stream)
        torch.cuda.synchronize()
        cw_ms = np.array([a.elapsed_time(b) for a, b in cw][5:])
        moved = 2 * case.num_tokens * cfg.num_kv_heads * cfg.head_dim * (3 if e4m3 else 4)   # read + written
        cache_write = {"entry_point": "optgqa_reshape_and_cache" + ("_fp8" if e4m3 else ""), "tokens": case.num_tokens,
                       "bytes_moved": moved, "call_ms": float(cw_ms.mean()),
                       "what": "separate launch, event-timed per call (launch latency included)"}

        stream_probe = None
        if decode and not e4m3 and not window and not args.no_stream_probe and cfg.head_dim == 128:
            # The decode kernels' load pattern with no arithmetic, over the same caches: every wave of a
            # one-workgroup-per-CU launch streams an equal share of randomly chosen 16-token pieces
            # (4 KiB of K and 4 KiB of V each), as many bytes as the batch's KV.
            pool_bytes = dev.k_cache.numel() * 2
            wgs = 256
            tiles = max(int(kv_bytes // 8192 // (wgs * 4)), 1)
            rng = np.random.default_rng(123)
            pairs = rng.permutation(pool_bytes // 8192)[:(wgs * 4 * tiles + 1) // 2]
            lst = np.stack([2 * pairs, 2 * pairs + 1], axis=1).reshape(-1)[:wgs * 4 * tiles].astype(np.int32)
            sink = torch.zeros(4, dtype=torch.int32, device="cuda")
            lst_dev = G.stream_probe(dev.k_cache, dev.v_cache, lst, wgs, tiles, sink, None, stream)
            ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(30)]
            for a, b in ev:
                a.record(stream)
                G.stream_probe(dev.k_cache, dev.v_cache, lst, wgs, tiles, sink, lst_dev, stream)
                b.record(stream)
            torch.cuda.synchronize()
            ms = np.array([a.elapsed_time(b) for a, b in ev][5:])
            nbytes = wgs * 4 * tiles * 8192
            stream_probe = {"bytes": nbytes, "kernel_ms": float(ms.mean()), "GB/s": nbytes / (ms.mean() * 1e-3) / 1e9,
                            "frac_of_peak": nbytes / (ms.mean() * 1e-3) / 1e9 / HBM_PEAK_GBS,
                            "what": "optgqa_stream_probe: same K/V load pattern, random 16-token pieces of the "
                                    "same caches, one wave per SIMD, no arithmetic; event-timed per launch"}

        result = {
            "metric": "paged GQA+ALiBi decode: KV-read HBM GB/s (% of peak) and query tokens/s",
            "value": value, "unit": "GB/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
            "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": case.dtype, "data": "synthetic",
            "config": {"workload": cfg.name, "kind": cfg.kind, "batch": cfg.batch, "num_heads": cfg.num_heads,
                       "num_kv_heads": cfg.num_kv_heads, "head_dim": cfg.head_dim, "block_size": cfg.block_size,
                       "context_len_range": [cfg.ctx_lo, cfg.ctx_hi], "sum_context_lens": int(case.context_lens.sum()),
                       "kv_bytes": kv_bytes, "partition_size": int(chosen_P), "num_blocks": cfg.num_blocks,
                       "calls_per_step": 1 if one_call or prompt or pf_one_call else 2,
                       "kv_cache": "e4m3, per-tensor scales" if e4m3 else case.dtype,
                       **({"window": window} if window else {}),
                       **({"shared_prefix_group": args.shared_prefix,
                           "aliased_context_tokens": int(shared_tokens),
                           "shared_prefix_kernel": args.shared_prefix_kernel,
                           "kv_bytes_read_once_per_bundle": int(kv_bytes - 2 * bundle_read_tokens * cfg.num_kv_heads
                                                                * cfg.head_dim * 2)} if shared_tokens else {})},
            "pct_of_hbm_peak": 100.0 * value / HBM_PEAK_GBS,
            "query_tokens_per_s": n_q / (ms_per_step * 1e-3),
            "roofline": roofline,
        }
        if cold:
            result["cold_step"] = cold
        if shared_tokens:
            result["roofline"]["note"] = ("`value` counts every sequence's logical KV bytes; %d of %d context "
                                          "tokens alias another sequence's blocks (%s); `roofline` counts the "
                                          "bytes the kernel has to read"
                                          % (shared_tokens, int(case.context_lens.sum()),
                                             "the bundled kernel reads a bundle's shared blocks once" if bundled
                                             else "the plain kernel reads them once per sequence"))
        result["cache_write"] = cache_write
        if stream_probe:
            result["stream_probe"] = stream_probe
            result["roofline"]["frac_of_stream_probe"] = roofline["achieved"] / stream_probe["GB/s"]
        return result, case

    result, case = measure(args.workload, args.steps, args.warmup)
    if (args.workload == "C3" and args.head_dim in (None, 128) and args.partition_size is None and not args.no_target_check
            and args.kv_cache == "native" and args.window <= 0):
        # the target is worded "batch 64 / 8k context": the same batch with every context at 8192
        extra, _ = measure("C3-all8k", max(args.steps // 2, 1), max(args.warmup // 2, 1))
        result["target_check"] = {
            "workload": "C3-all8k", "what": "same batch with every context length 8192",
            "value": extra["value"], "unit": "GB/s", "pct_of_hbm_peak": extra["pct_of_hbm_peak"],
            "ms_per_step": extra["ms_per_step"], "steps": extra["steps"],
            "roofline_frac": extra["roofline"]["frac"], "kernel_ms": extra["roofline"]["launch_ms"]["mean"],
            "kv_bytes": extra["config"]["kv_bytes"],
        }
    if not args.no_cpu_baseline:
        if args.kv_cache == "e4m3":
            result["cpu_baseline"] = cpu_baseline_e4m3(case, W, args.cpu_sample_seqs)
        else:
            result["cpu_baseline"] = cpu_baseline(case, W, args.cpu_sample_seqs, window=max(args.window, 0))
    print(json.dumps(result))


if __name__ == "__main__":
    main()
