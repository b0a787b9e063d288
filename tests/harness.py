"""Harness helper for the tests, the smoke check and the bench: moves a generated batch
(workloads.Case, numpy bit patterns) to the GPU and runs it through the C-ABI binding."""
from __future__ import annotations

import numpy as np
import torch

import workloads as W

import paper_2505_02351_amd as G

TOL = {W.F16: 2e-3, W.BF16: 1e-2}          # max-abs error against the fp64 oracle
TORCH_DT = {W.F16: torch.float16, W.BF16: torch.bfloat16}


def to_dev(bits: np.ndarray, dtype: str) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to("cuda")
    return t.view(TORCH_DT[dtype])


def to_host(t: torch.Tensor) -> np.ndarray:
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


class DevCase:
    """Device copies of a workloads.Case."""

    def __init__(self, case: W.Case):
        self.case = case
        dt = case.dtype
        self.q = to_dev(case.q, dt)
        self.k_new = to_dev(case.k_new, dt)
        self.v_new = to_dev(case.v_new, dt)
        self.k_cache = to_dev(case.k_cache, dt)
        self.v_cache = to_dev(case.v_cache, dt)
        self.slot_mapping = torch.from_numpy(case.slot_mapping).to("cuda")
        self.block_tables = torch.from_numpy(case.block_tables).to("cuda")
        self.context_lens = torch.from_numpy(case.context_lens).to("cuda")
        self.cu_q_lens = torch.from_numpy(case.cu_q_lens).to("cuda")
        self.slopes = torch.from_numpy(case.slopes).to("cuda")
        self.out = torch.empty_like(self.q)

    def write_cache(self):
        G.reshape_and_cache(self.k_new, self.v_new, self.k_cache, self.v_cache, self.slot_mapping)

    def workspace(self, partition_size=0):
        c = self.case.cfg
        n, chosen = G.paged_attention_workspace_bytes(c.batch, c.num_heads, c.num_kv_heads, c.head_dim,
                                                      c.block_size, max(self.case.max_context_len, 1),
                                                      partition_size)
        ws = torch.empty(max(n, 16) // 4, dtype=torch.float32, device="cuda") if n else None
        return ws, chosen

    def decode(self, partition_size=0, slopes="case", workspace="auto"):
        sl = self.slopes if isinstance(slopes, str) else slopes
        ws = self.workspace(partition_size)[0] if isinstance(workspace, str) else workspace
        self.out.fill_(float("nan"))
        G.paged_attention(self.out, self.q, self.k_cache, self.v_cache, self.block_tables, self.context_lens,
                          sl, float(self.case.scale), self.case.max_context_len, partition_size, ws)
        torch.cuda.synchronize()
        return to_host(self.out)

    def step(self, workspace="auto"):
        """Cache write + decode attention through the single-call entry point."""
        ws = self.workspace(0)[0] if isinstance(workspace, str) else workspace
        self.out.fill_(float("nan"))
        G.decode_step(self.out, self.q, self.k_new, self.v_new, self.k_cache, self.v_cache, self.block_tables,
                      self.context_lens, self.slopes, float(self.case.scale), self.case.max_context_len, ws)
        torch.cuda.synchronize()
        return to_host(self.out)

    def decode_window(self, window, slopes="case", fused=False):
        """Windowed decode: over filled caches, or (fused) with the step's cache write in the call."""
        sl = self.slopes if isinstance(slopes, str) else slopes
        ws = self.workspace(G.SPLIT_BALANCED)[0]
        self.out.fill_(float("nan"))
        if fused:
            G.decode_step_window(self.out, self.q, self.k_new, self.v_new, self.k_cache, self.v_cache,
                                 self.block_tables, self.context_lens, sl, float(self.case.scale), window,
                                 self.case.max_context_len, ws)
        else:
            G.paged_attention_window(self.out, self.q, self.k_cache, self.v_cache, self.block_tables,
                                     self.context_lens, sl, float(self.case.scale), window,
                                     self.case.max_context_len, ws)
        torch.cuda.synchronize()
        return to_host(self.out)

    def prefill_window(self, window, slopes="case"):
        sl = self.slopes if isinstance(slopes, str) else slopes
        self.out.fill_(float("nan"))
        G.paged_prefill_window(self.out, self.q, self.k_cache, self.v_cache, self.block_tables, self.context_lens,
                               self.cu_q_lens, sl, float(self.case.scale), window, self.case.max_q_len)
        torch.cuda.synchronize()
        return to_host(self.out)

    def prefill(self):
        self.out.fill_(float("nan"))
        G.paged_prefill(self.out, self.q, self.k_cache, self.v_cache, self.block_tables, self.context_lens,
                        self.cu_q_lens, self.slopes, float(self.case.scale), self.case.max_q_len)
        torch.cuda.synchronize()
        return to_host(self.out)


def max_abs_err(bits: np.ndarray, ref: np.ndarray, dtype: str) -> float:
    got = W.from_bits(bits, dtype)
    assert np.all(np.isfinite(got)), "non-finite values in the GPU output"
    return float(np.max(np.abs(got - ref))) if ref.size else 0.0
