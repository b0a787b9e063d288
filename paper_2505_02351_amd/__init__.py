"""Python binding of liboptgqa.so: paged GQA + ALiBi attention for MI355X.

Argument marshalling only -- every step of the path runs in the HIP kernels behind the C ABI
declared in include/optgqa.h.  PyTorch is used for device memory and streams; tensors are passed
as raw device pointers.  There is no CPU or PyTorch fallback: if the shared library is missing
or fails to load, importing the functions raises.

Tensor conventions (see include/optgqa.h for the full contract):
  q, out        [rows, Hq, D]            float16 or bfloat16
  k, v          [T, Hkv, D]
  k_cache, v_cache  [NB, Hkv, bs, D]
  block_tables  [B, MB] int32,  context_lens [B] int32,  slot_mapping [T] int64
  alibi_slopes  [Hq] float32 or None
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "liboptgqa.so")

F16, BF16 = 0, 1
SPLIT_BALANCED = -2          # partition_size: equal-work split (OPTGQA_SPLIT_BALANCED)
OK = 0

_lib: Optional[ctypes.CDLL] = None


class OptGqaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


def load_library(path: str = LIB_PATH) -> ctypes.CDLL:
    """Load the C-ABI library and declare its signatures.  Raises if it is not built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: build it first (python -m paper_2505_02351_amd.build)")
    lib = ctypes.CDLL(path)
    vp, i32, i64, f32, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_float, ctypes.c_size_t
    lib.optgqa_abi_version.restype = i32
    lib.optgqa_abi_version.argtypes = []
    lib.optgqa_status_string.restype = ctypes.c_char_p
    lib.optgqa_status_string.argtypes = [i32]
    lib.optgqa_reshape_and_cache.restype = i32
    lib.optgqa_reshape_and_cache.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, i64, i64, i32, vp]
    lib.optgqa_paged_attention.restype = i32
    lib.optgqa_paged_attention.argtypes = [vp, vp, vp, vp, vp, vp, vp, f32, i32, i32, i32, i32, i32, i32, i32,
                                           i32, vp, sz, i32, vp]
    lib.optgqa_paged_attention_static.restype = i32
    lib.optgqa_paged_attention_static.argtypes = [vp, vp, vp, vp, vp, vp, vp, f32, i32, i32, i32, i32, i32, i32, i32,
                                                  i32, vp]
    lib.optgqa_shared_prefix_bundle.restype = i32
    lib.optgqa_shared_prefix_bundle.argtypes = [i32, i32, i32]
    lib.optgqa_shared_prefix_workspace_bytes.restype = sz
    lib.optgqa_shared_prefix_workspace_bytes.argtypes = [i32, i32, i32, i32, i32, i32]
    lib.optgqa_paged_attention_shared.restype = i32
    lib.optgqa_paged_attention_shared.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, f32, i32, i32, i32, i32, i32, i32,
                                                  i32, vp, sz, i32, vp]
    lib.optgqa_decode_step_shared.restype = i32
    lib.optgqa_decode_step_shared.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, f32, i32, i32, i32, i32, i32,
                                              i32, i32, i64, i64, vp, sz, i32, vp]
    lib.optgqa_validate_shared_prefix_host.restype = i32
    lib.optgqa_validate_shared_prefix_host.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32]
    lib.optgqa_set_kernel_events.restype = i32
    lib.optgqa_set_kernel_events.argtypes = [vp, vp]
    lib.optgqa_decode_step.restype = i32
    lib.optgqa_decode_step.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, f32, i32, i32, i32, i32, i32, i32, i32,
                                       i64, i64, vp, sz, i32, vp]
    lib.optgqa_reshape_and_cache_fp8.restype = i32
    lib.optgqa_reshape_and_cache_fp8.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, i64, i64, f32, f32, i32, vp]
    lib.optgqa_paged_attention_fp8.restype = i32
    lib.optgqa_paged_attention_fp8.argtypes = [vp, vp, vp, vp, vp, vp, vp, f32, f32, f32, i32, i32, i32, i32, i32,
                                               i32, i32, vp, sz, i32, vp]
    lib.optgqa_decode_step_fp8.restype = i32
    lib.optgqa_decode_step_fp8.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, f32, f32, f32, i32, i32, i32, i32, i32,
                                           i32, i32, i64, i64, vp, sz, i32, vp]
    lib.optgqa_paged_prefill_fp8.restype = i32
    lib.optgqa_paged_prefill_fp8.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, f32, f32, f32, i32, i32, i32, i32, i32,
                                             i32, i32, i32, vp]
    lib.optgqa_reshape_and_cache_fp8_heads.restype = i32
    lib.optgqa_reshape_and_cache_fp8_heads.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, i64, i64, vp, vp, i32, vp]
    lib.optgqa_paged_attention_fp8_heads.restype = i32
    lib.optgqa_paged_attention_fp8_heads.argtypes = [vp, vp, vp, vp, vp, vp, vp, f32, vp, vp, i32, i32, i32, i32, i32,
                                                     i32, i32, vp, sz, i32, vp]
    lib.optgqa_decode_step_fp8_heads.restype = i32
    lib.optgqa_decode_step_fp8_heads.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, f32, vp, vp, i32, i32, i32, i32,
                                                 i32, i32, i32, i64, i64, vp, sz, i32, vp]
    lib.optgqa_paged_prefill_fp8_heads.restype = i32
    lib.optgqa_paged_prefill_fp8_heads.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, f32, vp, vp, i32, i32, i32, i32, i32,
                                                   i32, i32, i32, vp]
    lib.optgqa_paged_attention_workspace_bytes.restype = sz
    lib.optgqa_paged_attention_workspace_bytes.argtypes = [i32, i32, i32, i32, i32, i32, i32,
                                                           ctypes.POINTER(ctypes.c_int)]
    lib.optgqa_paged_prefill.restype = i32
    lib.optgqa_paged_prefill.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, f32, i32, i32, i32, i32, i32, i32, i32,
                                         i32, vp]
    lib.optgqa_paged_attention_window.restype = i32
    lib.optgqa_paged_attention_window.argtypes = [vp, vp, vp, vp, vp, vp, vp, f32, i32, i32, i32, i32, i32, i32, i32,
                                                  i32, vp, sz, i32, vp]
    lib.optgqa_decode_step_window.restype = i32
    lib.optgqa_decode_step_window.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, f32, i32, i32, i32, i32, i32, i32,
                                              i32, i32, i64, i64, vp, sz, i32, vp]
    lib.optgqa_paged_prefill_window.restype = i32
    lib.optgqa_paged_prefill_window.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, f32, i32, i32, i32, i32, i32, i32,
                                                i32, i32, i32, vp]
    lib.optgqa_prompt_prefill.restype = i32
    lib.optgqa_prompt_prefill.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, f32, i32, i32, i32, i32, i32, i32, i32,
                                          i64, i64, i32, vp]
    lib.optgqa_prefill_step.restype = i32
    lib.optgqa_prefill_step.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, f32, i32, i32, i32, i32, i32, i32, i32,
                                        i64, i64, i32, vp]
    lib.optgqa_stream_probe.restype = i32
    lib.optgqa_stream_probe.argtypes = [vp, vp, sz, vp, vp, i32, i32, vp, vp]
    lib.optgqa_gather_kv.restype = i32
    lib.optgqa_gather_kv.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, i32, vp]
    lib.optgqa_validate_tables_host.restype = i32
    lib.optgqa_validate_tables_host.argtypes = [vp, vp, i32, i32, i32, i32]
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load_library().optgqa_status_string(int(status)).decode()


def abi_version() -> int:
    return int(load_library().optgqa_abi_version())


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float16:
        return F16
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"optgqa: expected float16 or bfloat16, got {t.dtype}")


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    handle = stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)
    return ctypes.c_void_p(handle)


def _check(status: int, where: str) -> None:
    if status != OK:
        raise OptGqaError(status, where)


def _dense(t: torch.Tensor, name: str) -> torch.Tensor:
    if not t.is_contiguous():
        raise ValueError(f"optgqa: {name} must be contiguous")
    return t


def _attn_typed(q, out, k_cache, v_cache, block_tables, context_lens, alibi_slopes, *, kv8=False, new=(),
                cu_q_lens=None) -> None:
    """_typed for the attention entry points: out, the new rows and (2-byte) caches as q, 8-bit caches
    uint8, tables / lengths / prefix sums int32, slopes float32, all on q's GPU."""
    caches = [("k_cache", k_cache), ("v_cache", v_cache)]
    same = [("out", out)] + [(n, t) for n, t in zip(("k_new", "v_new"), new)] + ([] if kv8 else caches)
    _typed(q, same=same, u8=caches if kv8 else (),
           i32=[("block_tables", block_tables), ("context_lens", context_lens), ("cu_q_lens", cu_q_lens)],
           f32=[("alibi_slopes", alibi_slopes)])


def _workspace(ws: Optional[torch.Tensor], ref: torch.Tensor) -> int:
    """Bytes of a caller-owned workspace (0 for None); it must be a dense tensor on ref's GPU."""
    if ws is None:
        return 0
    if not isinstance(ws, torch.Tensor) or not ws.is_cuda or ws.device != ref.device or not ws.is_contiguous():
        raise ValueError("optgqa: the workspace must be a contiguous tensor on the same GPU")
    return ws.numel() * ws.element_size()


def _typed(ref: torch.Tensor, *, same=(), u8=(), i32=(), i64=(), f32=()) -> None:
    """Refuse, before any pointer is taken, what the C ABI cannot check: the library reads raw
    device pointers, so a tensor of another element type or on another device would be misread
    (block ids and slots out of range make the kernels write out of bounds).  ``ref`` (q, or k for
    the cache writes) fixes the 2-byte type and the device; each group is a list of (name, tensor
    or None).  Element types first (TypeError), then devices (ValueError)."""
    _dtype_code(ref)
    groups = ((same, ref.dtype), (u8, torch.uint8), (i32, torch.int32), (i64, torch.int64), (f32, torch.float32))
    for group, want in groups:
        for name, t in group:
            if t is None:
                continue
            if not isinstance(t, torch.Tensor):
                raise TypeError(f"optgqa: {name} must be a torch.Tensor")
            if t.dtype != want:
                raise TypeError(f"optgqa: {name} must be {want}, got {t.dtype}")
    if not ref.is_cuda:
        raise ValueError("optgqa: tensors must live in GPU memory")
    for group, _ in groups:
        for name, t in group:
            if t is not None and t.device != ref.device:
                raise ValueError(f"optgqa: {name} is on {t.device}, expected {ref.device}")


def reshape_and_cache(k: torch.Tensor, v: torch.Tensor, k_cache: torch.Tensor, v_cache: torch.Tensor,
                      slot_mapping: torch.Tensor, stream=None) -> None:
    """optgqa_reshape_and_cache: scatter the new tokens' K/V rows into the paged caches."""
    lib = load_library()
    _typed(k, same=[("v", v), ("k_cache", k_cache), ("v_cache", v_cache)], i64=[("slot_mapping", slot_mapping)])
    NB, Hkv, bs, D = k_cache.shape
    T = int(slot_mapping.shape[0])
    _dense(k_cache, "k_cache"), _dense(v_cache, "v_cache"), _dense(slot_mapping, "slot_mapping")
    if T and (k.stride(-1) != 1 or k.stride(-2) != D or v.stride(-1) != 1 or v.stride(-2) != D):
        raise ValueError("optgqa: k and v must be dense in their last two dims")
    ks = int(k.stride(0)) if T else Hkv * D
    vs = int(v.stride(0)) if T else Hkv * D
    rc = lib.optgqa_reshape_and_cache(_ptr(k), _ptr(v), _ptr(k_cache), _ptr(v_cache), _ptr(slot_mapping),
                                      T, Hkv, D, bs, ks, vs, _dtype_code(k_cache), _stream(stream))
    _check(rc, "optgqa_reshape_and_cache")


def paged_attention_workspace_bytes(num_seqs: int, num_heads: int, num_kv_heads: int, head_dim: int,
                                    block_size: int, max_context_len: int, partition_size: int = 0):
    """optgqa_paged_attention_workspace_bytes -> (bytes, partition size the library would use)."""
    lib = load_library()
    chosen = ctypes.c_int(0)
    n = lib.optgqa_paged_attention_workspace_bytes(num_seqs, num_heads, num_kv_heads, head_dim, block_size,
                                                   max_context_len, partition_size, ctypes.byref(chosen))
    return int(n), int(chosen.value)


def paged_attention(out: torch.Tensor, q: torch.Tensor, k_cache: torch.Tensor, v_cache: torch.Tensor,
                    block_tables: torch.Tensor, context_lens: torch.Tensor,
                    alibi_slopes: Optional[torch.Tensor], scale: float, max_context_len: int,
                    partition_size: int = 0, workspace: Optional[torch.Tensor] = None, stream=None) -> None:
    """optgqa_paged_attention: decode attention of one query token per sequence."""
    lib = load_library()
    _attn_typed(q, out, k_cache, v_cache, block_tables, context_lens, alibi_slopes)
    B, Hq, D = q.shape
    NB, Hkv, bs, Dk = k_cache.shape
    if Dk != D or out.shape != q.shape:
        raise ValueError("optgqa: shape mismatch between q, out and the caches")
    for t, n in ((out, "out"), (q, "q"), (k_cache, "k_cache"), (v_cache, "v_cache"),
                 (block_tables, "block_tables"), (context_lens, "context_lens")):
        _dense(t, n)
    ws_bytes = _workspace(workspace, q)
    rc = lib.optgqa_paged_attention(_ptr(out), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(block_tables),
                                    _ptr(context_lens), _ptr(alibi_slopes), float(scale), B, Hq, Hkv, D, bs,
                                    int(block_tables.shape[1]), int(max_context_len), int(partition_size),
                                    _ptr(workspace), ws_bytes, _dtype_code(q), _stream(stream))
    _check(rc, "optgqa_paged_attention")


STATIC_SCRATCH_BYTES = 16 << 20    # OPTGQA_STATIC_SCRATCH_BYTES


def paged_attention_static(out: torch.Tensor, q: torch.Tensor, k_cache: torch.Tensor, v_cache: torch.Tensor,
                           block_tables: torch.Tensor, context_lens: torch.Tensor,
                           alibi_slopes: Optional[torch.Tensor], scale: float, max_context_len: int,
                           stream=None) -> None:
    """optgqa_paged_attention_static: decode attention whose split-context scratch is the library's
    own static device array (no workspace argument, nothing allocated)."""
    lib = load_library()
    _attn_typed(q, out, k_cache, v_cache, block_tables, context_lens, alibi_slopes)
    B, Hq, D = q.shape
    NB, Hkv, bs, Dk = k_cache.shape
    if Dk != D or out.shape != q.shape:
        raise ValueError("optgqa: shape mismatch between q, out and the caches")
    for t, n in ((out, "out"), (q, "q"), (k_cache, "k_cache"), (v_cache, "v_cache"),
                 (block_tables, "block_tables"), (context_lens, "context_lens")):
        _dense(t, n)
    rc = lib.optgqa_paged_attention_static(_ptr(out), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(block_tables),
                                           _ptr(context_lens), _ptr(alibi_slopes), float(scale), B, Hq, Hkv, D, bs,
                                           int(block_tables.shape[1]), int(max_context_len), _dtype_code(q),
                                           _stream(stream))
    _check(rc, "optgqa_paged_attention_static")


def shared_prefix_bundle(num_heads: int, num_kv_heads: int, head_dim: int) -> int:
    """optgqa_shared_prefix_bundle: sequences whose heads share one pass over a shared K/V tile."""
    m = int(load_library().optgqa_shared_prefix_bundle(num_heads, num_kv_heads, head_dim))
    if m <= 0:
        raise OptGqaError(m, "optgqa_shared_prefix_bundle")
    return m


def shared_prefix_workspace_bytes(num_seqs: int, num_heads: int, num_kv_heads: int, head_dim: int, block_size: int,
                                  max_context_len: int) -> int:
    """optgqa_shared_prefix_workspace_bytes."""
    return int(load_library().optgqa_shared_prefix_workspace_bytes(num_seqs, num_heads, num_kv_heads, head_dim,
                                                                   block_size, max_context_len))


def paged_attention_shared(out: torch.Tensor, q: torch.Tensor, k_cache: torch.Tensor, v_cache: torch.Tensor,
                           block_tables: torch.Tensor, context_lens: torch.Tensor, shared_blocks: torch.Tensor,
                           alibi_slopes: Optional[torch.Tensor], scale: float, max_context_len: int,
                           workspace: Optional[torch.Tensor], stream=None) -> None:
    """optgqa_paged_attention_shared: decode attention that reads a bundle's shared prefix blocks once."""
    lib = load_library()
    _attn_typed(q, out, k_cache, v_cache, block_tables, context_lens, alibi_slopes)
    _typed(q, i32=[("shared_blocks", shared_blocks)])
    B, Hq, D = q.shape
    NB, Hkv, bs, Dk = k_cache.shape
    if Dk != D or out.shape != q.shape or shared_blocks.shape != (B,):
        raise ValueError("optgqa: shape mismatch between q, out, shared_blocks and the caches")
    for t, n in ((out, "out"), (q, "q"), (k_cache, "k_cache"), (v_cache, "v_cache"),
                 (block_tables, "block_tables"), (context_lens, "context_lens"), (shared_blocks, "shared_blocks")):
        _dense(t, n)
    ws_bytes = _workspace(workspace, q)
    rc = lib.optgqa_paged_attention_shared(_ptr(out), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(block_tables),
                                           _ptr(context_lens), _ptr(shared_blocks), _ptr(alibi_slopes), float(scale),
                                           B, Hq, Hkv, D, bs, int(block_tables.shape[1]), int(max_context_len),
                                           _ptr(workspace), ws_bytes, _dtype_code(q), _stream(stream))
    _check(rc, "optgqa_paged_attention_shared")


def decode_step_shared(out: torch.Tensor, q: torch.Tensor, k_new: torch.Tensor, v_new: torch.Tensor,
                       k_cache: torch.Tensor, v_cache: torch.Tensor, block_tables: torch.Tensor,
                       context_lens: torch.Tensor, shared_blocks: torch.Tensor,
                       alibi_slopes: Optional[torch.Tensor], scale: float, max_context_len: int,
                       workspace: Optional[torch.Tensor], stream=None) -> None:
    """optgqa_decode_step_shared: the step's cache write and decode attention, shared prefix blocks
    read once per bundle of sequences."""
    lib = load_library()
    _attn_typed(q, out, k_cache, v_cache, block_tables, context_lens, alibi_slopes, new=(k_new, v_new))
    _typed(q, i32=[("shared_blocks", shared_blocks)])
    B, Hq, D = q.shape
    NB, Hkv, bs, Dk = k_cache.shape
    if (Dk != D or out.shape != q.shape or k_new.shape != (B, Hkv, D) or v_new.shape != (B, Hkv, D)
            or shared_blocks.shape != (B,)):
        raise ValueError("optgqa: shape mismatch between q, out, the new rows, shared_blocks and the caches")
    for t, n in ((out, "out"), (q, "q"), (k_cache, "k_cache"), (v_cache, "v_cache"),
                 (block_tables, "block_tables"), (context_lens, "context_lens"), (shared_blocks, "shared_blocks")):
        _dense(t, n)
    if B and (k_new.stride(-1) != 1 or k_new.stride(-2) != D or v_new.stride(-1) != 1 or v_new.stride(-2) != D):
        raise ValueError("optgqa: k_new and v_new must be dense in their last two dims")
    ks = int(k_new.stride(0)) if B else Hkv * D
    vs = int(v_new.stride(0)) if B else Hkv * D
    ws_bytes = _workspace(workspace, q)
    rc = lib.optgqa_decode_step_shared(_ptr(out), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(k_cache), _ptr(v_cache),
                                       _ptr(block_tables), _ptr(context_lens), _ptr(shared_blocks),
                                       _ptr(alibi_slopes), float(scale), B, Hq, Hkv, D, bs,
                                       int(block_tables.shape[1]), int(max_context_len), ks, vs, _ptr(workspace),
                                       ws_bytes, _dtype_code(q), _stream(stream))
    _check(rc, "optgqa_decode_step_shared")


def validate_shared_prefix_host(block_tables, context_lens, shared_blocks, block_size: int, bundle: int,
                                new_tokens: int) -> int:
    """optgqa_validate_shared_prefix_host on host numpy int32 arrays; returns the status code."""
    import numpy as np
    lib = load_library()
    bt = np.ascontiguousarray(block_tables, dtype=np.int32)
    cl = np.ascontiguousarray(context_lens, dtype=np.int32)
    sb = np.ascontiguousarray(shared_blocks, dtype=np.int32)
    return int(lib.optgqa_validate_shared_prefix_host(bt.ctypes.data_as(ctypes.c_void_p),
                                                      cl.ctypes.data_as(ctypes.c_void_p),
                                                      sb.ctypes.data_as(ctypes.c_void_p), int(cl.shape[0]),
                                                      int(bt.shape[1]), int(block_size), int(bundle), int(new_tokens)))


def set_kernel_events(start: Optional[torch.cuda.Event], stop: Optional[torch.cuda.Event]) -> None:
    """optgqa_set_kernel_events: record the two events around the KV-streaming kernel of later calls
    (None, None switches it off).  The events must have been recorded once already, so that
    torch has created the underlying HIP events."""
    lib = load_library()
    if start is None and stop is None:
        _check(lib.optgqa_set_kernel_events(None, None), "optgqa_set_kernel_events")
        return
    a, b = int(start.cuda_event), int(stop.cuda_event)
    if not a or not b:
        raise ValueError("optgqa: record the events once before handing them over")
    _check(lib.optgqa_set_kernel_events(ctypes.c_void_p(a), ctypes.c_void_p(b)), "optgqa_set_kernel_events")


def decode_step(out: torch.Tensor, q: torch.Tensor, k_new: torch.Tensor, v_new: torch.Tensor,
                k_cache: torch.Tensor, v_cache: torch.Tensor, block_tables: torch.Tensor,
                context_lens: torch.Tensor, alibi_slopes: Optional[torch.Tensor], scale: float,
                max_context_len: int, workspace: Optional[torch.Tensor] = None, stream=None) -> None:
    """optgqa_decode_step: the step's cache write and its decode attention in one call."""
    lib = load_library()
    _attn_typed(q, out, k_cache, v_cache, block_tables, context_lens, alibi_slopes, new=(k_new, v_new))
    B, Hq, D = q.shape
    NB, Hkv, bs, Dk = k_cache.shape
    if Dk != D or out.shape != q.shape or k_new.shape != (B, Hkv, D) or v_new.shape != (B, Hkv, D):
        raise ValueError("optgqa: shape mismatch between q, out, the new rows and the caches")
    for t, n in ((out, "out"), (q, "q"), (k_cache, "k_cache"), (v_cache, "v_cache"),
                 (block_tables, "block_tables"), (context_lens, "context_lens")):
        _dense(t, n)
    if B and (k_new.stride(-1) != 1 or k_new.stride(-2) != D or v_new.stride(-1) != 1 or v_new.stride(-2) != D):
        raise ValueError("optgqa: k_new and v_new must be dense in their last two dims")
    ks = int(k_new.stride(0)) if B else Hkv * D
    vs = int(v_new.stride(0)) if B else Hkv * D
    ws_bytes = _workspace(workspace, q)
    rc = lib.optgqa_decode_step(_ptr(out), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(k_cache), _ptr(v_cache),
                                _ptr(block_tables), _ptr(context_lens), _ptr(alibi_slopes), float(scale), B, Hq,
                                Hkv, D, bs, int(block_tables.shape[1]), int(max_context_len), ks, vs,
                                _ptr(workspace), ws_bytes, _dtype_code(q), _stream(stream))
    _check(rc, "optgqa_decode_step")


def reshape_and_cache_fp8(k: torch.Tensor, v: torch.Tensor, k_cache: torch.Tensor, v_cache: torch.Tensor,
                          slot_mapping: torch.Tensor, k_scale: float, v_scale: float, stream=None) -> None:
    """optgqa_reshape_and_cache_fp8: quantise the new tokens' K/V rows to E4M3 codes in the paged
    caches (uint8 tensors [NB, Hkv, bs, D])."""
    lib = load_library()
    _typed(k, same=[("v", v)], u8=[("k_cache", k_cache), ("v_cache", v_cache)], i64=[("slot_mapping", slot_mapping)])
    NB, Hkv, bs, D = k_cache.shape
    T = int(slot_mapping.shape[0])
    _dense(k_cache, "k_cache"), _dense(v_cache, "v_cache"), _dense(slot_mapping, "slot_mapping")
    if T and (k.stride(-1) != 1 or k.stride(-2) != D or v.stride(-1) != 1 or v.stride(-2) != D):
        raise ValueError("optgqa: k and v must be dense in their last two dims")
    ks = int(k.stride(0)) if T else Hkv * D
    vs = int(v.stride(0)) if T else Hkv * D
    rc = lib.optgqa_reshape_and_cache_fp8(_ptr(k), _ptr(v), _ptr(k_cache), _ptr(v_cache), _ptr(slot_mapping),
                                          T, Hkv, D, bs, ks, vs, float(k_scale), float(v_scale),
                                          _dtype_code(k), _stream(stream))
    _check(rc, "optgqa_reshape_and_cache_fp8")


def paged_attention_fp8(out: torch.Tensor, q: torch.Tensor, k_cache: torch.Tensor, v_cache: torch.Tensor,
                        block_tables: torch.Tensor, context_lens: torch.Tensor,
                        alibi_slopes: Optional[torch.Tensor], scale: float, k_scale: float, v_scale: float,
                        max_context_len: int, workspace: Optional[torch.Tensor], stream=None) -> None:
    """optgqa_paged_attention_fp8: decode attention over E4M3 caches (uint8 tensors)."""
    lib = load_library()
    _attn_typed(q, out, k_cache, v_cache, block_tables, context_lens, alibi_slopes, kv8=True)
    B, Hq, D = q.shape
    NB, Hkv, bs, Dk = k_cache.shape
    if Dk != D or out.shape != q.shape:
        raise ValueError("optgqa: shape mismatch between q, out and the caches")
    for t, n in ((out, "out"), (q, "q"), (k_cache, "k_cache"), (v_cache, "v_cache"),
                 (block_tables, "block_tables"), (context_lens, "context_lens")):
        _dense(t, n)
    ws_bytes = _workspace(workspace, q)
    rc = lib.optgqa_paged_attention_fp8(_ptr(out), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(block_tables),
                                        _ptr(context_lens), _ptr(alibi_slopes), float(scale), float(k_scale),
                                        float(v_scale), B, Hq, Hkv, D, bs, int(block_tables.shape[1]),
                                        int(max_context_len), _ptr(workspace), ws_bytes, _dtype_code(q),
                                        _stream(stream))
    _check(rc, "optgqa_paged_attention_fp8")


def decode_step_fp8(out: torch.Tensor, q: torch.Tensor, k_new: torch.Tensor, v_new: torch.Tensor,
                    k_cache: torch.Tensor, v_cache: torch.Tensor, block_tables: torch.Tensor,
                    context_lens: torch.Tensor, alibi_slopes: Optional[torch.Tensor], scale: float, k_scale: float,
                    v_scale: float, max_context_len: int, workspace: Optional[torch.Tensor], stream=None) -> None:
    """optgqa_decode_step_fp8: quantising cache write of the step's new tokens and decode attention over
    the E4M3 caches in one call."""
    lib = load_library()
    _attn_typed(q, out, k_cache, v_cache, block_tables, context_lens, alibi_slopes, kv8=True, new=(k_new, v_new))
    B, Hq, D = q.shape
    NB, Hkv, bs, Dk = k_cache.shape
    if Dk != D or out.shape != q.shape or k_new.shape != (B, Hkv, D) or v_new.shape != (B, Hkv, D):
        raise ValueError("optgqa: shape mismatch between q, out, the new rows and the caches")
    for t, n in ((out, "out"), (q, "q"), (k_cache, "k_cache"), (v_cache, "v_cache"),
                 (block_tables, "block_tables"), (context_lens, "context_lens")):
        _dense(t, n)
    if B and (k_new.stride(-1) != 1 or k_new.stride(-2) != D or v_new.stride(-1) != 1 or v_new.stride(-2) != D):
        raise ValueError("optgqa: k_new and v_new must be dense in their last two dims")
    ks = int(k_new.stride(0)) if B else Hkv * D
    vs = int(v_new.stride(0)) if B else Hkv * D
    ws_bytes = _workspace(workspace, q)
    rc = lib.optgqa_decode_step_fp8(_ptr(out), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(k_cache), _ptr(v_cache),
                                    _ptr(block_tables), _ptr(context_lens), _ptr(alibi_slopes), float(scale),
                                    float(k_scale), float(v_scale), B, Hq, Hkv, D, bs, int(block_tables.shape[1]),
                                    int(max_context_len), ks, vs, _ptr(workspace), ws_bytes, _dtype_code(q),
                                    _stream(stream))
    _check(rc, "optgqa_decode_step_fp8")


def paged_prefill_fp8(out: torch.Tensor, q: torch.Tensor, k_cache: torch.Tensor, v_cache: torch.Tensor,
                      block_tables: torch.Tensor, context_lens: torch.Tensor, cu_q_lens: torch.Tensor,
                      alibi_slopes: Optional[torch.Tensor], scale: float, k_scale: float, v_scale: float,
                      max_q_len: int, stream=None) -> None:
    """optgqa_paged_prefill_fp8: causal + ALiBi attention of the new tokens over E4M3 caches."""
    lib = load_library()
    _attn_typed(q, out, k_cache, v_cache, block_tables, context_lens, alibi_slopes, kv8=True, cu_q_lens=cu_q_lens)
    T, Hq, D = q.shape
    NB, Hkv, bs, Dk = k_cache.shape
    if Dk != D or out.shape != q.shape:
        raise ValueError("optgqa: shape mismatch between q, out and the caches")
    for t, n in ((out, "out"), (q, "q"), (k_cache, "k_cache"), (v_cache, "v_cache"),
                 (block_tables, "block_tables"), (context_lens, "context_lens"), (cu_q_lens, "cu_q_lens")):
        _dense(t, n)
    rc = lib.optgqa_paged_prefill_fp8(_ptr(out), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(block_tables),
                                      _ptr(context_lens), _ptr(cu_q_lens), _ptr(alibi_slopes), float(scale),
                                      float(k_scale), float(v_scale), int(context_lens.shape[0]), Hq, Hkv, D, bs,
                                      int(block_tables.shape[1]), int(max_q_len), _dtype_code(q), _stream(stream))
    _check(rc, "optgqa_paged_prefill_fp8")


def _head_scales(ref: torch.Tensor, k_cache: torch.Tensor, k_scales, v_scales) -> None:
    """Per-KV-head scale arrays: float32, dense, [Hkv], on ref's GPU."""
    _typed(ref, f32=[("k_scales", k_scales), ("v_scales", v_scales)])
    hkv = k_cache.shape[1]
    for t, n in ((k_scales, "k_scales"), (v_scales, "v_scales")):
        if t is None or tuple(t.shape) != (hkv,) or not t.is_contiguous():
            raise ValueError(f"optgqa: {n} must be a dense tensor of {hkv} values, one per KV head")


def reshape_and_cache_fp8_heads(k: torch.Tensor, v: torch.Tensor, k_cache: torch.Tensor, v_cache: torch.Tensor,
                          slot_mapping: torch.Tensor, k_scales: torch.Tensor, v_scales: torch.Tensor, stream=None) -> None:
    """optgqa_reshape_and_cache_fp8_heads (one scale pair per KV head, float32 device tensors [Hkv]): quantise the new tokens' K/V rows to E4M3 codes in the paged
    caches (uint8 tensors [NB, Hkv, bs, D])."""
    lib = load_library()
    _head_scales(k, k_cache, k_scales, v_scales)
    _typed(k, same=[("v", v)], u8=[("k_cache", k_cache), ("v_cache", v_cache)], i64=[("slot_mapping", slot_mapping)])
    NB, Hkv, bs, D = k_cache.shape
    T = int(slot_mapping.shape[0])
    _dense(k_cache, "k_cache"), _dense(v_cache, "v_cache"), _dense(slot_mapping, "slot_mapping")
    if T and (k.stride(-1) != 1 or k.stride(-2) != D or v.stride(-1) != 1 or v.stride(-2) != D):
        raise ValueError("optgqa: k and v must be dense in their last two dims")
    ks = int(k.stride(0)) if T else Hkv * D
    vs = int(v.stride(0)) if T else Hkv * D
    rc = lib.optgqa_reshape_and_cache_fp8_heads(_ptr(k), _ptr(v), _ptr(k_cache), _ptr(v_cache), _ptr(slot_mapping),
                                          T, Hkv, D, bs, ks, vs, _ptr(k_scales), _ptr(v_scales),
                                          _dtype_code(k), _stream(stream))
    _check(rc, "optgqa_reshape_and_cache_fp8_heads")


def paged_attention_fp8_heads(out: torch.Tensor, q: torch.Tensor, k_cache: torch.Tensor, v_cache: torch.Tensor,
                        block_tables: torch.Tensor, context_lens: torch.Tensor,
                        alibi_slopes: Optional[torch.Tensor], scale: float, k_scales: torch.Tensor, v_scales: torch.Tensor,
                        max_context_len: int, workspace: Optional[torch.Tensor], stream=None) -> None:
    """optgqa_paged_attention_fp8_heads (one scale pair per KV head, float32 device tensors [Hkv]): decode attention over E4M3 caches (uint8 tensors)."""
    lib = load_library()
    _head_scales(q, k_cache, k_scales, v_scales)
    _attn_typed(q, out, k_cache, v_cache, block_tables, context_lens, alibi_slopes, kv8=True)
    B, Hq, D = q.shape
    NB, Hkv, bs, Dk = k_cache.shape
    if Dk != D or out.shape != q.shape:
        raise ValueError("optgqa: shape mismatch between q, out and the caches")
    for t, n in ((out, "out"), (q, "q"), (k_cache, "k_cache"), (v_cache, "v_cache"),
                 (block_tables, "block_tables"), (context_lens, "context_lens")):
        _dense(t, n)
    ws_bytes = _workspace(workspace, q)
    rc = lib.optgqa_paged_attention_fp8_heads(_ptr(out), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(block_tables),
                                        _ptr(context_lens), _ptr(alibi_slopes), float(scale), _ptr(k_scales),
                                        _ptr(v_scales), B, Hq, Hkv, D, bs, int(block_tables.shape[1]),
                                        int(max_context_len), _ptr(workspace), ws_bytes, _dtype_code(q),
                                        _stream(stream))
    _check(rc, "optgqa_paged_attention_fp8_heads")


def decode_step_fp8_heads(out: torch.Tensor, q: torch.Tensor, k_new: torch.Tensor, v_new: torch.Tensor,
                    k_cache: torch.Tensor, v_cache: torch.Tensor, block_tables: torch.Tensor,
                    context_lens: torch.Tensor, alibi_slopes: Optional[torch.Tensor], scale: float, k_scales: torch.Tensor,
                    v_scales: torch.Tensor, max_context_len: int, workspace: Optional[torch.Tensor], stream=None) -> None:
    """optgqa_decode_step_fp8_heads (one scale pair per KV head, float32 device tensors [Hkv]): quantising cache write of the step's new tokens and decode attention over
    the E4M3 caches in one call."""
    lib = load_library()
    _head_scales(q, k_cache, k_scales, v_scales)
    _attn_typed(q, out, k_cache, v_cache, block_tables, context_lens, alibi_slopes, kv8=True, new=(k_new, v_new))
    B, Hq, D = q.shape
    NB, Hkv, bs, Dk = k_cache.shape
    if Dk != D or out.shape != q.shape or k_new.shape != (B, Hkv, D) or v_new.shape != (B, Hkv, D):
        raise ValueError("optgqa: shape mismatch between q, out, the new rows and the caches")
    for t, n in ((out, "out"), (q, "q"), (k_cache, "k_cache"), (v_cache, "v_cache"),
                 (block_tables, "block_tables"), (context_lens, "context_lens")):
        _dense(t, n)
    if B and (k_new.stride(-1) != 1 or k_new.stride(-2) != D or v_new.stride(-1) != 1 or v_new.stride(-2) != D):
        raise ValueError("optgqa: k_new and v_new must be dense in their last two dims")
    ks = int(k_new.stride(0)) if B else Hkv * D
    vs = int(v_new.stride(0)) if B else Hkv * D
    ws_bytes = _workspace(workspace, q)
    rc = lib.optgqa_decode_step_fp8_heads(_ptr(out), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(k_cache), _ptr(v_cache),
                                    _ptr(block_tables), _ptr(context_lens), _ptr(alibi_slopes), float(scale),
                                    _ptr(k_scales), _ptr(v_scales), B, Hq, Hkv, D, bs, int(block_tables.shape[1]),
                                    int(max_context_len), ks, vs, _ptr(workspace), ws_bytes, _dtype_code(q),
                                    _stream(stream))
    _check(rc, "optgqa_decode_step_fp8_heads")


def paged_prefill_fp8_heads(out: torch.Tensor, q: torch.Tensor, k_cache: torch.Tensor, v_cache: torch.Tensor,
                      block_tables: torch.Tensor, context_lens: torch.Tensor, cu_q_lens: torch.Tensor,
                      alibi_slopes: Optional[torch.Tensor], scale: float, k_scales: torch.Tensor, v_scales: torch.Tensor,
                      max_q_len: int, stream=None) -> None:
    """optgqa_paged_prefill_fp8_heads (one scale pair per KV head, float32 device tensors [Hkv]): causal + ALiBi attention of the new tokens over E4M3 caches."""
    lib = load_library()
    _head_scales(q, k_cache, k_scales, v_scales)
    _attn_typed(q, out, k_cache, v_cache, block_tables, context_lens, alibi_slopes, kv8=True, cu_q_lens=cu_q_lens)
    T, Hq, D = q.shape
    NB, Hkv, bs, Dk = k_cache.shape
    if Dk != D or out.shape != q.shape:
        raise ValueError("optgqa: shape mismatch between q, out and the caches")
    for t, n in ((out, "out"), (q, "q"), (k_cache, "k_cache"), (v_cache, "v_cache"),
                 (block_tables, "block_tables"), (context_lens, "context_lens"), (cu_q_lens, "cu_q_lens")):
        _dense(t, n)
    rc = lib.optgqa_paged_prefill_fp8_heads(_ptr(out), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(block_tables),
                                      _ptr(context_lens), _ptr(cu_q_lens), _ptr(alibi_slopes), float(scale),
                                      _ptr(k_scales), _ptr(v_scales), int(context_lens.shape[0]), Hq, Hkv, D, bs,
                                      int(block_tables.shape[1]), int(max_q_len), _dtype_code(q), _stream(stream))
    _check(rc, "optgqa_paged_prefill_fp8_heads")


def paged_prefill(out: torch.Tensor, q: torch.Tensor, k_cache: torch.Tensor, v_cache: torch.Tensor,
                  block_tables: torch.Tensor, context_lens: torch.Tensor, cu_q_lens: torch.Tensor,
                  alibi_slopes: Optional[torch.Tensor], scale: float, max_q_len: int, stream=None) -> None:
    """optgqa_paged_prefill: causal + ALiBi attention of the new tokens over the paged cache."""
    lib = load_library()
    _attn_typed(q, out, k_cache, v_cache, block_tables, context_lens, alibi_slopes, cu_q_lens=cu_q_lens)
    T, Hq, D = q.shape
    NB, Hkv, bs, Dk = k_cache.shape
    if Dk != D or out.shape != q.shape:
        raise ValueError("optgqa: shape mismatch between q, out and the caches")
    for t, n in ((out, "out"), (q, "q"), (k_cache, "k_cache"), (v_cache, "v_cache"),
                 (block_tables, "block_tables"), (context_lens, "context_lens"), (cu_q_lens, "cu_q_lens")):
        _dense(t, n)
    B = int(context_lens.shape[0])
    rc = lib.optgqa_paged_prefill(_ptr(out), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(block_tables),
                                  _ptr(context_lens), _ptr(cu_q_lens), _ptr(alibi_slopes), float(scale), B, Hq,
                                  Hkv, D, bs, int(block_tables.shape[1]), int(max_q_len), _dtype_code(q),
                                  _stream(stream))
    _check(rc, "optgqa_paged_prefill")


def paged_attention_window(out: torch.Tensor, q: torch.Tensor, k_cache: torch.Tensor, v_cache: torch.Tensor,
                           block_tables: torch.Tensor, context_lens: torch.Tensor,
                           alibi_slopes: Optional[torch.Tensor], scale: float, window: int, max_context_len: int,
                           workspace: Optional[torch.Tensor], stream=None) -> None:
    """optgqa_paged_attention_window: decode attention over the last ``window`` tokens."""
    lib = load_library()
    _attn_typed(q, out, k_cache, v_cache, block_tables, context_lens, alibi_slopes)
    B, Hq, D = q.shape
    NB, Hkv, bs, Dk = k_cache.shape
    if Dk != D or out.shape != q.shape:
        raise ValueError("optgqa: shape mismatch between q, out and the caches")
    for t, n in ((out, "out"), (q, "q"), (k_cache, "k_cache"), (v_cache, "v_cache"),
                 (block_tables, "block_tables"), (context_lens, "context_lens")):
        _dense(t, n)
    ws_bytes = _workspace(workspace, q)
    rc = lib.optgqa_paged_attention_window(_ptr(out), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(block_tables),
                                           _ptr(context_lens), _ptr(alibi_slopes), float(scale), int(window), B, Hq,
                                           Hkv, D, bs, int(block_tables.shape[1]), int(max_context_len),
                                           _ptr(workspace), ws_bytes, _dtype_code(q), _stream(stream))
    _check(rc, "optgqa_paged_attention_window")


def decode_step_window(out: torch.Tensor, q: torch.Tensor, k_new: torch.Tensor, v_new: torch.Tensor,
                       k_cache: torch.Tensor, v_cache: torch.Tensor, block_tables: torch.Tensor,
                       context_lens: torch.Tensor, alibi_slopes: Optional[torch.Tensor], scale: float, window: int,
                       max_context_len: int, workspace: Optional[torch.Tensor], stream=None) -> None:
    """optgqa_decode_step_window: the step's cache write and its windowed decode attention."""
    lib = load_library()
    _attn_typed(q, out, k_cache, v_cache, block_tables, context_lens, alibi_slopes, new=(k_new, v_new))
    B, Hq, D = q.shape
    NB, Hkv, bs, Dk = k_cache.shape
    if Dk != D or out.shape != q.shape or k_new.shape != (B, Hkv, D) or v_new.shape != (B, Hkv, D):
        raise ValueError("optgqa: shape mismatch between q, out, the new rows and the caches")
    for t, n in ((out, "out"), (q, "q"), (k_cache, "k_cache"), (v_cache, "v_cache"),
                 (block_tables, "block_tables"), (context_lens, "context_lens")):
        _dense(t, n)
    if B and (k_new.stride(-1) != 1 or k_new.stride(-2) != D or v_new.stride(-1) != 1 or v_new.stride(-2) != D):
        raise ValueError("optgqa: k_new and v_new must be dense in their last two dims")
    ks = int(k_new.stride(0)) if B else Hkv * D
    vs = int(v_new.stride(0)) if B else Hkv * D
    ws_bytes = _workspace(workspace, q)
    rc = lib.optgqa_decode_step_window(_ptr(out), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(k_cache), _ptr(v_cache),
                                       _ptr(block_tables), _ptr(context_lens), _ptr(alibi_slopes), float(scale),
                                       int(window), B, Hq, Hkv, D, bs, int(block_tables.shape[1]),
                                       int(max_context_len), ks, vs, _ptr(workspace), ws_bytes, _dtype_code(q),
                                       _stream(stream))
    _check(rc, "optgqa_decode_step_window")


def paged_prefill_window(out: torch.Tensor, q: torch.Tensor, k_cache: torch.Tensor, v_cache: torch.Tensor,
                         block_tables: torch.Tensor, context_lens: torch.Tensor, cu_q_lens: torch.Tensor,
                         alibi_slopes: Optional[torch.Tensor], scale: float, window: int, max_q_len: int,
                         stream=None) -> None:
    """optgqa_paged_prefill_window: causal attention of the new tokens, each over its last ``window`` keys."""
    lib = load_library()
    _attn_typed(q, out, k_cache, v_cache, block_tables, context_lens, alibi_slopes, cu_q_lens=cu_q_lens)
    T, Hq, D = q.shape
    NB, Hkv, bs, Dk = k_cache.shape
    if Dk != D or out.shape != q.shape:
        raise ValueError("optgqa: shape mismatch between q, out and the caches")
    for t, n in ((out, "out"), (q, "q"), (k_cache, "k_cache"), (v_cache, "v_cache"),
                 (block_tables, "block_tables"), (context_lens, "context_lens"), (cu_q_lens, "cu_q_lens")):
        _dense(t, n)
    B = int(context_lens.shape[0])
    rc = lib.optgqa_paged_prefill_window(_ptr(out), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(block_tables),
                                         _ptr(context_lens), _ptr(cu_q_lens), _ptr(alibi_slopes), float(scale),
                                         int(window), B, Hq, Hkv, D, bs, int(block_tables.shape[1]), int(max_q_len),
                                         _dtype_code(q), _stream(stream))
    _check(rc, "optgqa_paged_prefill_window")


def prompt_prefill(out: torch.Tensor, q: torch.Tensor, k: torch.Tensor, v: torch.Tensor,
                   k_cache: Optional[torch.Tensor], v_cache: Optional[torch.Tensor],
                   block_tables: Optional[torch.Tensor], cu_seq_lens: torch.Tensor,
                   alibi_slopes: Optional[torch.Tensor], scale: float, max_seq_len: int, stream=None) -> None:
    """optgqa_prompt_prefill: causal (+ ALiBi) attention of whole prompts over their own K / V, storing
    K / V into the paged caches in the same launch when the caches are given."""
    lib = load_library()
    _typed(q, same=[("out", out), ("k", k), ("v", v), ("k_cache", k_cache), ("v_cache", v_cache)],
           i32=[("block_tables", block_tables), ("cu_seq_lens", cu_seq_lens)], f32=[("alibi_slopes", alibi_slopes)])
    T, Hq, D = q.shape
    Hkv = k.shape[1]
    if out.shape != q.shape or k.shape != (T, Hkv, D) or v.shape != (T, Hkv, D):
        raise ValueError("optgqa: shape mismatch between q, out, k and v")
    _dense(out, "out"), _dense(q, "q"), _dense(cu_seq_lens, "cu_seq_lens")
    if T and (k.stride(-1) != 1 or k.stride(-2) != D or v.stride(-1) != 1 or v.stride(-2) != D):
        raise ValueError("optgqa: k and v must be dense in their last two dims")
    ks = int(k.stride(0)) if T else Hkv * D
    vs = int(v.stride(0)) if T else Hkv * D
    bs, mb = 0, 0
    if k_cache is not None:
        NB, Hkv2, bs, Dk = k_cache.shape
        if Dk != D or Hkv2 != Hkv or block_tables is None:
            raise ValueError("optgqa: cache shape / block tables do not match k and v")
        _dense(k_cache, "k_cache"), _dense(v_cache, "v_cache"), _dense(block_tables, "block_tables")
        mb = int(block_tables.shape[1])
    rc = lib.optgqa_prompt_prefill(_ptr(out), _ptr(q), _ptr(k), _ptr(v), _ptr(k_cache), _ptr(v_cache),
                                   _ptr(block_tables), _ptr(cu_seq_lens), _ptr(alibi_slopes), float(scale),
                                   int(cu_seq_lens.shape[0]) - 1, Hq, Hkv, D, int(bs), mb, int(max_seq_len), ks, vs,
                                   _dtype_code(q), _stream(stream))
    _check(rc, "optgqa_prompt_prefill")


def prefill_step(out: torch.Tensor, q: torch.Tensor, k_new: torch.Tensor, v_new: torch.Tensor,
                 k_cache: torch.Tensor, v_cache: torch.Tensor, block_tables: torch.Tensor,
                 context_lens: torch.Tensor, cu_q_lens: torch.Tensor, alibi_slopes: Optional[torch.Tensor],
                 scale: float, max_q_len: int, stream=None) -> None:
    """optgqa_prefill_step: store the new tokens' K / V rows into the paged caches and attend over the
    caches, in one launch."""
    lib = load_library()
    _typed(q, same=[("out", out), ("k_new", k_new), ("v_new", v_new), ("k_cache", k_cache), ("v_cache", v_cache)],
           i32=[("block_tables", block_tables), ("context_lens", context_lens), ("cu_q_lens", cu_q_lens)],
           f32=[("alibi_slopes", alibi_slopes)])
    T, Hq, D = q.shape
    NB, Hkv, bs, Dk = k_cache.shape
    if (out.shape != q.shape or Dk != D or v_cache.shape != k_cache.shape or k_new.shape != (T, Hkv, D)
            or v_new.shape != (T, Hkv, D) or cu_q_lens.shape[0] != context_lens.shape[0] + 1
            or block_tables.shape[0] != context_lens.shape[0]):
        raise ValueError("optgqa: shape mismatch between q, out, the new rows, the tables and the caches")
    _dense(out, "out"), _dense(q, "q"), _dense(k_cache, "k_cache"), _dense(v_cache, "v_cache")
    _dense(block_tables, "block_tables"), _dense(context_lens, "context_lens"), _dense(cu_q_lens, "cu_q_lens")
    if T and (k_new.stride(-1) != 1 or k_new.stride(-2) != D or v_new.stride(-1) != 1 or v_new.stride(-2) != D):
        raise ValueError("optgqa: k_new and v_new must be dense in their last two dims")
    ks = int(k_new.stride(0)) if T else Hkv * D
    vs = int(v_new.stride(0)) if T else Hkv * D
    rc = lib.optgqa_prefill_step(_ptr(out), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(k_cache), _ptr(v_cache),
                                 _ptr(block_tables), _ptr(context_lens), _ptr(cu_q_lens), _ptr(alibi_slopes),
                                 float(scale), int(context_lens.shape[0]), Hq, Hkv, D, int(bs),
                                 int(block_tables.shape[1]), int(max_q_len), ks, vs, _dtype_code(q), _stream(stream))
    _check(rc, "optgqa_prefill_step")


def gather_kv(k_out: torch.Tensor, v_out: torch.Tensor, k_cache: torch.Tensor, v_cache: torch.Tensor,
              block_tables: torch.Tensor, context_lens: torch.Tensor, stream=None) -> None:
    """optgqa_gather_kv: un-page the caches into [B, max_context_len, Hkv, D] (bit copy)."""
    lib = load_library()
    _typed(k_cache, same=[("k_out", k_out), ("v_out", v_out), ("v_cache", v_cache)],
           i32=[("block_tables", block_tables), ("context_lens", context_lens)])
    B, Lmax, Hkv, D = k_out.shape
    NB, Hkv2, bs, D2 = k_cache.shape
    if (Hkv, D) != (Hkv2, D2) or v_out.shape != k_out.shape:
        raise ValueError("optgqa: shape mismatch in gather_kv")
    for t, n in ((k_out, "k_out"), (v_out, "v_out"), (k_cache, "k_cache"), (v_cache, "v_cache"),
                 (block_tables, "block_tables"), (context_lens, "context_lens")):
        _dense(t, n)
    rc = lib.optgqa_gather_kv(_ptr(k_out), _ptr(v_out), _ptr(k_cache), _ptr(v_cache), _ptr(block_tables),
                              _ptr(context_lens), B, Hkv, D, bs, int(block_tables.shape[1]), Lmax,
                              _dtype_code(k_cache), _stream(stream))
    _check(rc, "optgqa_gather_kv")


def stream_probe(k_pool: torch.Tensor, v_pool: torch.Tensor, tile_list_host, num_workgroups: int,
                 tiles_per_wave: int, sink: torch.Tensor, tile_list_dev: Optional[torch.Tensor] = None,
                 stream=None) -> torch.Tensor:
    """optgqa_stream_probe: stream 4 KiB pieces of two device buffers with the decode kernels' load
    pattern and no arithmetic.  ``tile_list_host`` is a numpy int32 array
    [num_workgroups * 4 * tiles_per_wave]; returns the device copy of it (pass it back in as
    ``tile_list_dev`` for repeated launches)."""
    import numpy as np
    lib = load_library()
    host = np.ascontiguousarray(tile_list_host, dtype=np.int32)
    if host.size != num_workgroups * 4 * tiles_per_wave:
        raise ValueError("optgqa: tile list size does not match the launch")
    dev = tile_list_dev if tile_list_dev is not None else torch.from_numpy(host).to(k_pool.device)
    nbytes = k_pool.numel() * k_pool.element_size()
    if v_pool.numel() * v_pool.element_size() != nbytes:
        raise ValueError("optgqa: the two pools must have the same size")
    rc = lib.optgqa_stream_probe(_ptr(k_pool), _ptr(v_pool), nbytes, _ptr(dev),
                                 host.ctypes.data_as(ctypes.c_void_p), int(num_workgroups), int(tiles_per_wave),
                                 _ptr(sink), _stream(stream))
    _check(rc, "optgqa_stream_probe")
    return dev


def validate_tables_host(block_tables, context_lens, block_size: int, num_blocks: int) -> int:
    """optgqa_validate_tables_host on host numpy int32 arrays; returns the status code."""
    import numpy as np
    lib = load_library()
    bt = np.ascontiguousarray(block_tables, dtype=np.int32)
    cl = np.ascontiguousarray(context_lens, dtype=np.int32)
    return int(lib.optgqa_validate_tables_host(bt.ctypes.data_as(ctypes.c_void_p),
                                               cl.ctypes.data_as(ctypes.c_void_p), int(cl.shape[0]),
                                               int(bt.shape[1]), int(block_size), int(num_blocks)))
