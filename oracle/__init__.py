"""fp64 CPU oracle for paged GQA + ALiBi attention -- TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper around ``optgqa_oracle.c`` (plain C, fp64, the paper's
definitions written out; see the header of that file for the passages it
follows).  Only the tests, the smoke check and the bench's CPU-baseline leg may
import this package.  It never imports the HIP library or its binding.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "optgqa_oracle.c")
_SRC_E4M3 = os.path.join(_HERE, "optgqa_oracle_e4m3.c")        # 8-bit KV-cache variant
_SRC_WINDOW = os.path.join(_HERE, "optgqa_oracle_window.c")    # causal + sliding-window masks
_SRC_PROMPT = os.path.join(_HERE, "optgqa_oracle_prompt.c")    # whole prompt over its own K/V
_LIB = os.path.join(_HERE, "liboptgqa_oracle.so")

DTYPES = {"f16": 0, "bf16": 1}


def build(src: str = _SRC, out: str = _LIB, force: bool = True, src_e4m3: str = _SRC_E4M3,
          src_window: str = _SRC_WINDOW, src_prompt: str = _SRC_PROMPT) -> str:
    """Compile the oracle with gcc (OpenMP over independent (sequence, head) rows)."""
    newest = max(os.path.getmtime(src), os.path.getmtime(src_e4m3), os.path.getmtime(src_window),
                 os.path.getmtime(src_prompt))
    if force or not os.path.exists(out) or os.path.getmtime(out) < newest:
        tmp = out + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp",
                               "-ffp-contract=off", "-o", tmp, src, src_e4m3, src_window, src_prompt, "-lm"])
        os.replace(tmp, out)
    return out


def load(path: Optional[str] = None) -> ctypes.CDLL:
    if path is None:
        path = build(force=False)
    lib = ctypes.CDLL(path)
    lib.oracle_num_threads.restype = ctypes.c_int
    return lib


_lib: Optional[ctypes.CDLL] = None


def _get() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        _lib = load()
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dt) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=dt)


def num_threads() -> int:
    return int(_get().oracle_num_threads())


def set_num_threads(n: int) -> None:
    _get().oracle_set_num_threads(ctypes.c_int(n))


def reshape_and_cache(k, v, k_cache, v_cache, slot_mapping, lib=None) -> None:
    """In place on k_cache / v_cache (uint16 [NB, Hkv, bs, D])."""
    lib = lib or _get()
    assert k_cache.dtype == np.uint16 and v_cache.dtype == np.uint16
    assert k_cache.flags.c_contiguous and v_cache.flags.c_contiguous
    k, v = _c(k, np.uint16), _c(v, np.uint16)
    slots = _c(slot_mapping, np.int64)
    T = slots.shape[0]
    NB, Hkv, bs, D = k_cache.shape
    stride = Hkv * D
    lib.oracle_reshape_and_cache(_p(k), _p(v), _p(k_cache), _p(v_cache), _p(slots),
                                 ctypes.c_int(T), ctypes.c_int(Hkv), ctypes.c_int(D),
                                 ctypes.c_int(bs), ctypes.c_int64(stride), ctypes.c_int64(stride))


def _common(q, k_cache, block_tables, context_lens, slopes):
    q = _c(q, np.uint16)
    bt = _c(block_tables, np.int32)
    cl = _c(context_lens, np.int32)
    sl = None if slopes is None else _c(slopes, np.float32)
    NB, Hkv, bs, D = k_cache.shape
    assert k_cache.dtype == np.uint16 and k_cache.flags.c_contiguous
    return q, bt, cl, sl, Hkv, bs, D


def paged_attention(q, k_cache, v_cache, block_tables, context_lens, slopes, scale, dtype,
                    rows: Optional[Sequence] = None, lib=None) -> np.ndarray:
    """Decode attention in fp64.  Returns [B, Hq, D], or [n_rows, D] when ``rows`` lists
    (sequence, head) pairs."""
    lib = lib or _get()
    q, bt, cl, sl, Hkv, bs, D = _common(q, k_cache, block_tables, context_lens, slopes)
    B, Hq, _ = q.shape
    MB = bt.shape[1]
    assert v_cache.dtype == np.uint16 and v_cache.flags.c_contiguous
    if rows is None:
        out = np.zeros((B, Hq, D), dtype=np.float64)
        lib.oracle_paged_attention(_p(out), _p(q), _p(k_cache), _p(v_cache), _p(bt), _p(cl), _p(sl),
                                   ctypes.c_float(scale), ctypes.c_int(B), ctypes.c_int(Hq),
                                   ctypes.c_int(Hkv), ctypes.c_int(D), ctypes.c_int(bs),
                                   ctypes.c_int(MB), ctypes.c_int(DTYPES[dtype]))
        return out
    rows = np.asarray(rows, dtype=np.int32).reshape(-1, 2)
    rs, rh = _c(rows[:, 0], np.int32), _c(rows[:, 1], np.int32)
    out = np.zeros((rows.shape[0], D), dtype=np.float64)
    lib.oracle_paged_attention_rows(_p(out), _p(rs), _p(rh), ctypes.c_int(rows.shape[0]), _p(q),
                                    _p(k_cache), _p(v_cache), _p(bt), _p(cl), _p(sl),
                                    ctypes.c_float(scale), ctypes.c_int(Hq), ctypes.c_int(Hkv),
                                    ctypes.c_int(D), ctypes.c_int(bs), ctypes.c_int(MB),
                                    ctypes.c_int(DTYPES[dtype]))
    return out


def paged_attention_partitioned(q, k_cache, v_cache, block_tables, context_lens, slopes, scale,
                                dtype, partition_size: int, lib=None) -> np.ndarray:
    lib = lib or _get()
    q, bt, cl, sl, Hkv, bs, D = _common(q, k_cache, block_tables, context_lens, slopes)
    B, Hq, _ = q.shape
    out = np.zeros((B, Hq, D), dtype=np.float64)
    lib.oracle_paged_attention_partitioned(_p(out), _p(q), _p(k_cache), _p(v_cache), _p(bt), _p(cl),
                                           _p(sl), ctypes.c_float(scale), ctypes.c_int(B),
                                           ctypes.c_int(Hq), ctypes.c_int(Hkv), ctypes.c_int(D),
                                           ctypes.c_int(bs), ctypes.c_int(bt.shape[1]),
                                           ctypes.c_int(partition_size),
                                           ctypes.c_int(DTYPES[dtype]))
    return out


def paged_prefill(q, k_cache, v_cache, block_tables, context_lens, cu_q_lens, slopes, scale, dtype,
                  rows: Optional[Sequence] = None, lib=None) -> np.ndarray:
    """Causal + ALiBi attention of the new tokens over the paged cache, fp64.
    Returns [T, Hq, D], or [n_rows, D] when ``rows`` lists (query token, head) pairs."""
    lib = lib or _get()
    q, bt, cl, sl, Hkv, bs, D = _common(q, k_cache, block_tables, context_lens, slopes)
    cu = _c(cu_q_lens, np.int32)
    T, Hq, _ = q.shape
    B = cl.shape[0]
    assert int(cu[-1]) == T
    if rows is None:
        out = np.zeros((T, Hq, D), dtype=np.float64)
        lib.oracle_paged_prefill(_p(out), _p(q), _p(k_cache), _p(v_cache), _p(bt), _p(cl), _p(cu),
                                 _p(sl), ctypes.c_float(scale), ctypes.c_int(B), ctypes.c_int(Hq),
                                 ctypes.c_int(Hkv), ctypes.c_int(D), ctypes.c_int(bs),
                                 ctypes.c_int(bt.shape[1]), ctypes.c_int(DTYPES[dtype]))
        return out
    rows = np.asarray(rows, dtype=np.int32).reshape(-1, 2)
    rt, rh = _c(rows[:, 0], np.int32), _c(rows[:, 1], np.int32)
    out = np.zeros((rows.shape[0], D), dtype=np.float64)
    lib.oracle_paged_prefill_rows(_p(out), _p(rt), _p(rh), ctypes.c_int(rows.shape[0]), _p(q),
                                  _p(k_cache), _p(v_cache), _p(bt), _p(cl), _p(cu), _p(sl),
                                  ctypes.c_float(scale), ctypes.c_int(B), ctypes.c_int(Hq),
                                  ctypes.c_int(Hkv), ctypes.c_int(D), ctypes.c_int(bs),
                                  ctypes.c_int(bt.shape[1]), ctypes.c_int(DTYPES[dtype]))
    return out


# ---------------------------------------------------------------------------------------------
# 8-bit (E4M3) KV-cache variant: optgqa_oracle_e4m3.c
# ---------------------------------------------------------------------------------------------
def e4m3_values(lib=None) -> np.ndarray:
    """Value of each of the 256 codes (fp64; the two NaN codes give NaN)."""
    lib = lib or _get()
    out = np.zeros(256, dtype=np.float64)
    lib.oracle_e4m3_values(_p(out))
    return out


def e4m3_nearest(x, lib=None) -> np.ndarray:
    """Nearest code (ties to even, saturating at +-448, NaN -> 0x7f) of each float32."""
    lib = lib or _get()
    x = _c(x, np.float32).ravel()
    out = np.zeros(x.shape[0], dtype=np.uint8)
    lib.oracle_e4m3_nearest(_p(x), ctypes.c_int(x.shape[0]), _p(out))
    return out


def reshape_and_cache_e4m3(k, v, k_cache, v_cache, slot_mapping, k_scale, v_scale, dtype, lib=None) -> None:
    """Quantising cache write, in place on k_cache / v_cache (uint8 [NB, Hkv, bs, D])."""
    lib = lib or _get()
    assert k_cache.dtype == np.uint8 and v_cache.dtype == np.uint8
    assert k_cache.flags.c_contiguous and v_cache.flags.c_contiguous
    k, v = _c(k, np.uint16), _c(v, np.uint16)
    slots = _c(slot_mapping, np.int64)
    NB, Hkv, bs, D = k_cache.shape
    stride = Hkv * D
    lib.oracle_reshape_and_cache_e4m3(_p(k), _p(v), _p(k_cache), _p(v_cache), _p(slots),
                                      ctypes.c_int(slots.shape[0]), ctypes.c_int(Hkv), ctypes.c_int(D),
                                      ctypes.c_int(bs), ctypes.c_int64(stride), ctypes.c_int64(stride),
                                      ctypes.c_float(k_scale), ctypes.c_float(v_scale),
                                      ctypes.c_int(DTYPES[dtype]))


def paged_attention_e4m3(q, k_cache, v_cache, block_tables, context_lens, slopes, scale, k_scale, v_scale,
                         dtype, rows: Optional[Sequence] = None, lib=None) -> np.ndarray:
    """Decode attention over an E4M3 cache in fp64: [B, Hq, D], or [n_rows, D] for listed
    (sequence, head) pairs."""
    lib = lib or _get()
    q = _c(q, np.uint16)
    bt, cl = _c(block_tables, np.int32), _c(context_lens, np.int32)
    sl = None if slopes is None else _c(slopes, np.float32)
    assert k_cache.dtype == np.uint8 and v_cache.dtype == np.uint8
    assert k_cache.flags.c_contiguous and v_cache.flags.c_contiguous
    NB, Hkv, bs, D = k_cache.shape
    B, Hq, _ = q.shape
    if rows is None:
        n, rs, rh = B * Hq, None, None
        out = np.zeros((B, Hq, D), dtype=np.float64)
    else:
        rows = np.asarray(rows, dtype=np.int32).reshape(-1, 2)
        n, rs, rh = rows.shape[0], _c(rows[:, 0], np.int32), _c(rows[:, 1], np.int32)
        out = np.zeros((n, D), dtype=np.float64)
    lib.oracle_paged_attention_e4m3(_p(out), _p(rs), _p(rh), ctypes.c_int(n), _p(q), _p(k_cache), _p(v_cache),
                                    _p(bt), _p(cl), _p(sl), ctypes.c_float(scale), ctypes.c_float(k_scale),
                                    ctypes.c_float(v_scale), ctypes.c_int(Hq), ctypes.c_int(Hkv),
                                    ctypes.c_int(D), ctypes.c_int(bs), ctypes.c_int(bt.shape[1]),
                                    ctypes.c_int(DTYPES[dtype]))
    return out


def paged_prefill_e4m3(q, k_cache, v_cache, block_tables, context_lens, cu_q_lens, slopes, scale, k_scale,
                       v_scale, dtype, rows: Optional[Sequence] = None, lib=None) -> np.ndarray:
    """Causal + ALiBi attention of the new tokens over an E4M3 cache, fp64: [T, Hq, D], or [n_rows, D]
    for listed (query token, head) pairs."""
    lib = lib or _get()
    q = _c(q, np.uint16)
    bt, cl, cu = _c(block_tables, np.int32), _c(context_lens, np.int32), _c(cu_q_lens, np.int32)
    sl = None if slopes is None else _c(slopes, np.float32)
    assert k_cache.dtype == np.uint8 and v_cache.dtype == np.uint8
    assert k_cache.flags.c_contiguous and v_cache.flags.c_contiguous
    NB, Hkv, bs, D = k_cache.shape
    T, Hq, _ = q.shape
    assert int(cu[-1]) == T
    if rows is None:
        n, rt, rh = T * Hq, None, None
        out = np.zeros((T, Hq, D), dtype=np.float64)
    else:
        rows = np.asarray(rows, dtype=np.int32).reshape(-1, 2)
        n, rt, rh = rows.shape[0], _c(rows[:, 0], np.int32), _c(rows[:, 1], np.int32)
        out = np.zeros((n, D), dtype=np.float64)
    lib.oracle_paged_prefill_e4m3(_p(out), _p(rt), _p(rh), ctypes.c_int(n), _p(q), _p(k_cache), _p(v_cache),
                                  _p(bt), _p(cl), _p(cu), _p(sl), ctypes.c_float(scale), ctypes.c_float(k_scale),
                                  ctypes.c_float(v_scale), ctypes.c_int(cl.shape[0]), ctypes.c_int(Hq),
                                  ctypes.c_int(Hkv), ctypes.c_int(D), ctypes.c_int(bs), ctypes.c_int(bt.shape[1]),
                                  ctypes.c_int(DTYPES[dtype]))
    return out


def _scales(x, n: int) -> np.ndarray:
    a = np.ascontiguousarray(x, dtype=np.float32).reshape(-1)
    assert a.shape == (n,), f"expected {n} per-KV-head scales"
    return a


def reshape_and_cache_e4m3_heads(k, v, k_cache, v_cache, slot_mapping, k_scales, v_scales, dtype, lib=None) -> None:
    """Quantising cache write with one scale pair per KV head (arrays [Hkv]), in place."""
    lib = lib or _get()
    assert k_cache.dtype == np.uint8 and v_cache.dtype == np.uint8
    assert k_cache.flags.c_contiguous and v_cache.flags.c_contiguous
    k, v = _c(k, np.uint16), _c(v, np.uint16)
    slots = _c(slot_mapping, np.int64)
    NB, Hkv, bs, D = k_cache.shape
    ks, vs = _scales(k_scales, Hkv), _scales(v_scales, Hkv)
    stride = Hkv * D
    lib.oracle_reshape_and_cache_e4m3_heads(_p(k), _p(v), _p(k_cache), _p(v_cache), _p(slots),
                                            ctypes.c_int(slots.shape[0]), ctypes.c_int(Hkv), ctypes.c_int(D),
                                            ctypes.c_int(bs), ctypes.c_int64(stride), ctypes.c_int64(stride),
                                            _p(ks), _p(vs), ctypes.c_int(DTYPES[dtype]))


def paged_attention_e4m3_heads(q, k_cache, v_cache, block_tables, context_lens, slopes, scale, k_scales, v_scales,
                               dtype, rows: Optional[Sequence] = None, lib=None) -> np.ndarray:
    """Decode attention over an E4M3 cache with per-KV-head scales, fp64."""
    lib = lib or _get()
    q = _c(q, np.uint16)
    bt, cl = _c(block_tables, np.int32), _c(context_lens, np.int32)
    sl = None if slopes is None else _c(slopes, np.float32)
    assert k_cache.dtype == np.uint8 and v_cache.dtype == np.uint8
    assert k_cache.flags.c_contiguous and v_cache.flags.c_contiguous
    NB, Hkv, bs, D = k_cache.shape
    ks, vs = _scales(k_scales, Hkv), _scales(v_scales, Hkv)
    B, Hq, _ = q.shape
    if rows is None:
        n, rs, rh = B * Hq, None, None
        out = np.zeros((B, Hq, D), dtype=np.float64)
    else:
        rows = np.asarray(rows, dtype=np.int32).reshape(-1, 2)
        n, rs, rh = rows.shape[0], _c(rows[:, 0], np.int32), _c(rows[:, 1], np.int32)
        out = np.zeros((n, D), dtype=np.float64)
    lib.oracle_paged_attention_e4m3_heads(_p(out), _p(rs), _p(rh), ctypes.c_int(n), _p(q), _p(k_cache), _p(v_cache),
                                          _p(bt), _p(cl), _p(sl), ctypes.c_float(scale), _p(ks), _p(vs),
                                          ctypes.c_int(Hq), ctypes.c_int(Hkv), ctypes.c_int(D), ctypes.c_int(bs),
                                          ctypes.c_int(bt.shape[1]), ctypes.c_int(DTYPES[dtype]))
    return out


def paged_prefill_e4m3_heads(q, k_cache, v_cache, block_tables, context_lens, cu_q_lens, slopes, scale, k_scales,
                             v_scales, dtype, rows: Optional[Sequence] = None, lib=None) -> np.ndarray:
    """Causal + ALiBi attention of the new tokens over an E4M3 cache with per-KV-head scales, fp64."""
    lib = lib or _get()
    q = _c(q, np.uint16)
    bt, cl, cu = _c(block_tables, np.int32), _c(context_lens, np.int32), _c(cu_q_lens, np.int32)
    sl = None if slopes is None else _c(slopes, np.float32)
    assert k_cache.dtype == np.uint8 and v_cache.dtype == np.uint8
    assert k_cache.flags.c_contiguous and v_cache.flags.c_contiguous
    NB, Hkv, bs, D = k_cache.shape
    ks, vs = _scales(k_scales, Hkv), _scales(v_scales, Hkv)
    T, Hq, _ = q.shape
    assert int(cu[-1]) == T
    if rows is None:
        n, rt, rh = T * Hq, None, None
        out = np.zeros((T, Hq, D), dtype=np.float64)
    else:
        rows = np.asarray(rows, dtype=np.int32).reshape(-1, 2)
        n, rt, rh = rows.shape[0], _c(rows[:, 0], np.int32), _c(rows[:, 1], np.int32)
        out = np.zeros((n, D), dtype=np.float64)
    lib.oracle_paged_prefill_e4m3_heads(_p(out), _p(rt), _p(rh), ctypes.c_int(n), _p(q), _p(k_cache), _p(v_cache),
                                        _p(bt), _p(cl), _p(cu), _p(sl), ctypes.c_float(scale), _p(ks), _p(vs),
                                        ctypes.c_int(cl.shape[0]), ctypes.c_int(Hq), ctypes.c_int(Hkv),
                                        ctypes.c_int(D), ctypes.c_int(bs), ctypes.c_int(bt.shape[1]),
                                        ctypes.c_int(DTYPES[dtype]))
    return out


# ---------------------------------------------------------------------------------------------
# causal + sliding-window masks: optgqa_oracle_window.c
# ---------------------------------------------------------------------------------------------
def paged_attention_window(q, k_cache, v_cache, block_tables, context_lens, slopes, scale, window, dtype,
                           rows: Optional[Sequence] = None, lib=None) -> np.ndarray:
    """Decode attention over the last ``window`` tokens (<= 0: all), fp64: [B, Hq, D], or
    [n_rows, D] for listed (sequence, head) pairs."""
    lib = lib or _get()
    q, bt, cl, sl, Hkv, bs, D = _common(q, k_cache, block_tables, context_lens, slopes)
    assert v_cache.dtype == np.uint16 and v_cache.flags.c_contiguous
    B, Hq, _ = q.shape
    if rows is None:
        n, rs, rh = B * Hq, None, None
        out = np.zeros((B, Hq, D), dtype=np.float64)
    else:
        rows = np.asarray(rows, dtype=np.int32).reshape(-1, 2)
        n, rs, rh = rows.shape[0], _c(rows[:, 0], np.int32), _c(rows[:, 1], np.int32)
        out = np.zeros((n, D), dtype=np.float64)
    lib.oracle_paged_attention_window(_p(out), _p(rs), _p(rh), ctypes.c_int(n), _p(q), _p(k_cache), _p(v_cache),
                                      _p(bt), _p(cl), _p(sl), ctypes.c_float(scale), ctypes.c_int(int(window)),
                                      ctypes.c_int(Hq), ctypes.c_int(Hkv), ctypes.c_int(D), ctypes.c_int(bs),
                                      ctypes.c_int(bt.shape[1]), ctypes.c_int(DTYPES[dtype]))
    return out


def paged_prefill_window(q, k_cache, v_cache, block_tables, context_lens, cu_q_lens, slopes, scale, window, dtype,
                         rows: Optional[Sequence] = None, lib=None) -> np.ndarray:
    """Causal attention of the new tokens, each over its last ``window`` keys (<= 0: all), fp64:
    [T, Hq, D], or [n_rows, D] for listed (query token, head) pairs."""
    lib = lib or _get()
    q, bt, cl, sl, Hkv, bs, D = _common(q, k_cache, block_tables, context_lens, slopes)
    assert v_cache.dtype == np.uint16 and v_cache.flags.c_contiguous
    cu = _c(cu_q_lens, np.int32)
    T, Hq, _ = q.shape
    assert int(cu[-1]) == T
    if rows is None:
        n, rt, rh = T * Hq, None, None
        out = np.zeros((T, Hq, D), dtype=np.float64)
    else:
        rows = np.asarray(rows, dtype=np.int32).reshape(-1, 2)
        n, rt, rh = rows.shape[0], _c(rows[:, 0], np.int32), _c(rows[:, 1], np.int32)
        out = np.zeros((n, D), dtype=np.float64)
    lib.oracle_paged_prefill_window(_p(out), _p(rt), _p(rh), ctypes.c_int(n), _p(q), _p(k_cache), _p(v_cache),
                                    _p(bt), _p(cl), _p(cu), _p(sl), ctypes.c_float(scale), ctypes.c_int(int(window)),
                                    ctypes.c_int(cl.shape[0]), ctypes.c_int(Hq), ctypes.c_int(Hkv), ctypes.c_int(D),
                                    ctypes.c_int(bs), ctypes.c_int(bt.shape[1]), ctypes.c_int(DTYPES[dtype]))
    return out


# ---------------------------------------------------------------------------------------------
# whole prompt over its own K / V (caches empty): optgqa_oracle_prompt.c
# ---------------------------------------------------------------------------------------------
def prompt_attention(q, k, v, cu_seq_lens, slopes, scale, dtype, rows: Optional[Sequence] = None,
                     lib=None) -> np.ndarray:
    """Causal (+ ALiBi) attention of every prompt token over the earlier tokens of its own sequence,
    from dense q [T, Hq, D], k / v [T, Hkv, D], fp64: [T, Hq, D], or [n_rows, D] for listed
    (token, head) pairs."""
    lib = lib or _get()
    q, k, v = _c(q, np.uint16), _c(k, np.uint16), _c(v, np.uint16)
    cu = _c(cu_seq_lens, np.int32)
    sl = None if slopes is None else _c(slopes, np.float32)
    T, Hq, D = q.shape
    Hkv = k.shape[1]
    assert k.shape == (T, Hkv, D) and v.shape == (T, Hkv, D) and int(cu[-1]) == T
    if rows is None:
        n, rt, rh = T * Hq, None, None
        out = np.zeros((T, Hq, D), dtype=np.float64)
    else:
        rows = np.asarray(rows, dtype=np.int32).reshape(-1, 2)
        n, rt, rh = rows.shape[0], _c(rows[:, 0], np.int32), _c(rows[:, 1], np.int32)
        out = np.zeros((n, D), dtype=np.float64)
    lib.oracle_prompt_attention(_p(out), _p(rt), _p(rh), ctypes.c_int(n), _p(q), _p(k), _p(v), _p(cu), _p(sl),
                                ctypes.c_float(scale), ctypes.c_int(cu.shape[0] - 1), ctypes.c_int(Hq),
                                ctypes.c_int(Hkv), ctypes.c_int(D), ctypes.c_int(DTYPES[dtype]))
    return out
