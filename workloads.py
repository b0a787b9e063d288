"""Seeded synthetic inputs for the paged GQA + ALiBi attention path.

This module only *draws and arranges* inputs: random values, context lengths,
block-table permutations, slot mappings and the cache image that exists before
a step runs.  It holds none of the method's arithmetic (no scores, no softmax)
and imports neither the CPU oracle nor the HIP library; both are fed from here
so that they see the very same bits.  The one place that touches the cache
layout is index arrangement of inputs: ``make_case`` scatters the drawn values
into the pool and lifts the step's new rows out of it, and ``all_token_rows``
reads them back through ``slot // block_size, slot % block_size`` to hand the
same logical tokens to caches of another element type.  Neither is what a
cache-write result is compared with: those come from the oracle alone.

All 2-byte tensors are carried as ``numpy.uint16`` bit patterns (IEEE fp16 or
bfloat16), so nothing downstream depends on a framework's dtype support.

Shapes follow the paper's forward pass (Alg. 1 / Alg. 2: Q, K, V, the caches
C_K, C_V and the metadata M) with the paged cache laid out as
``[num_blocks, num_kv_heads, block_size, head_dim]``.

Recipe (fixed draw order for a given seed):
  context_lens -> physical block permutation -> q -> K values -> V values.
K/V values are drawn per *logical* token and then scattered to the physical
blocks the permutation assigned, so two cases that differ only in
``perm_seed`` hold identical logical content under different block tables.
Every pool block no sequence owns, and the rows of a partial last block
beyond the context, are filled with NaN bit patterns.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Optional

import numpy as np

F16 = "f16"
BF16 = "bf16"

NAN_BITS = {F16: np.uint16(0x7E00), BF16: np.uint16(0x7FC0)}


# --------------------------------------------------------------------------
# 2-byte encodings of drawn values (input quantisation, not method arithmetic)
# --------------------------------------------------------------------------
def to_bits(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round float32 values to fp16 / bf16 (nearest-even) and return uint16 bits."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == F16:
        return x.astype(np.float16).view(np.uint16)
    if dtype == BF16:
        u = x.view(np.uint32)
        rounded = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
        return rounded.astype(np.uint16)
    raise ValueError(f"unknown dtype {dtype!r}")


def from_bits(bits: np.ndarray, dtype: str) -> np.ndarray:
    """Exact widening of uint16 fp16 / bf16 bit patterns to float64 (for reports and tests)."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    if dtype == F16:
        with np.errstate(invalid="ignore"):
            return bits.view(np.float16).astype(np.float64)
    if dtype == BF16:
        with np.errstate(invalid="ignore"):     # signalling-NaN patterns are legal inputs here
            return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    raise ValueError(f"unknown dtype {dtype!r}")


def alibi_slopes(num_heads: int) -> np.ndarray:
    """Slopes 2^(-8(h+1)/Hq), h = 0..Hq-1, evaluated in fp64 and stored as fp32."""
    h = np.arange(1, num_heads + 1, dtype=np.float64)
    return np.exp2(-8.0 * h / num_heads).astype(np.float32)


# --------------------------------------------------------------------------
# Workload table: the five configurations this build is measured on
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class Config:
    name: str
    kind: str                 # "decode" | "prefill"
    dtype: str
    batch: int
    num_heads: int            # Hq
    num_kv_heads: int         # Hkv
    head_dim: int             # D
    block_size: int           # bs
    num_blocks: int           # NB, size of the physical pool
    ctx_lo: int               # context length range (inclusive), incl. the new tokens
    ctx_hi: int
    q_len: int = 1            # new tokens per sequence (1 = decode)
    partition_size: int = 0   # 0 = library chooses
    seed: int = 0


CONFIGS: Dict[str, Config] = {
    "C1": Config("C1", "decode", F16, 1, 8, 2, 64, 16, 8, 128, 128, seed=0),
    "C2": Config("C2", "decode", F16, 16, 32, 8, 128, 16, 4096, 256, 2048, seed=1),
    "C3": Config("C3", "decode", BF16, 64, 32, 4, 128, 32, 20000, 1024, 8192, seed=2),
    "C3-all8k": Config("C3-all8k", "decode", BF16, 64, 32, 4, 128, 32, 20000, 8192, 8192, seed=2),
    "C4": Config("C4", "decode", F16, 4, 64, 8, 128, 16, 16384, 32768, 32768,
                 partition_size=512, seed=3),
    "C5": Config("C5", "prefill", BF16, 8, 32, 8, 128, 16, 2560, 2560, 2560, q_len=512, seed=4),
    # the same sequences as whole prompts with empty caches (every token new)
    "C5-prompt": Config("C5-prompt", "prefill", BF16, 8, 32, 8, 128, 16, 2560, 2560, 2560, q_len=2560, seed=5),
}


@dataclass
class Case:
    """One batch of inputs, as the state *before* the step's cache write."""
    cfg: Config
    dtype: str
    context_lens: np.ndarray      # int32 [B], includes the new tokens
    q_lens: np.ndarray            # int32 [B], new tokens per sequence
    cu_q_lens: np.ndarray         # int32 [B+1]
    block_tables: np.ndarray      # int32 [B, MB], unused entries -1
    q: np.ndarray                 # uint16 [T, Hq, D]
    k_new: np.ndarray             # uint16 [T, Hkv, D]  the new tokens' keys
    v_new: np.ndarray             # uint16 [T, Hkv, D]
    slot_mapping: np.ndarray      # int64 [T]  physical_block * bs + row
    k_cache: np.ndarray           # uint16 [NB, Hkv, bs, D]; new tokens' rows still NaN
    v_cache: np.ndarray           # uint16 [NB, Hkv, bs, D]
    slopes: np.ndarray            # float32 [Hq]
    scale: np.float32
    partition_size: int
    extras: dict = field(default_factory=dict)

    @property
    def num_tokens(self) -> int:
        return int(self.q.shape[0])

    @property
    def max_context_len(self) -> int:
        return int(self.context_lens.max()) if self.context_lens.size else 0

    @property
    def max_q_len(self) -> int:
        return int(self.q_lens.max()) if self.q_lens.size else 0

    def kv_bytes(self) -> int:
        """K and V bytes of the context, each element counted once per KV head."""
        c = self.cfg
        return int(2 * int(self.context_lens.astype(np.int64).sum()) * c.num_kv_heads * c.head_dim * 2)


def all_token_rows(case: "Case", include_new: bool = True):
    """The 2-byte K and V rows of every token of the batch, sequence after sequence in logical
    order, and each token's slot (physical_block * block_size + row): ``(k [N, Hkv, D],
    v [N, Hkv, D], slots [N] int64)``.  Plain indexing of the cache image (the new tokens' rows are
    put back first unless ``include_new`` is False, in which case those tokens are left out).
    Used to build caches of another element type from the same logical content."""
    cfg, bs = case.cfg, case.cfg.block_size
    kc, vc = case.k_cache, case.v_cache
    if include_new:
        kc, vc = kc.copy(), vc.copy()
        s = case.slot_mapping
        kc[s // bs, :, s % bs, :] = case.k_new
        vc[s // bs, :, s % bs, :] = case.v_new
    ks, vs, slots = [], [], []
    for b in range(cfg.batch):
        n = int(case.context_lens[b]) - (0 if include_new else int(case.q_lens[b]))
        j = np.arange(max(n, 0))
        blk = case.block_tables[b, j // bs].astype(np.int64)
        ks.append(kc[blk, :, j % bs, :])
        vs.append(vc[blk, :, j % bs, :])
        slots.append(blk * bs + j % bs)
    return np.concatenate(ks), np.concatenate(vs), np.concatenate(slots).astype(np.int64)


def share_prefix_blocks(case: "Case", group: int, fraction: float = 0.9) -> int:
    """Rewrite the block tables so that the sequences of every run of ``group`` consecutive
    sequences share their leading blocks with the run's first one (a common prompt prefix served
    from the same physical blocks): ``fraction`` of the run's shortest cached length, rounded
    down to whole blocks, never the block that receives a new token.  Returns the number of
    context tokens that now alias another sequence's.  Pure index work."""
    bs = case.cfg.block_size
    shared = 0
    for g0 in range(0, case.cfg.batch, group):
        members = list(range(g0, min(g0 + group, case.cfg.batch)))
        cached = case.context_lens[members].astype(np.int64) - case.q_lens[members]
        nblk = int(max(int(cached.min()), 0) * fraction) // bs
        for m in members[1:]:
            case.block_tables[m, :nblk] = case.block_tables[g0, :nblk]
            shared += nblk * bs
    return shared


def share_prefix_in_bundles(case: "Case", bundle: int, seed: int, share_prob: float = 0.8) -> np.ndarray:
    """Ragged prefix sharing in aligned bundles of ``bundle`` consecutive sequences: every non-leading
    member shares, with probability ``share_prob``, a random number of leading whole cached blocks
    (at least one, at most what both it and the bundle's first sequence hold in the cache, never a
    block that receives a new token) with the bundle's first sequence; its block table is rewritten
    to alias those blocks.  Returns ``shared_blocks`` (int32 [B], 0 = shares nothing).  Pure index work."""
    bs, B = case.cfg.block_size, case.cfg.batch
    rng = np.random.default_rng(seed)
    shared = np.zeros(B, dtype=np.int32)
    cached = case.context_lens.astype(np.int64) - case.q_lens
    for b in range(B):
        b0 = b - b % bundle
        if b == b0 or rng.random() >= share_prob:
            continue
        most = int(min(cached[b], cached[b0])) // bs
        if most < 1:
            continue
        n = int(rng.integers(1, most + 1))
        if rng.random() < 0.3:
            n = most                                    # often everything that can be shared
        case.block_tables[b, :n] = case.block_tables[b0, :n]
        shared[b] = n
    return shared


def bundle_shared_blocks(case: "Case", bundle: int) -> np.ndarray:
    """``shared_blocks`` for aligned bundles of ``bundle`` sequences, read off the block tables as they
    are: for every non-leading member, the number of leading table entries equal to those of the
    bundle's first sequence, limited to whole blocks both hold in the cache.  Pure index work (what
    a scheduler that aliased the tables would know anyway)."""
    bs, B = case.cfg.block_size, case.cfg.batch
    cached = case.context_lens.astype(np.int64) - case.q_lens
    shared = np.zeros(B, dtype=np.int32)
    for b in range(B):
        b0 = b - b % bundle
        if b == b0:
            continue
        most = int(min(cached[b], cached[b0])) // bs
        same = case.block_tables[b, :most] == case.block_tables[b0, :most]
        shared[b] = most if same.all() else int(np.argmin(same))
    return shared


def make_case(cfg: Config, seed: Optional[int] = None, perm_seed: Optional[int] = None,
              context_lens: Optional[np.ndarray] = None, slopes: Optional[np.ndarray] = None,
              identity_blocks: bool = False) -> Case:
    """Draw one batch for ``cfg``.

    ``perm_seed`` re-draws only the physical block assignment; ``context_lens`` overrides
    the drawn lengths; ``identity_blocks`` assigns physical blocks in logical order.
    """
    seed = cfg.seed if seed is None else seed
    rng = np.random.default_rng(seed)
    B, Hq, Hkv, D, bs, NB = (cfg.batch, cfg.num_heads, cfg.num_kv_heads, cfg.head_dim,
                             cfg.block_size, cfg.num_blocks)

    # 1. context lengths
    drawn = rng.integers(cfg.ctx_lo, cfg.ctx_hi + 1, size=B).astype(np.int32)
    ctx = drawn if context_lens is None else np.asarray(context_lens, dtype=np.int32)
    assert ctx.shape == (B,)
    q_lens = np.minimum(np.full(B, cfg.q_len, dtype=np.int32), ctx)
    cu = np.zeros(B + 1, dtype=np.int32)
    cu[1:] = np.cumsum(q_lens)
    T = int(cu[-1])

    # 2. physical block permutation, dealt to sequences in order
    perm = rng.permutation(NB).astype(np.int32)
    if perm_seed is not None:
        perm = np.random.default_rng(perm_seed).permutation(NB).astype(np.int32)
    if identity_blocks:
        perm = np.arange(NB, dtype=np.int32)
    nblk = (ctx.astype(np.int64) + bs - 1) // bs
    total_blocks = int(nblk.sum())
    if total_blocks > NB:
        raise ValueError(f"{cfg.name}: needs {total_blocks} blocks, pool has {NB}")
    MB = max(int(nblk.max()) if B else 0, 1)
    block_tables = np.full((B, MB), -1, dtype=np.int32)
    owned = perm[:total_blocks]
    starts = np.concatenate([[0], np.cumsum(nblk)]).astype(np.int64)
    for b in range(B):
        block_tables[b, : nblk[b]] = owned[starts[b]: starts[b + 1]]

    # 3. q
    q = to_bits(rng.standard_normal((T, Hq, D), dtype=np.float32), cfg.dtype)

    # 4./5. K then V, per logical block, scattered to the physical pool
    nan = NAN_BITS[cfg.dtype]
    k_cache = np.full((NB, Hkv, bs, D), nan, dtype=np.uint16)
    v_cache = np.full((NB, Hkv, bs, D), nan, dtype=np.uint16)
    # values are drawn token-major ([token, head, dim]) so that the logical content of a
    # sequence does not depend on block_size, then re-tiled to [block, head, row, dim]
    for cache in (k_cache, v_cache):
        vals = to_bits(rng.standard_normal((total_blocks * bs, Hkv, D), dtype=np.float32), cfg.dtype)
        cache[owned] = vals.reshape(total_blocks, bs, Hkv, D).transpose(0, 2, 1, 3)
        del vals

    # tail rows of each partial last block -> NaN; new tokens' rows -> moved out to k_new/v_new
    k_new = np.empty((T, Hkv, D), dtype=np.uint16)
    v_new = np.empty((T, Hkv, D), dtype=np.uint16)
    slot_mapping = np.empty(T, dtype=np.int64)
    for b in range(B):
        L = int(ctx[b])
        if L == 0:
            continue
        last = int(block_tables[b, (L - 1) // bs])
        tail = L % bs
        if tail:
            k_cache[last, :, tail:, :] = nan
            v_cache[last, :, tail:, :] = nan
        for i in range(int(q_lens[b])):
            pos = L - int(q_lens[b]) + i
            pb, r = int(block_tables[b, pos // bs]), pos % bs
            t = int(cu[b]) + i
            k_new[t] = k_cache[pb, :, r, :]
            v_new[t] = v_cache[pb, :, r, :]
            k_cache[pb, :, r, :] = nan
            v_cache[pb, :, r, :] = nan
            slot_mapping[t] = pb * bs + r

    sl = alibi_slopes(Hq) if slopes is None else np.asarray(slopes, dtype=np.float32)
    scale = np.float32(1.0 / np.sqrt(np.float64(D)))
    return Case(cfg=cfg, dtype=cfg.dtype, context_lens=ctx, q_lens=q_lens, cu_q_lens=cu,
                block_tables=block_tables, q=q, k_new=k_new, v_new=v_new,
                slot_mapping=slot_mapping, k_cache=k_cache, v_cache=v_cache, slopes=sl,
                scale=scale, partition_size=cfg.partition_size)


def small_config(name: str = "tiny", kind: str = "decode", dtype: str = F16, batch: int = 2,
                 num_heads: int = 4, num_kv_heads: int = 2, head_dim: int = 8, block_size: int = 4,
                 num_blocks: int = 64, ctx_lo: int = 1, ctx_hi: int = 40, q_len: int = 1,
                 partition_size: int = 0, seed: int = 0) -> Config:
    """Helper for the small cases tests sweep over."""
    return Config(name, kind, dtype, batch, num_heads, num_kv_heads, head_dim, block_size,
                  num_blocks, ctx_lo, ctx_hi, q_len, partition_size, seed)
