"""Seeded synthetic inputs for the intercept hot path (descriptors, KV pools, swap lists).

This module is shared by the CPU oracle's tests and by the HIP path's tests and
benchmark.  It holds no attention or swap arithmetic: it only draws shapes,
lengths, block ids and N(0,1) values, and rounds those values to bf16 once so
that both sides read the same bit patterns.

The shapes stand in for the paper's workloads: model shapes follow the three
evaluated models (Section 5, GPT-J-6B / Vicuna-13B) and the context-length
ranges bracket the per-augmentation means of Table 1 (about 750 to 2200 tokens).
A mixed batch is what the scheduler of Section 4.3 hands to one iteration:
running requests contribute one decode token each, resumed discarded requests
contribute one recomputation chunk each (Section 4.2).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

import numpy as np

BASE_SEED = 20240201
BLOCK_SIZE = 16


@dataclass(frozen=True)
class AttnConfig:
    """Shape of one mixed-batch workload."""
    name: str
    index: int
    num_heads: int
    head_dim: int
    block_size: int
    pool_blocks: int
    n_decode: int
    decode_ctx: Tuple[int, int]          # inclusive integer range
    n_span: int = 0
    span_len: int = 0
    span_prefix: Tuple[int, int] = (0, 0)  # inclusive range of the cached prefix before the span
    span_ctx: Optional[Tuple[int, int]] = None  # if set: draw total context instead of prefix
    num_kv_heads: int = 0                # 0: as many as query heads (multi-head attention)

    @property
    def kv_heads(self) -> int:
        return self.num_kv_heads or self.num_heads

    @property
    def token_bytes(self) -> int:
        """KV bytes per token for one layer (the paper's M, Section 3.2): K and V, all K/V heads, bf16."""
        return 2 * self.kv_heads * self.head_dim * 2

    @property
    def block_bytes(self) -> int:
        return self.block_size * self.token_bytes

    @property
    def seed(self) -> int:
        return BASE_SEED + self.index


@dataclass(frozen=True)
class SwapConfig:
    name: str
    index: int
    num_heads: int
    head_dim: int
    block_size: int
    pool_blocks: int
    n_move: int

    @property
    def token_bytes(self) -> int:
        return 2 * self.num_heads * self.head_dim * 2

    @property
    def block_bytes(self) -> int:
        return self.block_size * self.token_bytes

    @property
    def seed(self) -> int:
        return BASE_SEED + self.index


TINY = AttnConfig("tiny", 0, num_heads=4, head_dim=64, block_size=16, pool_blocks=64,
                  n_decode=2, decode_ctx=(16, 128), n_span=2, span_len=32, span_ctx=(16, 128))
GPTJ_DECODE = AttnConfig("gptj_decode", 1, num_heads=16, head_dim=256, block_size=16,
                         pool_blocks=16384, n_decode=64, decode_ctx=(512, 2048))
MIXED_13B = AttnConfig("mixed_13b", 2, num_heads=40, head_dim=128, block_size=16,
                       pool_blocks=65536, n_decode=128, decode_ctx=(256, 4096),
                       n_span=8, span_len=512, span_prefix=(1024, 4096))
# Grouped-query shape of the paper's largest model (Section 5: Llama3-70B, 64 query heads over 8 K/V heads)
GQA_70B = AttnConfig("gqa_70b", 5, num_heads=64, head_dim=128, block_size=16, pool_blocks=65536,
                     n_decode=128, decode_ctx=(256, 4096), n_span=8, span_len=512, span_prefix=(1024, 4096),
                     num_kv_heads=8)
LONG_CTX = AttnConfig("long_ctx", 4, num_heads=32, head_dim=128, block_size=16,
                      pool_blocks=524288, n_decode=256, decode_ctx=(1024, 8192),
                      n_span=16, span_len=2048, span_prefix=(16384, 16384))
# GPT-J-6B-shaped mixed batch (Section 5's single-GPU model; Section 3.2: recomputation takes 37-40 % of its forwarding
# time under the discard baseline): config 1's decode batch plus 8 recomputation chunks, head_dim 256
GPTJ_MIXED = AttnConfig("gptj_mixed", 6, num_heads=16, head_dim=256, block_size=16, pool_blocks=16384,
                        n_decode=64, decode_ctx=(512, 2048), n_span=8, span_len=512, span_prefix=(512, 2048))
TINY_SWAP = SwapConfig("tiny_swap", 0, num_heads=4, head_dim=64, block_size=16,
                       pool_blocks=64, n_move=8)
KV_SWAP = SwapConfig("kv_swap", 3, num_heads=40, head_dim=128, block_size=16,
                     pool_blocks=20000, n_move=2000)

ATTN_CONFIGS: Dict[str, AttnConfig] = {c.name: c for c in (TINY, GPTJ_DECODE, MIXED_13B, LONG_CTX, GQA_70B, GPTJ_MIXED)}
SWAP_CONFIGS: Dict[str, SwapConfig] = {c.name: c for c in (TINY_SWAP, KV_SWAP)}


@dataclass
class Batch:
    """Host-side batch descriptor: what one scheduler iteration hands to the attention call.

    ctx_len[s]   KV tokens visible to sequence s, including the query span's own tokens
    q_len[s]     1 for a decode sequence, >1 for a recomputation chunk
    q_start[s]   first row of sequence s in the packed Q / out arrays
    block_tables [num_seqs][max_blocks_per_seq] int32, entries past ceil(ctx_len/block_size) unused (-1)
    """
    num_heads: int
    head_dim: int
    block_size: int
    pool_blocks: int
    ctx_len: np.ndarray
    q_len: np.ndarray
    q_start: np.ndarray
    block_tables: np.ndarray
    scale: float
    extra: dict = field(default_factory=dict)
    num_kv_heads: int = 0                # 0: as many as query heads

    @property
    def kv_heads(self) -> int:
        return self.num_kv_heads or self.num_heads

    @property
    def num_seqs(self) -> int:
        return int(self.ctx_len.shape[0])

    @property
    def max_blocks_per_seq(self) -> int:
        return int(self.block_tables.shape[1])

    @property
    def total_q_rows(self) -> int:
        return int(self.q_len.sum())

    @property
    def token_bytes(self) -> int:
        return 2 * self.kv_heads * self.head_dim * 2

    def kv_bytes(self) -> int:
        """Algorithmic KV bytes of the call: every sequence's context read once."""
        return int(self.ctx_len.astype(np.int64).sum()) * self.token_bytes

    def blocks_of(self, s: int) -> np.ndarray:
        nb = -(-int(self.ctx_len[s]) // self.block_size)
        return self.block_tables[s, :nb]

    def span_flops(self) -> int:
        """Dense multiply-add flops of the multi-row spans (QK^T and PV, causal triangle counted exactly)."""
        total = 0
        for s in range(self.num_seqs):
            n, c = int(self.q_len[s]), int(self.ctx_len[s])
            if n > 1:
                keys = n * (c - n) + n * (n + 1) // 2
                total += 4 * keys * self.num_heads * self.head_dim
        return total


def _streams(seed: int, n: int) -> List[np.random.Generator]:
    """Independent sub-streams (lengths / block ids / values ...) so changing one does not shift the others."""
    return [np.random.default_rng(s) for s in np.random.SeedSequence(seed).spawn(n)]


def make_batch(cfg: AttnConfig, seed: Optional[int] = None) -> Batch:
    """Draw a mixed batch for `cfg`: decode sequences first, then recomputation spans.

    Context lengths are integers uniform on the inclusive range and are not rounded to the
    block size, so the last block of a sequence is usually partial.  Block tables are disjoint
    slices of one random permutation of the pool's block ids (non-contiguous, no sharing).
    A span longer than its drawn context (tiny config only) becomes a prefill from position 0.
    """
    seed = cfg.seed if seed is None else seed
    r_len, r_ids = _streams(seed, 4)[:2]
    ctx: List[int] = []
    qlen: List[int] = []
    lo, hi = cfg.decode_ctx
    for _ in range(cfg.n_decode):
        ctx.append(int(r_len.integers(lo, hi + 1)))
        qlen.append(1)
    for _ in range(cfg.n_span):
        if cfg.span_ctx is not None:
            c = int(r_len.integers(cfg.span_ctx[0], cfg.span_ctx[1] + 1))
            n = min(cfg.span_len, c)
        else:
            p = int(r_len.integers(cfg.span_prefix[0], cfg.span_prefix[1] + 1))
            c, n = p + cfg.span_len, cfg.span_len
        ctx.append(c)
        qlen.append(n)
    return assemble_batch(cfg.num_heads, cfg.head_dim, cfg.block_size, cfg.pool_blocks,
                          ctx, qlen, r_ids, num_kv_heads=cfg.num_kv_heads)


def assemble_batch(num_heads: int, head_dim: int, block_size: int, pool_blocks: int,
                   ctx: List[int], qlen: List[int], rng: np.random.Generator,
                   scale: Optional[float] = None, num_kv_heads: int = 0) -> Batch:
    """Build a Batch from explicit lengths; block ids come from one permutation of the pool."""
    ctx_a = np.asarray(ctx, dtype=np.int32)
    q_a = np.asarray(qlen, dtype=np.int32)
    nblk = -(-ctx_a.astype(np.int64) // block_size)
    need = int(nblk.sum())
    if need > pool_blocks:
        raise ValueError(f"batch needs {need} blocks, pool has {pool_blocks}")
    perm = rng.permutation(pool_blocks)[:need].astype(np.int32)
    width = int(nblk.max()) if len(nblk) else 0
    tables = np.full((len(ctx), width), -1, dtype=np.int32)
    off = 0
    for s, nb in enumerate(nblk):
        tables[s, :nb] = perm[off:off + nb]
        off += int(nb)
    q_start = np.zeros(len(ctx), dtype=np.int32)
    if len(ctx) > 1:
        q_start[1:] = np.cumsum(q_a)[:-1]
    sc = float(np.float32(1.0 / np.sqrt(np.float32(head_dim)))) if scale is None else float(scale)
    return Batch(num_heads, head_dim, block_size, pool_blocks, ctx_a, q_a, q_start, tables, sc,
                 num_kv_heads=num_kv_heads)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round-to-nearest-even) and return the 16-bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    rounded = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return rounded.astype(np.uint16)


def bf16_bits_to_f64(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns exactly to fp64."""
    u = (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16)
    return u.view(np.float32).astype(np.float64)


def randn_bf16(shape, rng: np.random.Generator) -> np.ndarray:
    """N(0,1) drawn in fp32 and rounded once to bf16; returned as uint16 bit patterns."""
    return f32_to_bf16_bits(rng.standard_normal(shape, dtype=np.float32))


def pool_shape(num_blocks: int, num_heads: int, block_size: int, head_dim: int) -> Tuple[int, ...]:
    """Pool layout: [block][K=0 / V=1][head][token slot][dim]."""
    return (num_blocks, 2, num_heads, block_size, head_dim)


def make_host_inputs(batch: Batch, seed: int, poison_unused: bool = True):
    """Host pool + Q for a batch small enough to generate on the CPU.

    Returns (pool_bits uint16 [blocks][2][H][B][D], q_bits uint16 [rows][H][D]).
    With poison_unused, every slot no sequence may read (unreferenced blocks and the tail of
    each last block) holds the bf16 NaN pattern 0x7FFF, so any stray read shows up in the output.
    """
    r_pool, r_q = _streams(seed, 4)[2:4]
    shp = pool_shape(batch.pool_blocks, batch.kv_heads, batch.block_size, batch.head_dim)
    pool = randn_bf16(shp, r_pool)
    if poison_unused:
        poison_pool(pool, batch)
    q = randn_bf16((batch.total_q_rows, batch.num_heads, batch.head_dim), r_q)
    return pool, q


def poison_pool(pool: np.ndarray, batch: Batch, pattern: int = 0x7FFF) -> None:
    """Overwrite every don't-care slot of `pool` (in place) with `pattern`."""
    used = np.zeros(pool.shape[0], dtype=bool)
    for s in range(batch.num_seqs):
        ids = batch.blocks_of(s)
        used[ids] = True
        tail = int(batch.ctx_len[s]) % batch.block_size
        if tail:
            pool[ids[-1], :, :, tail:, :] = pattern
    pool[~used] = pattern


def make_swap_lists(cfg: SwapConfig, seed: Optional[int] = None):
    """Source ids (distinct, random) and destination ids (distinct, random, disjoint from the sources)."""
    seed = cfg.seed if seed is None else seed
    r = _streams(seed, 4)[1]
    perm = r.permutation(cfg.pool_blocks).astype(np.int32)
    return perm[:cfg.n_move].copy(), perm[cfg.n_move:2 * cfg.n_move].copy()


def random_pool_bytes(cfg: SwapConfig, seed: Optional[int] = None) -> np.ndarray:
    """Random bytes for a whole swap pool, shape [blocks][block_bytes] uint8 (host; small configs only)."""
    seed = cfg.seed if seed is None else seed
    r = _streams(seed, 4)[2]
    return r.integers(0, 256, size=(cfg.pool_blocks, cfg.block_bytes), dtype=np.uint8)


# ---------------------------------------------------------------------------
# Device-side fills for pools too large to generate on the host (torch is used
# only as an allocator / random source here; nothing below is part of the method).
# ---------------------------------------------------------------------------

def fill_pool_device_normal(pool_t, seed: int, chunk_blocks: int = 2048) -> None:
    """Fill a bf16 device tensor [blocks][2][H][B][D] with N(0,1), chunk by chunk (fp32 draw, one rounding)."""
    import torch
    g = torch.Generator(device=pool_t.device)
    g.manual_seed(seed)
    nb = pool_t.shape[0]
    for b0 in range(0, nb, chunk_blocks):
        b1 = min(nb, b0 + chunk_blocks)
        shp = (b1 - b0,) + tuple(pool_t.shape[1:])
        tmp = torch.randn(shp, generator=g, device=pool_t.device, dtype=torch.float32)
        pool_t[b0:b1].copy_(tmp)
        del tmp


def fill_bytes_device(buf_t, seed: int, chunk: int = 1 << 28) -> None:
    """Fill a uint8 device tensor with random bytes."""
    import torch
    g = torch.Generator(device=buf_t.device)
    g.manual_seed(seed)
    flat = buf_t.view(-1)
    n = flat.numel()
    for o in range(0, n, chunk):
        e = min(n, o + chunk)
        flat[o:e] = torch.randint(0, 256, (e - o,), generator=g, device=buf_t.device, dtype=torch.uint8)


def compact_referenced(batch: Batch, seqs, fetch_blocks):
    """Gather only the blocks the listed sequences reference into a small host pool.

    fetch_blocks(ids int64 array) -> uint16 array [len(ids)][2][H][B][D] (for example a device read-back).
    Returns (small_pool, sub_batch) where sub_batch's tables index small_pool.  Relabelling physical
    blocks is legitimate because attention depends on the table-to-block mapping only.
    """
    seqs = list(seqs)
    ids = np.concatenate([batch.blocks_of(s) for s in seqs]).astype(np.int64)
    small = fetch_blocks(ids)
    width = max(len(batch.blocks_of(s)) for s in seqs)
    tables = np.full((len(seqs), width), -1, dtype=np.int32)
    off = 0
    for i, s in enumerate(seqs):
        nb = len(batch.blocks_of(s))
        tables[i, :nb] = np.arange(off, off + nb, dtype=np.int32)
        off += nb
    sub = Batch(batch.num_heads, batch.head_dim, batch.block_size, len(ids),
                batch.ctx_len[seqs].copy(), batch.q_len[seqs].copy(), batch.q_start[seqs].copy(),
                tables, batch.scale, num_kv_heads=batch.num_kv_heads)
    return small, sub
