"""Test-side helpers written independently of both the oracle and the HIP path."""
from __future__ import annotations

import numpy as np

from paper_2402_01869_amd import workloads as W


def bits(x) -> np.ndarray:
    return W.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


def paged_pool_from_dense(K, V, table, block_size, num_blocks, fill_bits=0x7FFF):
    """Scatter dense K, V ([ctx][H][D] uint16 bit patterns) into a fresh pool through `table`."""
    ctx, H, D = K.shape
    pool = np.full(W.pool_shape(num_blocks, H, block_size, D), fill_bits, dtype=np.uint16)
    for t in range(ctx):
        b, s = table[t // block_size], t % block_size
        pool[b, 0, :, s, :] = K[t]
        pool[b, 1, :, s, :] = V[t]
    return pool


def dense_causal_attention(q, K, V, scale, first_pos):
    """numpy fp64 reference on contiguous tensors: q [n][H][D], K/V [ctx][H][D] (float64).

    Row i sees keys 0..first_pos+i.  Written with einsum + a mask, no paging.
    """
    n, H, D = q.shape
    ctx = K.shape[0]
    s = np.einsum("ihd,thd->hit", q, K) * scale
    pos = first_pos + np.arange(n)[:, None]
    mask = np.arange(ctx)[None, :] > pos
    s = np.where(mask[None], -np.inf, s)
    s = s - s.max(axis=-1, keepdims=True)
    w = np.exp(s)
    w /= w.sum(axis=-1, keepdims=True)
    return np.einsum("hit,thd->ihd", w, V)
