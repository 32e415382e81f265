"""GPU-side test plumbing: torch is used for device memory only; all compute goes through the C ABI."""
from __future__ import annotations

import numpy as np
import torch

from paper_2402_01869_amd import binding as B
from paper_2402_01869_amd import workloads as W

DEV = "cuda:0"


def to_dev_bits(bits: np.ndarray) -> torch.Tensor:
    """uint16 bit patterns -> device int16 tensor with the same bits."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(DEV)


def from_dev_bits(t: torch.Tensor) -> np.ndarray:
    return t.cpu().numpy().view(np.uint16)


class AttnRunner:
    """Owns device q / out / workspace for one batch and calls paged_attn_mixed."""

    def __init__(self, pool: B.KvPool, batch, q_bits: np.ndarray, flags: int = 0):
        self.pool, self.batch = pool, batch
        self.desc = B.HostDesc.from_batch(batch, flags=flags)
        self.q = to_dev_bits(q_bits)
        # NaN-filled output: rows the call must write are checked to be finite afterwards
        self.out = torch.full(tuple(q_bits.shape), 0x7FFF, dtype=torch.int16, device=DEV)
        self.ws = None

    def run(self, stream: int = 0) -> np.ndarray:
        need = self.pool.workspace_bytes(self.desc)
        assert need > 0
        if self.ws is None or self.ws.numel() < need:
            self.ws = torch.empty(need, dtype=torch.uint8, device=DEV)
        self.pool.paged_attn_mixed(self.desc, self.q.data_ptr(), self.out.data_ptr(), self.ws.data_ptr(),
                                   self.ws.numel(), stream)
        torch.cuda.synchronize()
        return from_dev_bits(self.out)


def make_pool(pool_bits: np.ndarray, num_heads: int = 0):
    """pool_bits [blocks][2][Hkv][B][D]; num_heads = query heads (0: as many as K/V heads)."""
    nb, two, Hkv, Bs, D = pool_bits.shape
    t = to_dev_bits(pool_bits)
    return B.KvPool.from_tensor(t, num_heads or Hkv, D, Bs, num_kv_heads=Hkv), t


def max_abs_err(out_bits: np.ndarray, want_f64: np.ndarray) -> float:
    got = W.bf16_bits_to_f64(out_bits)
    return float(np.max(np.abs(got - want_f64)))
