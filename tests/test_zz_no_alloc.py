"""kv_pack_blocks_static (the entry point for callers that cannot allocate) against kv_pack_blocks: two calls in a
row on one stream, the second with a shorter list, byte for byte; and its fixed capacity."""
import numpy as np
import pytest
import torch

from paper_2402_01869_amd import binding as B
from gpu_common import DEV

pytestmark = pytest.mark.gpu


def test_static_pack_matches_kv_pack_blocks_on_two_calls_in_a_row():
    H, D, blocks = 4, 64, 4096                                       # 16 KiB blocks, 64 MiB pool
    rng = np.random.default_rng(77)
    cfg = B.make_cfg(blocks, H, D)
    bb = 16 * 2 * H * D * 2
    pool_t = torch.from_numpy(rng.integers(0, 256, size=(blocks, bb), dtype=np.uint8)).to(DEV)
    pool = B.KvPool(cfg, pool_t.data_ptr(), pool_t.numel())
    assert pool.block_bytes == bb
    n_max = 2500
    st_a = torch.zeros((n_max, bb), dtype=torch.uint8, device=DEV)   # kv_pack_blocks
    st_b = torch.zeros((n_max, bb), dtype=torch.uint8, device=DEV)   # kv_pack_blocks_static
    stream = torch.cuda.Stream()
    for n in (2500, 700, 1, 961):                                    # three argument chunks, then fewer; one id; one past a chunk
        ids = rng.integers(0, blocks, size=n).astype(np.int32)       # duplicates allowed in a pack list
        st_a.fill_(0x5A)
        st_b.fill_(0x5A)
        torch.cuda.synchronize()
        pool.kv_pack_blocks(ids, st_a.data_ptr(), st_a.numel(), stream.cuda_stream)
        pool.kv_pack_blocks_static(ids, st_b.data_ptr(), st_b.numel(), stream.cuda_stream)
        stream.synchronize()
        a, b = st_a.cpu().numpy(), st_b.cpu().numpy()
        assert np.array_equal(a, b), n
        assert (b[n:] == 0x5A).all(), "wrote past the list"
        assert np.array_equal(b[:n], pool_t.cpu().numpy()[ids])
    # back to back without a host wait between the calls: the second list replaces the first in the same array
    ids1 = rng.integers(0, blocks, size=1500).astype(np.int32)
    ids2 = rng.integers(0, blocks, size=400).astype(np.int32)
    st_c = torch.zeros((n_max, bb), dtype=torch.uint8, device=DEV)
    pool.kv_pack_blocks_static(ids1, st_b.data_ptr(), st_b.numel(), stream.cuda_stream)
    pool.kv_pack_blocks_static(ids2, st_c.data_ptr(), st_c.numel(), stream.cuda_stream)
    stream.synchronize()
    host = pool_t.cpu().numpy()
    assert np.array_equal(st_b.cpu().numpy()[:1500], host[ids1])
    assert np.array_equal(st_c.cpu().numpy()[:400], host[ids2])
    # validation, before anything is launched
    assert pool.kv_pack_blocks_static([], st_b.data_ptr(), st_b.numel(), check=False) == B.IC_OK
    assert pool.kv_pack_blocks_static([blocks], st_b.data_ptr(), st_b.numel(), check=False) == B.IC_ERANGE
    assert pool.kv_pack_blocks_static([1, 2], st_b.data_ptr(), bb, check=False) == B.IC_ESIZE
    assert pool.kv_pack_blocks_static([1, 2], st_b.data_ptr() + 4, st_b.numel(), check=False) == B.IC_EALIGN
    too_many = np.zeros(B.IC_STATIC_PACK_MAX_BLOCKS + 1, dtype=np.int32)
    assert pool.kv_pack_blocks_static(too_many, st_b.data_ptr(), 1 << 62, check=False) == B.IC_ELIMIT
    pool.close()
