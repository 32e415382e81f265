"""HIP pack / unpack against the memcpy oracle, bit for bit (swap of scattered blocks, Section 3.2)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2402_01869_amd import binding as B
from paper_2402_01869_amd import workloads as W
from gpu_common import DEV, to_dev_bits

pytestmark = pytest.mark.gpu


def _roundtrip(cfg, pool_host: np.ndarray, src, dst):
    """pool_host uint8 [blocks][block_bytes].  Returns nothing; asserts bit-exactness everywhere."""
    bb = cfg.block_bytes
    pool_t = torch.from_numpy(pool_host).to(DEV)
    pool = B.KvPool(B.make_cfg(cfg.pool_blocks, cfg.num_heads, cfg.head_dim), pool_t.data_ptr(), pool_t.numel())
    assert pool.block_bytes == bb
    n = len(src)
    staging = torch.full((n * bb,), 0xA5, dtype=torch.uint8, device=DEV)
    pool.kv_pack_blocks(src, staging.data_ptr(), staging.numel())
    torch.cuda.synchronize()
    want_staging = oracle.pack_blocks(pool_host, src)
    assert np.array_equal(staging.cpu().numpy().reshape(n, bb), want_staging)
    assert np.array_equal(pool_t.cpu().numpy(), pool_host), "pack must not write the pool"
    pool.kv_unpack_blocks(dst, staging.data_ptr(), staging.numel())
    torch.cuda.synchronize()
    want_pool = pool_host.copy()
    oracle.unpack_blocks(want_pool, dst, want_staging)
    assert np.array_equal(pool_t.cpu().numpy(), want_pool)
    pool.close()


def test_tiny_swap_bit_exact():
    cfg = W.TINY_SWAP
    src, dst = W.make_swap_lists(cfg)
    _roundtrip(cfg, W.random_pool_bytes(cfg), src, dst)


@pytest.mark.parametrize("H,D,n", [(1, 64, 1), (3, 64, 5), (5, 128, 7), (2, 256, 3)])
def test_odd_shapes_and_duplicate_sources(H, D, n):
    cfg = W.SwapConfig("odd", 7, H, D, 16, 11, n)
    rng = np.random.default_rng(H * 1000 + D + n)
    pool_host = rng.integers(0, 256, size=(cfg.pool_blocks, cfg.block_bytes), dtype=np.uint8)
    src = rng.integers(0, cfg.pool_blocks, size=n).astype(np.int32)   # may repeat
    dst = rng.permutation(cfg.pool_blocks)[:n].astype(np.int32)
    _roundtrip(cfg, pool_host, src, dst)


def test_full_kv_swap_config_bit_exact():
    """13B-shaped swap: 2000 of 20000 blocks of 320 KiB, whole pool compared after the round trip."""
    cfg = W.KV_SWAP
    src, dst = W.make_swap_lists(cfg)
    pool_t = torch.empty((cfg.pool_blocks, cfg.block_bytes), dtype=torch.uint8, device=DEV)
    W.fill_bytes_device(pool_t, cfg.seed)
    pool_host = pool_t.cpu().numpy()
    pool = B.KvPool(B.make_cfg(cfg.pool_blocks, cfg.num_heads, cfg.head_dim), pool_t.data_ptr(), pool_t.numel())
    staging = torch.zeros((cfg.n_move, cfg.block_bytes), dtype=torch.uint8, device=DEV)
    pool.kv_pack_blocks(src, staging.data_ptr(), staging.numel())
    pool.kv_unpack_blocks(dst, staging.data_ptr(), staging.numel())
    torch.cuda.synchronize()
    want_staging = oracle.pack_blocks(pool_host, src)
    assert np.array_equal(staging.cpu().numpy(), want_staging)
    oracle.unpack_blocks(pool_host, dst, want_staging)
    got = pool_t.cpu().numpy()
    assert np.array_equal(got, pool_host)
    # swapped-in context equals the swapped-out one
    assert np.array_equal(got[dst], got[src])
    pool.close()


def test_errors_leave_memory_untouched():
    cfg = W.TINY_SWAP
    pool_host = W.random_pool_bytes(cfg)
    pool_t = torch.from_numpy(pool_host).to(DEV)
    pool = B.KvPool(B.make_cfg(cfg.pool_blocks, cfg.num_heads, cfg.head_dim), pool_t.data_ptr(), pool_t.numel())
    bb = cfg.block_bytes
    staging = torch.full((4 * bb,), 7, dtype=torch.uint8, device=DEV)
    sp, sb = staging.data_ptr(), staging.numel()
    assert pool.kv_pack_blocks([0, 64], sp, sb, check=False) == B.IC_ERANGE
    assert pool.kv_pack_blocks([-1], sp, sb, check=False) == B.IC_ERANGE
    assert pool.kv_unpack_blocks([3, 3], sp, sb, check=False) == B.IC_EDUP
    assert pool.kv_pack_blocks([1, 2, 3, 4, 5], sp, sb, check=False) == B.IC_ESIZE
    assert pool.kv_pack_blocks([1], sp + 8, sb - 8, check=False) == B.IC_EALIGN
    assert pool.kv_pack_blocks([1], pool_t.data_ptr() + bb, bb, check=False) == B.IC_EINVAL  # overlaps pool
    assert pool.kv_pack_blocks([], sp, sb, check=False) == B.IC_OK
    torch.cuda.synchronize()
    assert (staging.cpu().numpy() == 7).all()
    assert np.array_equal(pool_t.cpu().numpy(), pool_host)
    pool.close()


@pytest.mark.gpu
def test_mfma_ceiling_reports_a_rate_and_a_clock():
    """The measurement aid runs and returns plausible figures: a rate below the vendor peak (plus timer slack) and a
    shader clock between 0.3 and 2.6 GHz."""
    rng = np.random.default_rng(3)
    n16 = B.IC_CEILING_OPERAND_BYTES // 2
    sink = torch.empty(B.IC_CEILING_SINK_BYTES, dtype=torch.uint8, device=DEV)
    for name, bits in (("zeros", np.zeros(n16, dtype=np.uint16)), ("random", W.randn_bf16((n16,), rng))):
        ops = to_dev_bits(bits)
        for _ in range(2):   # the first call after an idle gap runs while the clocks ramp
            rc, tf, ghz = B.mfma_ceiling(ops.data_ptr(), ops.numel() * 2, sink.data_ptr(), sink.numel(), 20000)
            assert rc == B.IC_OK
        print(name, tf, ghz, flush=True)
        assert 50.0 < tf < 2600.0 and 0.3 < ghz < 2.6, (name, tf, ghz)


@pytest.mark.gpu
def test_hbm_ceiling_copy_is_exact_and_reports_a_rate():
    """The copy mode of the measurement aid really copies (bit for bit) and both modes return a rate below the vendor
    peak (plus timer slack)."""
    n = 64 << 20
    src = torch.randint(0, 256, (n,), dtype=torch.uint8, device=DEV)
    dst = torch.zeros(n, dtype=torch.uint8, device=DEV)
    rc, g = B.hbm_ceiling(src.data_ptr(), dst.data_ptr(), n, 1, 3)
    assert rc == B.IC_OK and 100.0 < g < 8800.0, g
    assert torch.equal(src, dst)
    rc, g = B.hbm_ceiling(src.data_ptr(), dst.data_ptr(), n, 0, 3)
    assert rc == B.IC_OK and 100.0 < g < 8800.0, g


@pytest.mark.gpu
@pytest.mark.parametrize("D", [64, 128, 256])
def test_paged_read_ceiling_runs_on_every_head_dim(D):
    """The compute-free read of listed blocks (duplicates allowed) returns a plausible rate and leaves the pool alone."""
    H, nb = 3, 300
    pool_t = torch.randint(-30000, 30000, (nb, 2, H, 16, D), dtype=torch.int16, device=DEV)
    before = pool_t.clone()
    pool = B.KvPool.from_tensor(pool_t, H, D)
    sink = torch.zeros(16, dtype=torch.uint8, device=DEV)
    ids = np.random.default_rng(D).integers(0, nb, size=1000).astype(np.int32)
    g = pool.paged_read_ceiling(ids, sink.data_ptr(), 3)
    assert 1.0 < g < 8800.0, g
    assert torch.equal(pool_t, before)
    pool.close()


def test_repeated_and_changing_id_lists():
    """The library keeps the device copy of the last pack list and of the last unpack list and skips the upload
    when a call brings the same list again (one swap = the same blocks for every layer).  Same list with changed
    pool contents, another list of the same length, a shorter list, the first list again: always the oracle's bytes."""
    H, D, blocks, n = 2, 64, 300, 40
    bb = 16 * 2 * H * D * 2
    rng = np.random.default_rng(31)
    host = rng.integers(0, 256, size=(blocks, bb), dtype=np.uint8)
    pool_t = torch.from_numpy(host.copy()).to(DEV)
    pool = B.KvPool(B.make_cfg(blocks, H, D), pool_t.data_ptr(), pool_t.numel())
    staging = torch.zeros((n, bb), dtype=torch.uint8, device=DEV)
    a = rng.permutation(blocks)[:n].astype(np.int32)
    b = rng.permutation(blocks)[:n].astype(np.int32)
    for step, ids in enumerate([a, a, b, a[:7], a, b, b]):
        if step % 2:      # change what the listed blocks hold between calls with the same list
            host[ids[0]] = rng.integers(0, 256, size=bb, dtype=np.uint8)
            pool_t[int(ids[0])] = torch.from_numpy(host[ids[0]]).to(DEV)
        staging.fill_(0x11)
        pool.kv_pack_blocks(ids, staging.data_ptr(), staging.numel())
        torch.cuda.synchronize()
        got = staging.cpu().numpy()
        assert np.array_equal(got[:len(ids)], oracle.pack_blocks(host, ids)), step
        assert (got[len(ids):] == 0x11).all(), step
    # unpack: the same destinations twice with different staging contents, then other destinations
    for step, ids in enumerate([a, a, b, b[:5], a]):
        src = rng.integers(0, 256, size=(n, bb), dtype=np.uint8)
        staging.copy_(torch.from_numpy(src).to(DEV))
        pool.kv_unpack_blocks(ids, staging.data_ptr(), staging.numel())
        torch.cuda.synchronize()
        oracle.unpack_blocks(host, ids, src[:len(ids)])
        assert np.array_equal(pool_t.cpu().numpy(), host), step
    # a list with a duplicate destination is refused also right after a call with the same length
    dup = a.copy(); dup[3] = dup[9]
    assert pool.kv_unpack_blocks(dup, staging.data_ptr(), staging.numel(), check=False) == B.IC_EDUP
    pool.kv_unpack_blocks(a, staging.data_ptr(), staging.numel())
    torch.cuda.synchronize()
    pool.close()
