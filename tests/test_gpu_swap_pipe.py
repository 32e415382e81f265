"""Layer-pipelined swap to pinned host memory (Section 4.1) against the per-layer memcpy oracle, bit for bit."""
import numpy as np
import pytest
import torch

import oracle
from paper_2402_01869_amd import binding as B
from paper_2402_01869_amd import workloads as W
from gpu_common import DEV, AttnRunner, from_dev_bits, max_abs_err

pytestmark = pytest.mark.gpu


class Layers:
    """L same-shaped pools on the device, their host copies for the oracle, and a swapper over them."""

    def __init__(self, L, nb, H, D, max_blocks, stages, seed):
        self.cfg = B.make_cfg(nb, H, D)
        self.bb = 16 * 2 * H * D * 2
        rng = np.random.default_rng(seed)
        self.host = [rng.integers(0, 256, size=(nb, self.bb), dtype=np.uint8) for _ in range(L)]
        self.dev = [torch.from_numpy(h).to(DEV) for h in self.host]
        self.pools = [B.KvPool(self.cfg, t.data_ptr(), t.numel()) for t in self.dev]
        need = B.LayerSwapper.staging_bytes(self.pools[0], L, max_blocks, stages)
        assert need == stages * max_blocks * self.bb
        self.staging = torch.zeros(need, dtype=torch.uint8, device=DEV)
        self.sw = B.LayerSwapper(self.pools, max_blocks, self.staging.data_ptr(), need, stages)

    def close(self):
        self.sw.close()
        for p in self.pools:
            p.close()


@pytest.mark.parametrize("L,stages,n", [(1, 2, 5), (3, 2, 12), (5, 3, 7), (7, 8, 1)])
def test_out_then_in_matches_oracle(L, stages, n):
    ly = Layers(L, 64, 4, 64, 12, stages, seed=L * 10 + n)
    rng = np.random.default_rng(n)
    perm = rng.permutation(64).astype(np.int32)
    src, dst = perm[:n], perm[n:2 * n]
    stride = n * ly.bb + 4096                      # padded layer stride
    pin = B.PinnedBuffer(L * stride)
    pin.array[:] = 0xEE
    ly.sw.swap_out(src, pin.ptr, stride)
    ly.sw.sync()
    want_host = oracle.swap_out_layers(ly.host, src, stride)
    assert np.array_equal(pin.array.reshape(L, stride), want_host)          # payload AND untouched padding
    for l in range(L):
        assert np.array_equal(ly.dev[l].cpu().numpy(), ly.host[l]), "swap-out must not write the pools"
    ly.sw.swap_in(dst, pin.ptr, stride)
    ly.sw.sync()
    want = [h.copy() for h in ly.host]
    oracle.swap_in_layers(want, dst, want_host)
    for l in range(L):
        assert np.array_equal(ly.dev[l].cpu().numpy(), want[l]), l
    pin.close()
    ly.close()


def test_many_calls_in_flight_reuse_stages_and_id_slots():
    """Ten chunks of one sequence's swap queued without a host wait (a chunk per iteration, Section 4.1):
    more calls than id slots, far more layer-moves than staging buffers; then all of them back in."""
    L, n_calls = 4, 10
    ly = Layers(L, 128, 2, 128, 6, 2, seed=99)
    rng = np.random.default_rng(1)
    perm = rng.permutation(128).astype(np.int32)
    sizes = [int(x) for x in rng.integers(1, 7, size=n_calls)]
    offs = np.concatenate([[0], np.cumsum(sizes)])
    pins, strides = [], []
    for c in range(n_calls):
        strides.append(sizes[c] * ly.bb)
        pins.append(B.PinnedBuffer(L * strides[c]))
        ly.sw.swap_out(perm[offs[c]:offs[c + 1]], pins[c].ptr, strides[c])
    ly.sw.sync()
    for c in range(n_calls):
        want = oracle.swap_out_layers(ly.host, perm[offs[c]:offs[c + 1]], strides[c])
        assert np.array_equal(pins[c].array.reshape(L, strides[c]), want), c
    # back in, to the blocks after the sources in the permutation, again without waiting in between
    want_pools = [h.copy() for h in ly.host]
    base = int(offs[-1])
    for c in range(n_calls):
        dst = perm[base + offs[c]:base + offs[c + 1]]
        ly.sw.swap_in(dst, pins[c].ptr, strides[c])
        oracle.swap_in_layers(want_pools, dst, pins[c].array.reshape(L, strides[c]).copy())
    ly.sw.sync()
    for l in range(L):
        assert np.array_equal(ly.dev[l].cpu().numpy(), want_pools[l]), l
    for p in pins:
        p.close()
    ly.close()


def test_swap_in_then_attention_ordered_by_wait_layer():
    """An intercepted sequence is swapped out, its blocks are overwritten, it is swapped back into other
    blocks and attention over the new block table, ordered per layer with wait_layer on the caller's
    stream, gives what the oracle gives on the original cache."""
    L, H, D, nb = 3, 4, 64, 96
    rng = np.random.default_rng(5)
    batch = W.assemble_batch(H, D, 16, nb, [200, 77, 130], [1, 1, 40], rng)
    qs = [W.randn_bf16((batch.total_q_rows, H, D), np.random.default_rng(50 + l)) for l in range(L)]
    pools_bits = [W.randn_bf16(W.pool_shape(nb, H, 16, D), np.random.default_rng(60 + l)) for l in range(L)]
    want = [oracle.attn_batch(batch, pools_bits[l], qs[l]) for l in range(L)]
    dev = [torch.from_numpy(pb.view(np.int16)).to(DEV) for pb in pools_bits]
    pools = [B.KvPool.from_tensor(t, H, D) for t in dev]
    used = np.unique(np.concatenate([batch.blocks_of(s) for s in range(batch.num_seqs)]))
    free = np.setdiff1d(np.arange(nb), used).astype(np.int32)
    moved = batch.blocks_of(0).astype(np.int32)            # sequence 0 is intercepted
    new_home = free[:len(moved)]
    n = len(moved)
    need = B.LayerSwapper.staging_bytes(pools[0], L, n, 2)
    staging = torch.zeros(need, dtype=torch.uint8, device=DEV)
    sw = B.LayerSwapper(pools, n, staging.data_ptr(), need, 2)
    bb = pools[0].block_bytes
    pin = B.PinnedBuffer(L * n * bb)
    fg = torch.cuda.Stream()
    with torch.cuda.stream(fg):
        sw.swap_out(moved, pin.ptr, n * bb, fg.cuda_stream)
        for l in range(L):
            sw.wait_layer(B.IC_SWAP_OUT, l, fg.cuda_stream)      # the layer's blocks may be reused from here on
            dev[l][torch.from_numpy(moved).to(DEV)] = 0x7FFF      # ... and are: NaN patterns
        sw.swap_in(new_home, pin.ptr, n * bb, fg.cuda_stream)
        tables = batch.block_tables.copy()
        tables[0, :n] = new_home
        import dataclasses
        moved_batch = dataclasses.replace(batch, block_tables=tables)
        runners = [AttnRunner(pools[l], moved_batch, qs[l]) for l in range(L)]
        for l in range(L):
            r = runners[l]
            r.ws = torch.empty(pools[l].workspace_bytes(r.desc), dtype=torch.uint8, device=DEV)
            sw.wait_layer(B.IC_SWAP_IN, l, fg.cuda_stream)
            pools[l].paged_attn_mixed(r.desc, r.q.data_ptr(), r.out.data_ptr(), r.ws.data_ptr(), r.ws.numel(),
                                      fg.cuda_stream)
    fg.synchronize()
    sw.sync()
    for l in range(L):
        assert max_abs_err(from_dev_bits(runners[l].out), want[l]) <= 1e-2, l
    pin.close()
    sw.close()
    for p in pools:
        p.close()


def test_pageable_host_memory_is_refused():
    ly = Layers(2, 32, 2, 64, 4, 2, seed=3)
    plain = np.zeros(2 * 4 * ly.bb + 64, dtype=np.uint8)
    addr = (plain.ctypes.data + 15) // 16 * 16
    assert ly.sw.swap_out([1, 2], addr, 4 * ly.bb, check=False) == B.IC_EUNSUPPORTED
    assert ly.sw.swap_in([1, 2], addr, 4 * ly.bb, check=False) == B.IC_EUNSUPPORTED
    # the failed pointer query leaves no error behind: a valid call still works
    pin = B.PinnedBuffer(2 * 4 * ly.bb)
    ly.sw.swap_out([1, 2], pin.ptr, 4 * ly.bb)
    ly.sw.sync()
    assert np.array_equal(pin.array.reshape(2, 4 * ly.bb)[:, :2 * ly.bb], oracle.swap_out_layers(ly.host, [1, 2]))
    torch.cuda.synchronize()
    pin.close()
    ly.close()


def test_13b_shaped_layers_sampled():
    """Two layers of the 13B-shaped swap (320 KiB blocks, 2000 of 20000 per layer): every moved byte
    against the oracle, whose input pools hold the listed blocks fetched from the device."""
    cfg = W.KV_SWAP
    L = 2
    src, dst = W.make_swap_lists(cfg)
    n, bb = cfg.n_move, cfg.block_bytes
    dev = []
    for l in range(L):
        t = torch.empty((cfg.pool_blocks, bb), dtype=torch.uint8, device=DEV)
        W.fill_bytes_device(t, cfg.seed + l)
        dev.append(t)
    pools = [B.KvPool(B.make_cfg(cfg.pool_blocks, cfg.num_heads, cfg.head_dim), t.data_ptr(), t.numel()) for t in dev]
    need = B.LayerSwapper.staging_bytes(pools[0], L, n, 2)
    staging = torch.empty(need, dtype=torch.uint8, device=DEV)
    sw = B.LayerSwapper(pools, n, staging.data_ptr(), need, 2)
    pin = B.PinnedBuffer(L * n * bb)
    sw.swap_out(src, pin.ptr, n * bb)
    sw.sync()
    src_t = torch.from_numpy(src).to(DEV).long()
    compact = [t[src_t].cpu().numpy() for t in dev]                  # the listed blocks, list order
    want = oracle.swap_out_layers(compact, np.arange(n, dtype=np.int32))
    assert np.array_equal(pin.array.reshape(L, n * bb), want)
    sw.swap_in(dst, pin.ptr, n * bb)
    sw.sync()
    dst_t = torch.from_numpy(dst).to(DEV).long()
    for l in range(L):
        assert np.array_equal(dev[l][dst_t].cpu().numpy(), compact[l]), l
        assert torch.equal(dev[l][src_t], torch.from_numpy(compact[l]).to(DEV)), "sources unchanged"
    pin.close()
    sw.close()
    for p in pools:
        p.close()


@pytest.mark.parametrize("seed", range(8))
def test_random_sequences_of_swaps_in_both_directions(seed):
    """Three to thirteen calls in random order and size, both directions in flight at once (on disjoint blocks, as
    the caller must ensure), with and without syncs in between, one to five layers, two to four staging buffers:
    every host buffer and every pool must end up as the per-layer memcpy oracle says."""
    rng = np.random.default_rng(77000 + seed)
    L, stages = int(rng.integers(1, 6)), int(rng.integers(2, 5))
    H, D, nb = int(rng.choice([1, 2, 5])), int(rng.choice([64, 128])), int(rng.integers(8, 200))
    max_blocks = int(rng.integers(1, nb + 1))
    ly = Layers(L, nb, H, D, max_blocks, stages, seed)
    model = [h.copy() for h in ly.host]          # what the pools must hold at the end
    out_busy, in_busy = set(), set()             # blocks a queued swap still reads / writes
    outs, keep = [], []

    def drain():
        ly.sw.sync()
        out_busy.clear()
        in_busy.clear()

    for _ in range(int(rng.integers(3, 14))):
        n = int(rng.integers(1, max_blocks + 1))
        if rng.random() < 0.5:                   # swap-out: duplicates allowed, must not read what a swap-in writes
            free = [b for b in range(nb) if b not in in_busy]
            if not free:
                drain()
                free = list(range(nb))
            ids = rng.choice(free, size=n).astype(np.int32)
            stride = n * ly.bb + 16 * int(rng.integers(0, 3))
            buf = B.PinnedBuffer(L * stride)
            buf.array[:] = 0xEE
            ly.sw.swap_out(ids, buf.ptr, stride)
            out_busy |= set(ids.tolist())
            outs.append((buf, stride, oracle.swap_out_layers(model, ids)))
        else:                                    # swap-in: distinct blocks that no queued swap-out still reads
            free = [b for b in range(nb) if b not in out_busy]
            if len(free) < n:
                drain()
                free = list(range(nb))
            ids = rng.permutation(free)[:n].astype(np.int32)
            buf = B.PinnedBuffer(L * n * ly.bb)
            buf.array[:] = rng.integers(0, 256, size=buf.nbytes, dtype=np.uint8)
            ly.sw.swap_in(ids, buf.ptr, n * ly.bb)
            oracle.swap_in_layers(model, ids, buf.array.reshape(L, n * ly.bb))
            in_busy |= set(ids.tolist())
            keep.append(buf)
        if rng.random() < 0.3:
            drain()
    ly.sw.sync()
    for buf, stride, want in outs:
        n_bytes = want.shape[1]
        for l in range(L):
            assert np.array_equal(buf.array[l * stride: l * stride + n_bytes], want[l]), ("swap-out", l)
    for l in range(L):
        assert np.array_equal(ly.dev[l].cpu().numpy(), model[l]), ("pool", l)
    ly.close()
    for buf, _, _ in outs:
        buf.close()
    for buf in keep:
        buf.close()
