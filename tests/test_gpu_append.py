"""HIP kv_write_span against the oracle, bit for bit, and the append -> attention sequence of one iteration."""
import numpy as np
import pytest
import torch

import oracle
from paper_2402_01869_amd import binding as B
from paper_2402_01869_amd import workloads as W
from gpu_common import DEV, AttnRunner, from_dev_bits, make_pool, max_abs_err, to_dev_bits

pytestmark = pytest.mark.gpu


def _append_and_compare(batch, seed, extra_rows=0):
    rng = np.random.default_rng(seed)
    H, D = batch.num_heads, batch.head_dim
    pool_bits = W.randn_bf16(W.pool_shape(batch.pool_blocks, H, 16, D), rng)
    rows = batch.total_q_rows + extra_rows                   # trailing rows no sequence owns
    k_new, v_new = W.randn_bf16((rows, H, D), rng), W.randn_bf16((rows, H, D), rng)
    want = pool_bits.copy()
    oracle.kv_append(want, batch.ctx_len, batch.q_len, batch.q_start, batch.block_tables, k_new, v_new)
    pool, pool_t = make_pool(pool_bits)
    desc = B.HostDesc(batch.ctx_len, batch.q_len, batch.q_start, batch.block_tables, batch.scale, rows)
    k_t, v_t = to_dev_bits(k_new), to_dev_bits(v_new)
    pool.kv_write_span(desc, k_t.data_ptr(), v_t.data_ptr())
    torch.cuda.synchronize()
    assert np.array_equal(from_dev_bits(pool_t), want)
    pool.close()


def test_tiny_config_append_bit_exact():
    _append_and_compare(W.make_batch(W.TINY), 1)


@pytest.mark.parametrize("D", [64, 128, 256])
@pytest.mark.parametrize("H", [1, 5])
def test_append_edge_lengths(D, H):
    """Positions at block boundaries, whole prefills from position 0, single tokens, rows nobody owns."""
    ctx = [1, 15, 16, 17, 31, 32, 33, 64, 65, 100, 257, 300, 40, 129]
    qlen = [1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 40, 33]
    batch = W.assemble_batch(H, D, 16, 96, ctx, qlen, np.random.default_rng(D + H))
    _append_and_compare(batch, 10 + D + H, extra_rows=3)


def test_append_then_attention_is_one_iteration():
    """The chunk's positions hold NaN patterns until kv_write_span fills them; attention on the same
    stream right after must see the new keys (no host wait in between)."""
    H, D = 5, 128
    rng = np.random.default_rng(77)
    batch = W.assemble_batch(H, D, 16, 256, [700, 300, 129, 1000, 64], [200, 300, 128, 1, 1], rng)
    full_pool, q_bits = W.make_host_inputs(batch, 78, poison_unused=True)
    want = oracle.attn_batch(batch, full_pool, q_bits)
    # take the chunk's own K/V out of the cache into k_new / v_new
    start = full_pool.copy()
    k_new = np.zeros((batch.total_q_rows, H, D), dtype=np.uint16); v_new = np.zeros_like(k_new)
    for s in range(batch.num_seqs):
        for i in range(int(batch.q_len[s])):
            t = int(batch.ctx_len[s] - batch.q_len[s]) + i
            blk = int(batch.block_tables[s, t // 16])
            k_new[batch.q_start[s] + i] = full_pool[blk, 0, :, t % 16, :]
            v_new[batch.q_start[s] + i] = full_pool[blk, 1, :, t % 16, :]
            start[blk, :, :, t % 16, :] = 0x7FFF
    pool, pool_t = make_pool(start)
    r = AttnRunner(pool, batch, q_bits)
    r.ws = torch.empty(pool.workspace_bytes(r.desc), dtype=torch.uint8, device=DEV)
    k_t, v_t = to_dev_bits(k_new), to_dev_bits(v_new)
    st = torch.cuda.Stream()
    torch.cuda.synchronize()
    pool.kv_write_span(r.desc, k_t.data_ptr(), v_t.data_ptr(), st.cuda_stream)
    pool.paged_attn_mixed(r.desc, r.q.data_ptr(), r.out.data_ptr(), r.ws.data_ptr(), r.ws.numel(), st.cuda_stream)
    st.synchronize()
    assert np.array_equal(from_dev_bits(pool_t), full_pool)
    assert max_abs_err(from_dev_bits(r.out), want) <= 1e-2
    pool.close()


def test_planned_append_and_attention_over_layers():
    """An iteration over three layers from one plan: kv_write_span_planned then paged_attn_planned per layer,
    no descriptor traffic after the plan; caches and outputs equal the oracle's, layer by layer."""
    H, D, L = 4, 128, 3
    rng = np.random.default_rng(91)
    batch = W.assemble_batch(H, D, 16, 200, [500, 300, 129, 1000, 64], [100, 300, 128, 1, 1], rng)
    desc = B.HostDesc.from_batch(batch)
    pools, tensors, wants, outs, qs, knews, vnews, want_pools = [], [], [], [], [], [], [], []
    for l in range(L):
        r = np.random.default_rng(300 + l)
        start = W.randn_bf16(W.pool_shape(200, H, 16, D), r)
        k_new, v_new = W.randn_bf16((batch.total_q_rows, H, D), r), W.randn_bf16((batch.total_q_rows, H, D), r)
        q_bits = W.randn_bf16((batch.total_q_rows, H, D), r)
        full = start.copy()
        oracle.kv_append(full, batch.ctx_len, batch.q_len, batch.q_start, batch.block_tables, k_new, v_new)
        want_pools.append(full)
        wants.append(oracle.attn_batch(batch, full, q_bits))
        pool, t = make_pool(start)
        pools.append(pool); tensors.append(t)
        qs.append(to_dev_bits(q_bits)); knews.append(to_dev_bits(k_new)); vnews.append(to_dev_bits(v_new))
        outs.append(torch.full((batch.total_q_rows, H, D), 0x7FFF, dtype=torch.int16, device=DEV))
    ws = torch.empty(pools[0].workspace_bytes(desc), dtype=torch.uint8, device=DEV)
    st = torch.cuda.Stream()
    torch.cuda.synchronize()
    plan = pools[0].plan_create(desc, ws.data_ptr(), ws.numel(), st.cuda_stream)
    for l in range(L):
        pools[l].kv_write_span_planned(plan, knews[l].data_ptr(), vnews[l].data_ptr(), st.cuda_stream)
        pools[l].paged_attn_planned(plan, qs[l].data_ptr(), outs[l].data_ptr(), st.cuda_stream)
    st.synchronize()
    for l in range(L):
        assert np.array_equal(from_dev_bits(tensors[l]), want_pools[l]), l
        assert max_abs_err(from_dev_bits(outs[l]), wants[l]) <= 1e-2, l
    plan.close()
    # a plan whose (checked) descriptor has two rows on one slot refuses the append
    s0, s1 = 3, 4
    ctx = batch.ctx_len.copy(); ctx[s1] = ctx[s0]
    bt = batch.block_tables.copy(); bt[s1] = bt[s0]
    dup = B.HostDesc(ctx, batch.q_len, batch.q_start, bt, batch.scale, batch.total_q_rows)
    ws2 = torch.empty(pools[0].workspace_bytes(dup), dtype=torch.uint8, device=DEV)
    plan2 = pools[0].plan_create(dup, ws2.data_ptr(), ws2.numel())
    assert pools[0].kv_write_span_planned(plan2, knews[0].data_ptr(), vnews[0].data_ptr(), check=False) == B.IC_EDUP
    torch.cuda.synchronize()
    plan2.close()
    for p in pools:
        p.close()


def test_mixed_13b_shape_append_sampled():
    """13B-shaped mixed batch (4224 rows, H40 D128, pool of 65536 blocks): every written slot against
    the oracle run on the blocks the batch references, and a checksum over the rest of the pool."""
    cfg = W.MIXED_13B
    batch = W.make_batch(cfg)
    H, D = cfg.num_heads, cfg.head_dim
    pool_t = torch.empty(W.pool_shape(cfg.pool_blocks, H, 16, D), dtype=torch.bfloat16, device=DEV)
    W.fill_pool_device_normal(pool_t, cfg.seed)
    rng = np.random.default_rng(5)
    k_new, v_new = W.randn_bf16((batch.total_q_rows, H, D), rng), W.randn_bf16((batch.total_q_rows, H, D), rng)
    # blocks that receive rows, fetched before the call: the oracle's input
    touched = []
    for s in range(batch.num_seqs):
        t0 = int(batch.ctx_len[s] - batch.q_len[s])
        touched += [int(batch.block_tables[s, t // 16]) for t in range(t0, int(batch.ctx_len[s]))]
    touched = np.unique(np.array(touched, dtype=np.int64))
    remap = {int(b): j for j, b in enumerate(touched)}
    idx = torch.from_numpy(touched).to(DEV)
    view = pool_t.view(torch.int16)
    small = from_dev_bits(view[idx])
    tables = np.zeros_like(batch.block_tables)
    for s in range(batch.num_seqs):
        t0 = int(batch.ctx_len[s] - batch.q_len[s])
        for j in range(t0 // 16, (int(batch.ctx_len[s]) - 1) // 16 + 1):
            tables[s, j] = remap[int(batch.block_tables[s, j])]
    oracle.kv_append(small, batch.ctx_len, batch.q_len, batch.q_start, tables, k_new, v_new)
    mask = torch.ones(cfg.pool_blocks, dtype=torch.bool, device=DEV); mask[idx] = False
    rest_before = view[mask].to(torch.int64).sum().item()
    pool = B.KvPool.from_tensor(pool_t, H, D)
    desc = B.HostDesc.from_batch(batch, flags=B.IC_FLAG_TRUSTED)
    k_t, v_t = to_dev_bits(k_new), to_dev_bits(v_new)
    pool.kv_write_span(desc, k_t.data_ptr(), v_t.data_ptr())
    torch.cuda.synchronize()
    assert np.array_equal(from_dev_bits(view[idx]), small)
    assert view[mask].to(torch.int64).sum().item() == rest_before, "blocks outside the batch's new positions changed"
    pool.close()


def test_repeated_batches_and_the_trusted_flag():
    """kv_write_span keeps the device copy of the rows' destinations and skips the upload when the next call's batch
    has the same ones (every layer of an iteration).  Same batch with new K/V rows, another batch, the first again:
    always the oracle's bytes.  A destination list uploaded under IC_FLAG_TRUSTED has not been checked: the same
    list without the flag is still checked (two rows on one slot are refused)."""
    H, D = 3, 64
    rng = np.random.default_rng(5)
    b1 = W.assemble_batch(H, D, 16, 64, [40, 17, 100, 5], [1, 17, 30, 1], rng)
    b2 = W.assemble_batch(H, D, 16, 64, [33, 64, 90, 9], [1, 20, 27, 1], rng)
    assert b1.total_q_rows == b2.total_q_rows
    pool_bits = W.randn_bf16(W.pool_shape(64, H, 16, D), rng)
    want = pool_bits.copy()
    pool, pool_t = make_pool(pool_bits)
    for step, b in enumerate([b1, b1, b2, b1, b2, b2]):
        k_new, v_new = W.randn_bf16((b.total_q_rows, H, D), rng), W.randn_bf16((b.total_q_rows, H, D), rng)
        oracle.kv_append(want, b.ctx_len, b.q_len, b.q_start, b.block_tables, k_new, v_new)
        k_t, v_t = to_dev_bits(k_new), to_dev_bits(v_new)
        pool.kv_write_span(B.HostDesc.from_batch(b), k_t.data_ptr(), v_t.data_ptr())
        torch.cuda.synchronize()
        assert np.array_equal(from_dev_bits(pool_t), want), step
    # two decode sequences whose new tokens land on one slot
    dup = W.assemble_batch(H, D, 16, 64, [40, 40, 9], [1, 1, 1], rng)
    dup.block_tables[1] = dup.block_tables[0]
    k_t = to_dev_bits(W.randn_bf16((3, H, D), rng))
    assert pool.kv_write_span(B.HostDesc.from_batch(dup, flags=B.IC_FLAG_TRUSTED), k_t.data_ptr(), k_t.data_ptr(), check=False) == B.IC_OK
    torch.cuda.synchronize()
    assert pool.kv_write_span(B.HostDesc.from_batch(dup), k_t.data_ptr(), k_t.data_ptr(), check=False) == B.IC_EDUP
    pool.close()
