"""Pins of the CPU oracle against closed forms, invariants, library routines and brute force.

The paper prints no worked attention or swap values, so the oracle is pinned by what the
mathematics fixes.  Each test names the mistake it is meant to catch.
"""
import math

import numpy as np
import pytest

import oracle
from paper_2402_01869_amd import workloads as W
from helpers import bits, dense_causal_attention, paged_pool_from_dense

B = 16


def _single(K, V, q, scale, q_len=None, table=None, num_blocks=None, rng=None):
    """Run the oracle on one sequence given dense bf16-bit K, V [ctx][H][D] and q [n][H][D]."""
    ctx, H, D = K.shape
    nb = -(-ctx // B)
    num_blocks = num_blocks or (nb + 3)
    if table is None:
        rng = rng or np.random.default_rng(0)
        table = rng.permutation(num_blocks)[:nb].astype(np.int32)
    pool = paged_pool_from_dense(K, V, table, B, num_blocks)
    n = q.shape[0] if q_len is None else q_len
    return oracle.paged_attn(pool, [ctx], [n], [0], table[None, :], q, scale)


def test_single_key_returns_v0():
    # softmax over one key is 1: out == v_0 exactly.  Catches K/V offset mix-ups at slot 0.
    rng = np.random.default_rng(1)
    K, V, q = (W.randn_bf16((1, 3, 8), rng) for _ in range(3))
    out = _single(K, V, q, 0.35)
    assert np.array_equal(out[0], W.bf16_bits_to_f64(V[0]))


def test_constant_v_returns_v():
    # weights sum to one: a constant V comes back whatever Q and K are.  Catches a wrong normaliser.
    rng = np.random.default_rng(2)
    ctx, H, D, n = 45, 2, 16, 9
    K = W.randn_bf16((ctx, H, D), rng)
    c = W.randn_bf16((1, H, D), rng)
    V = np.repeat(c, ctx, axis=0)
    q = W.randn_bf16((n, H, D), rng)
    out = _single(K, V, q, 1 / 4)
    want = np.broadcast_to(W.bf16_bits_to_f64(c), out.shape)
    assert np.allclose(out, want, rtol=0, atol=1e-13)


@pytest.mark.parametrize("ctx,n", [(37, 1), (37, 37), (50, 20), (16, 16), (33, 2)])
def test_uniform_scores_give_running_mean(ctx, n):
    # q = 0 -> every visible key weighs the same; with v_t = t the answer is p_i / 2 exactly.
    # Catches a causal off-by-one (row i must see keys 0..p_i inclusive, p_i = ctx - n + i).
    H, D = 2, 8
    rng = np.random.default_rng(3)
    K = W.randn_bf16((ctx, H, D), rng)
    V = bits(np.broadcast_to(np.arange(ctx, dtype=np.float32)[:, None, None], (ctx, H, D)))
    q = np.zeros((n, H, D), dtype=np.uint16)
    out = _single(K, V, q, 0.5)
    for i in range(n):
        p = ctx - n + i
        assert np.allclose(out[i], p / 2.0, rtol=0, atol=1e-12), (i, p)


def test_scale_zero_is_uniform():
    rng = np.random.default_rng(4)
    ctx, H, D = 21, 1, 8
    K, q = W.randn_bf16((ctx, H, D), rng), W.randn_bf16((1, H, D), rng)
    V = bits(np.broadcast_to(np.arange(ctx, dtype=np.float32)[:, None, None], (ctx, H, D)))
    out = _single(K, V, q, 0.0)
    assert np.allclose(out, (ctx - 1) / 2.0, atol=1e-12)


def test_peaked_score_pins_block_table_gather():
    # One key is aligned with q and large, the rest are orthogonal: out -> v_{t*} up to a bounded
    # residual.  V encodes (head, physical block, slot), so a wrong block, slot, head or K/V plane shows.
    H, D, ctx = 3, 8, 70
    nb = -(-ctx // B)
    num_blocks = 11
    rng = np.random.default_rng(5)
    table = rng.permutation(num_blocks)[:nb].astype(np.int32)
    lam, scale = 64.0, 0.5
    for tstar in [0, 1, 15, 16, 17, 31, 32, 48, 69]:
        K = np.zeros((ctx, H, D), dtype=np.float32)
        q = np.zeros((1, H, D), dtype=np.float32)
        for h in range(H):
            q[0, h, h] = 1.0                 # unit vector, different axis per head
            K[:, h, (h + 1) % D] = 1.0       # orthogonal to q
            K[tstar, h, :] = 0.0
            K[tstar, h, h] = lam
        V = np.zeros((ctx, H, D), dtype=np.float32)
        for t in range(ctx):
            for h in range(H):
                V[t, h, 0] = table[t // B]    # physical block
                V[t, h, 1] = t % B            # slot
                V[t, h, 2] = h
                V[t, h, 3] = t
        out = _single(bits(K), bits(V), bits(q), scale, table=table, num_blocks=num_blocks)
        resid = (ctx - 1) * math.exp(-lam * scale) * ctx   # weight bound x value bound
        want = V[tstar].astype(np.float64)
        assert np.allclose(out[0], want, rtol=0, atol=resid + 1e-12), tstar


def test_two_keys_logistic_closed_form():
    # out = sigma(s0 - s1) v0 + sigma(s1 - s0) v1, computed by hand here.  Catches a dropped scale,
    # a sign error in the exponent, or transposed q/k operands.
    q = np.array([[[0.5, -1.0, 2.0, 0.25]]], dtype=np.float32)
    K = np.array([[[1.0, 0.5, 0.25, -2.0]], [[-0.5, 1.5, 1.0, 0.75]]], dtype=np.float32)
    V = np.array([[[1.0, -2.0, 3.0, 0.5]], [[-4.0, 0.25, 8.0, 1.5]]], dtype=np.float32)
    scale = 0.7
    s0 = scale * float((q[0, 0] * K[0, 0]).sum())
    s1 = scale * float((q[0, 0] * K[1, 0]).sum())
    w0 = 1.0 / (1.0 + math.exp(s1 - s0))
    want = w0 * V[0, 0].astype(np.float64) + (1.0 - w0) * V[1, 0].astype(np.float64)
    out = _single(bits(K), bits(V), bits(q), scale)
    assert np.allclose(out[0, 0], want, rtol=0, atol=1e-14)
    # row 0 of a 2-row span sees only key 0
    q2 = np.concatenate([q, q], axis=0)
    out2 = _single(bits(K), bits(V), bits(q2), scale)
    assert np.array_equal(out2[0, 0], V[0, 0].astype(np.float64))
    assert np.allclose(out2[1, 0], want, rtol=0, atol=1e-14)


@pytest.mark.parametrize("ctx,n,H,D", [(100, 1, 4, 64), (100, 100, 2, 32), (77, 32, 3, 16), (16, 5, 1, 128)])
def test_paged_equals_dense_numpy(ctx, n, H, D):
    # Paging is a pure re-mapping (Section 3.1): the paged result equals dense contiguous attention.
    rng = np.random.default_rng(6)
    K, V = W.randn_bf16((ctx, H, D), rng), W.randn_bf16((ctx, H, D), rng)
    q = W.randn_bf16((n, H, D), rng)
    scale = 1 / math.sqrt(D)
    out = _single(K, V, q, scale, rng=rng)
    want = dense_causal_attention(W.bf16_bits_to_f64(q), W.bf16_bits_to_f64(K), W.bf16_bits_to_f64(V),
                                  scale, ctx - n)
    assert np.allclose(out, want, rtol=0, atol=1e-13)


def test_matches_torch_cpu_fp64():
    # Second independent reference: plain torch CPU ops in fp64 (softmax(QK^T scale + mask) @ V).
    import torch
    rng = np.random.default_rng(7)
    ctx, n, H, D = 130, 40, 2, 64
    K, V = W.randn_bf16((ctx, H, D), rng), W.randn_bf16((ctx, H, D), rng)
    q = W.randn_bf16((n, H, D), rng)
    scale = 1 / math.sqrt(D)
    out = _single(K, V, q, scale, rng=rng)
    tq, tk, tv = (torch.from_numpy(W.bf16_bits_to_f64(a)).permute(1, 0, 2) for a in (q, K, V))
    s = tq @ tk.transpose(1, 2) * scale
    pos = (ctx - n) + torch.arange(n)[:, None]
    s = s.masked_fill(torch.arange(ctx)[None, :] > pos, float("-inf"))
    want = (torch.softmax(s, dim=-1) @ tv).permute(1, 0, 2).numpy()
    assert np.allclose(out, want, rtol=0, atol=1e-13)


def test_brute_force_tiny_pure_python():
    # Third formulation: sum_t e^{s_t} v_t / sum_t e^{s_t} with no max subtraction, python floats + fsum.
    rng = np.random.default_rng(8)
    ctx, n, H, D = 19, 4, 2, 4
    K, V, q = (W.randn_bf16(s, rng) for s in ((ctx, H, D), (ctx, H, D), (n, H, D)))
    scale = 0.5
    out = _single(K, V, q, scale, rng=rng)
    Kf, Vf, qf = (W.bf16_bits_to_f64(a) for a in (K, V, q))
    for i in range(n):
        p = ctx - n + i
        for h in range(H):
            e = [math.exp(scale * math.fsum(qf[i, h, d] * Kf[t, h, d] for d in range(D))) for t in range(p + 1)]
            z = math.fsum(e)
            for d in range(D):
                want = math.fsum(e[t] * Vf[t, h, d] for t in range(p + 1)) / z
                assert abs(out[i, h, d] - want) < 1e-12


def test_physical_permutation_invariance_bit_identical():
    # Relabelling physical blocks consistently changes nothing, bit for bit.
    rng = np.random.default_rng(9)
    cfg = W.TINY
    batch = W.make_batch(cfg, seed=99)
    pool, q = W.make_host_inputs(batch, seed=99)
    out1 = oracle.attn_batch(batch, pool, q)
    perm = rng.permutation(cfg.pool_blocks)
    pool2 = np.empty_like(pool)
    pool2[perm] = pool                       # block b moves to perm[b]
    tables2 = np.where(batch.block_tables >= 0, perm[np.clip(batch.block_tables, 0, None)], -1).astype(np.int32)
    out2 = oracle.paged_attn(pool2, batch.ctx_len, batch.q_len, batch.q_start, tables2, q, batch.scale)
    assert np.array_equal(out1, out2)


@pytest.mark.parametrize("chunk", [1, 7, 16, 32, 83])
def test_chunked_recompute_equals_one_shot_prefill(chunk):
    # Recomputing a context chunk by chunk over successive iterations, with ctx_len growing
    # (Section 4.2 and the partial-recompute rule of Section 4.3), reproduces the one-shot causal
    # prefill.  chunk = 1 also shows that a decode row equals the matching prefill row.
    rng = np.random.default_rng(10)
    L, H, D = 83, 2, 16
    K, V, q = (W.randn_bf16((L, H, D), rng) for _ in range(3))
    nb = -(-L // B)
    table = rng.permutation(nb + 2)[:nb].astype(np.int32)
    pool = paged_pool_from_dense(K, V, table, B, nb + 2)
    scale = 0.25
    full = oracle.paged_attn(pool, [L], [L], [0], table[None], q, scale)
    pieces = []
    done = 0
    while done < L:
        n = min(chunk, L - done)
        ctx = done + n
        # later tokens are not yet "recomputed": poison them to prove they are never read
        pool_c = pool.copy()
        for t in range(ctx, nb * B):
            pool_c[table[t // B], :, :, t % B, :] = 0x7FFF
        pieces.append(oracle.paged_attn(pool_c, [ctx], [n], [0], table[None], q[done:ctx], scale))
        done = ctx
    got = np.concatenate(pieces, axis=0)
    assert np.allclose(got, full, rtol=0, atol=1e-14)
    assert np.isfinite(got).all()


def test_common_score_shift_leaves_output_unchanged():
    # An extra dimension with q = 1, k_t = c adds the same constant to every score.
    rng = np.random.default_rng(11)
    ctx, H, D = 40, 2, 8
    K, V, q = (W.bf16_bits_to_f64(W.randn_bf16(s, rng)) for s in ((ctx, H, D), (ctx, H, D), (3, H, D)))
    base = _single(bits(K), bits(V), bits(q), 0.3)
    K2 = np.concatenate([K, np.full((ctx, H, 1), 24.0)], axis=-1)
    q2 = np.concatenate([q, np.ones((3, H, 1))], axis=-1)
    V2 = np.concatenate([V, np.zeros((ctx, H, 1))], axis=-1)
    shifted = _single(bits(K2), bits(V2), bits(q2), 0.3)
    assert np.allclose(shifted[..., :D], base, rtol=0, atol=1e-13)


def test_batch_equals_per_sequence_calls_and_poison_is_ignored():
    # A multi-sequence batch equals one call per sequence (catches q_start / table-row stride errors),
    # and NaN in every don't-care slot leaves the output finite and unchanged.
    batch = W.make_batch(W.TINY)
    clean, q = W.make_host_inputs(batch, seed=W.TINY.seed, poison_unused=False)
    poisoned = clean.copy()
    W.poison_pool(poisoned, batch)
    assert not np.array_equal(clean, poisoned)
    out_clean = oracle.attn_batch(batch, clean, q)
    out_pois = oracle.attn_batch(batch, poisoned, q)
    assert np.isfinite(out_pois).all()
    assert np.array_equal(out_clean, out_pois)
    for s in range(batch.num_seqs):
        n, c, r0 = int(batch.q_len[s]), int(batch.ctx_len[s]), int(batch.q_start[s])
        ids = batch.blocks_of(s)
        one = oracle.paged_attn(poisoned, [c], [n], [0], ids[None], q[r0:r0 + n], batch.scale)
        assert np.array_equal(one, out_pois[r0:r0 + n])
    assert batch.q_len.tolist()[:2] == [1, 1] and (batch.q_len[2:] > 1).all()


def test_items_subset_matches_full():
    batch = W.make_batch(W.TINY)
    pool, q = W.make_host_inputs(batch, seed=W.TINY.seed)
    full = oracle.attn_batch(batch, pool, q)
    iseq = [3, 0, 2, 2]
    irow = [int(batch.q_len[3]) - 1, 0, 0, 5]
    sub = oracle.paged_attn_items(pool, batch.ctx_len, batch.q_len, batch.q_start, batch.block_tables,
                                  q, batch.scale, iseq, irow)
    for k, (s, i) in enumerate(zip(iseq, irow)):
        assert np.array_equal(sub[k], full[batch.q_start[s] + i])


def test_statistics_at_moderate_shape():
    # N(0,1) inputs with scale 1/sqrt(D): scores ~ N(0,1), so out has mean ~ 0 and
    # variance ~ sum w_t^2 ~ e / ctx.  A coarse check that shapes and scale are wired as intended.
    rng = np.random.default_rng(12)
    ctx, H, D = 2048, 4, 128
    K, V = W.randn_bf16((ctx, H, D), rng), W.randn_bf16((ctx, H, D), rng)
    q = W.randn_bf16((1, H, D), rng)
    out = _single(K, V, q, 1 / math.sqrt(D), rng=rng)
    assert abs(out.mean()) < 0.02
    assert 0.3 * math.e / ctx < out.var() < 3.0 * math.e / ctx


def test_oracle_rejects_bad_descriptors():
    batch = W.make_batch(W.TINY)
    pool, q = W.make_host_inputs(batch, seed=1)
    bad = batch.block_tables.copy()
    bad[0, 0] = W.TINY.pool_blocks
    with pytest.raises(oracle.OracleError):
        oracle.paged_attn(pool, batch.ctx_len, batch.q_len, batch.q_start, bad, q, batch.scale)
    ql = batch.q_len.copy()
    ql[0] = batch.ctx_len[0] + 1
    with pytest.raises(oracle.OracleError):
        oracle.paged_attn(pool, batch.ctx_len, ql, batch.q_start, batch.block_tables, q, batch.scale)


# ------------------------------------------------------------------ swap (Section 3.2)

def test_pack_equals_numpy_fancy_index_and_roundtrip():
    cfg = W.TINY_SWAP
    pool = W.random_pool_bytes(cfg)
    src, dst = W.make_swap_lists(cfg)
    assert len(set(src.tolist())) == cfg.n_move and not set(src.tolist()) & set(dst.tolist())
    staging = oracle.pack_blocks(pool, src)
    assert np.array_equal(staging, pool[src])          # library gather, list order
    before = pool.copy()
    oracle.unpack_blocks(pool, dst, staging)
    assert np.array_equal(pool[dst], before[src])      # swapped-in context restored
    untouched = np.setdiff1d(np.arange(cfg.pool_blocks), dst)
    assert np.array_equal(pool[untouched], before[untouched])
    # unpack to the same ids is the identity on the whole pool
    pool2 = before.copy()
    oracle.unpack_blocks(pool2, src, oracle.pack_blocks(pool2, src))
    assert np.array_equal(pool2, before)


def test_pack_order_duplicates_and_errors():
    pool = np.arange(6 * 32, dtype=np.uint8).reshape(6, 32)
    st = oracle.pack_blocks(pool, [4, 1, 4])           # duplicate sources are legal
    assert np.array_equal(st, pool[[4, 1, 4]])
    assert oracle.pack_blocks(pool, []).shape == (0, 32)
    with pytest.raises(oracle.OracleError):
        oracle.pack_blocks(pool, [6])
    with pytest.raises(oracle.OracleError):
        oracle.unpack_blocks(pool.copy(), [2, 2], st[:2])   # duplicate destinations
    with pytest.raises(oracle.OracleError):
        oracle.unpack_blocks(pool.copy(), [-1], st[:1])


# ---------------------------------------------------------------------------------------------
# Section 4.1: layer-pipelined, chunked swap
# ---------------------------------------------------------------------------------------------
def _layer_pools(L, nb, bb, seed):
    rng = np.random.default_rng(seed)
    return [rng.integers(0, 256, size=(nb, bb), dtype=np.uint8) for _ in range(L)]


def test_swap_out_layers_equals_numpy_gather_per_layer():
    # Catches: a layer written to another layer's slice, list order lost, stride ignored.
    L, nb, bb = 5, 23, 48
    pools = _layer_pools(L, nb, bb, 3)
    ids = np.array([7, 0, 22, 7, 3], dtype=np.int32)       # duplicate sources are legal on the way out
    stride = len(ids) * bb + 32                            # padded layer stride
    host = oracle.swap_out_layers(pools, ids, stride)
    assert host.shape == (L, stride)
    for l in range(L):
        assert np.array_equal(host[l, :len(ids) * bb].reshape(len(ids), bb), pools[l][ids])
        assert (host[l, len(ids) * bb:] == 0xEE).all()     # padding untouched


def test_swap_in_layers_inverts_swap_out_and_touches_nothing_else():
    # out to host, wipe the pools, in to OTHER blocks: the listed blocks reappear, all others keep
    # their bytes.  Catches: scatter through the wrong list, a layer skipped, writes off the list.
    L, nb, bb = 4, 40, 64
    pools = _layer_pools(L, nb, bb, 4)
    orig = [p.copy() for p in pools]
    rng = np.random.default_rng(5)
    perm = rng.permutation(nb).astype(np.int32)
    src, dst = perm[:9], perm[9:18]
    host = oracle.swap_out_layers(pools, src)
    oracle.swap_in_layers(pools, dst, host)
    for l in range(L):
        assert np.array_equal(pools[l][dst], orig[l][src])
        others = np.setdiff1d(np.arange(nb), dst)
        assert np.array_equal(pools[l][others], orig[l][others])
    # back to the same ids: identity on every pool
    pools2 = [p.copy() for p in orig]
    oracle.swap_in_layers(pools2, src, oracle.swap_out_layers(pools2, src))
    assert all(np.array_equal(a, b) for a, b in zip(pools2, orig))


def test_swap_layers_reject_bad_lists():
    pools = _layer_pools(2, 8, 16, 6)
    with pytest.raises(oracle.OracleError):
        oracle.swap_out_layers(pools, [1, 8])
    host = oracle.swap_out_layers(pools, [1, 2])
    with pytest.raises(oracle.OracleError):
        oracle.swap_in_layers(pools, [3, 3], host)         # duplicate destinations
    with pytest.raises(oracle.OracleError):
        oracle.swap_out_layers(pools, [1, 2], layer_stride=16)   # stride shorter than the payload


def test_swap_limit_solves_t_swap_equals_t_fwd():
    # Worked by hand: 13B-shaped M = 40 layers x 20 KiB = 819 200 B per token; a 30 ms forward pass
    # over a 32 GB/s link hides 0.03 * 32e9 / 819200 = 1171.875 -> 1171 tokens.
    assert oracle.swap_limit_tokens(0.030, 32e9, 819200) == 1171
    # exact cases (powers of two keep fp64 exact): T_swap(N) = N * M / BW = T_fwd has the root N
    assert oracle.swap_limit_tokens(0.5, 2.0 ** 30, 2.0 ** 20) == 512
    assert oracle.swap_limit_tokens(0.0, 1e9, 1024) == 0
    # defining property on random inputs: N moves in time, N + 1 does not.  Catches an inverted
    # ratio (M / BW), a rounding up, and a bits/bytes factor.
    rng = np.random.default_rng(7)
    for _ in range(200):
        t = float(rng.uniform(1e-3, 0.2)); bw = float(rng.uniform(1e9, 128e9)); m = float(rng.integers(1024, 4 << 20))
        n = oracle.swap_limit_tokens(t, bw, m)
        assert n * m / bw <= t * (1 + 1e-12) and (n + 1) * m / bw > t * (1 - 1e-12)
    # doubling the link or the time doubles the limit (up to the rounding), doubling M halves it
    assert oracle.swap_limit_tokens(0.04, 64e9, 1 << 20) in (2 * oracle.swap_limit_tokens(0.04, 32e9, 1 << 20),
                                                             2 * oracle.swap_limit_tokens(0.04, 32e9, 1 << 20) + 1)
    assert oracle.swap_limit_tokens(-1.0, 1e9, 1024) == -1 and oracle.swap_limit_tokens(1.0, 0.0, 1024) == -1


def test_swap_schedule_respects_limits_and_moves_everything_once():
    # brute force in plain Python next to the oracle; catches: rounding blocks up past the limit,
    # moving more than is left, dropping the remainder.
    rng = np.random.default_rng(8)
    for _ in range(100):
        total = int(rng.integers(0, 200)); bs = int(rng.choice([1, 8, 16]))
        limits = rng.integers(0, 40 * bs, size=int(rng.integers(1, 30))).astype(np.int64)
        used, blocks = oracle.swap_schedule(total, bs, limits)
        assert (blocks * bs <= limits).all() and (blocks >= 0).all()
        left, want, want_used = total, [], 0
        for i, lim in enumerate(limits):
            mv = min(left, int(lim) // bs); want.append(mv); left -= mv
            if mv:
                want_used = i + 1
        assert list(blocks) == want
        if left:
            assert used == len(limits) + 1 and blocks.sum() == total - left
        else:
            assert used == want_used and blocks.sum() == total
    # hand example: 10 blocks of 16 tokens under limits 40, 16, 15, 100, 100 tokens -> 2, 1, 0, 6, 1
    used, blocks = oracle.swap_schedule(10, 16, [40, 16, 15, 100, 100])
    assert used == 5 and list(blocks) == [2, 1, 0, 6, 1]


# ---------------------------------------------------------------------------------------------
# KV append (Sections 4.2, 4.3): a chunk's own keys / values enter the paged cache before it attends
# ---------------------------------------------------------------------------------------------
def _append_case(seed, H=3, D=16, nb=40, ctx=(50, 17, 33, 16), qlen=(20, 1, 33, 5)):
    rng = np.random.default_rng(seed)
    batch = W.assemble_batch(H, D, B, nb, list(ctx), list(qlen), rng)
    pool = W.randn_bf16(W.pool_shape(nb, H, B, D), rng)
    k_new = W.randn_bf16((batch.total_q_rows, H, D), rng)
    v_new = W.randn_bf16((batch.total_q_rows, H, D), rng)
    return batch, pool, k_new, v_new


def test_kv_append_equals_slot_by_slot_numpy_writes_and_touches_nothing_else():
    # Catches: K/V planes swapped, position off by one, slot/block index transposed, head stride wrong.
    batch, pool, k_new, v_new = _append_case(21)
    want = pool.copy()
    touched = np.zeros(pool.shape[:1] + pool.shape[3:4], dtype=bool)           # [block][slot]
    for s in range(batch.num_seqs):
        for i in range(int(batch.q_len[s])):
            t = int(batch.ctx_len[s] - batch.q_len[s]) + i
            blk = int(batch.block_tables[s, t // B])
            want[blk, 0, :, t % B, :] = k_new[batch.q_start[s] + i]
            want[blk, 1, :, t % B, :] = v_new[batch.q_start[s] + i]
            touched[blk, t % B] = True
    got = pool.copy()
    oracle.kv_append(got, batch.ctx_len, batch.q_len, batch.q_start, batch.block_tables, k_new, v_new)
    assert np.array_equal(got, want)
    keep = ~touched
    assert np.array_equal(got.transpose(0, 3, 1, 2, 4)[keep], pool.transpose(0, 3, 1, 2, 4)[keep])
    assert touched.sum() == batch.total_q_rows


def test_kv_append_then_attention_equals_dense_attention_on_the_new_keys():
    # The appended rows must be exactly what attention then reads at those positions: append K/V for the
    # chunk, run the paged oracle, compare with dense attention on prefix + chunk (independent numpy).
    rng = np.random.default_rng(22)
    H, D, ctx, n = 2, 32, 77, 30
    K = W.randn_bf16((ctx, H, D), rng); V = W.randn_bf16((ctx, H, D), rng); q = W.randn_bf16((n, H, D), rng)
    table = rng.permutation(12)[:-(-ctx // B)].astype(np.int32)
    Kp, Vp = K.copy(), V.copy()
    Kp[ctx - n:] = 0x7FFF; Vp[ctx - n:] = 0x7FFF                               # chunk positions not yet written
    pool = paged_pool_from_dense(Kp, Vp, table, B, 12)
    oracle.kv_append(pool, [ctx], [n], [0], table[None, :], K[ctx - n:], V[ctx - n:])
    out = oracle.paged_attn(pool, [ctx], [n], [0], table[None, :], q, 0.2)
    want = dense_causal_attention(W.bf16_bits_to_f64(q), W.bf16_bits_to_f64(K), W.bf16_bits_to_f64(V), 0.2, ctx - n)
    assert np.abs(out - want).max() < 1e-12


@pytest.mark.parametrize("chunk", [1, 7, 16, 40])
def test_kv_append_chunk_by_chunk_equals_one_shot(chunk):
    # Section 4.3: a context recomputed over several iterations ends up with the same cache.
    rng = np.random.default_rng(23)
    H, D, L = 2, 16, 40
    table = rng.permutation(8)[:3].astype(np.int32)
    K = W.randn_bf16((L, H, D), rng); V = W.randn_bf16((L, H, D), rng)
    one = np.zeros(W.pool_shape(8, H, B, D), dtype=np.uint16)
    oracle.kv_append(one, [L], [L], [0], table[None, :], K, V)
    step = np.zeros_like(one)
    for a in range(0, L, chunk):
        b = min(L, a + chunk)
        oracle.kv_append(step, [b], [b - a], [0], table[None, :], K[a:b], V[a:b])
    assert np.array_equal(one, step)
    assert np.array_equal(one, paged_pool_from_dense(K, V, table, B, 8, fill_bits=0))


def test_kv_append_rejects_bad_descriptors_and_shared_slots():
    batch, pool, k_new, v_new = _append_case(24)
    before = pool.copy()
    bt = batch.block_tables.copy(); bt[0, 3] = 40
    with pytest.raises(oracle.OracleError):
        oracle.kv_append(pool, batch.ctx_len, batch.q_len, batch.q_start, bt, k_new, v_new)
    bt = batch.block_tables.copy(); bt[1, 1] = bt[3, 0]; bt[1, 0] = bt[1, 0]    # seq 1 (pos 16) and seq 3 share a block
    ctx = batch.ctx_len.copy(); ctx[3] = 5; ql = batch.q_len.copy(); ql[3] = 5  # seq 3 writes slots 0..4 of it
    with pytest.raises(oracle.OracleError):
        oracle.kv_append(pool, ctx, ql, batch.q_start, bt, k_new, v_new)        # slot 0 addressed twice
    assert np.array_equal(pool, before), "a rejected call must not write"


# ---------------------------------------------------------------------------------------------
# GPU-memory-waste model (Eq. 1-5), saturation point, interception schedule
# ---------------------------------------------------------------------------------------------
def test_tfwd_is_the_profile_at_its_points_and_linear_between():
    t = oracle.TfwdTable([100, 200, 400], [0.01, 0.02, 0.05])
    for x, y in zip([100, 200, 400], [0.01, 0.02, 0.05]):
        assert oracle.tfwd(t, x) == y
    assert oracle.tfwd(t, 0) == 0.0
    assert math.isclose(oracle.tfwd(t, 50), 0.005, rel_tol=1e-15)           # ray through the origin
    assert math.isclose(oracle.tfwd(t, 150), 0.015, rel_tol=1e-15)
    assert math.isclose(oracle.tfwd(t, 300), 0.035, rel_tol=1e-15)          # second segment has another slope
    assert math.isclose(oracle.tfwd(t, 800), 0.05 + 400 * 0.03 / 200, rel_tol=1e-15)   # last slope continues
    # a profile that IS a line is reproduced everywhere (catches an off-by-one in the segment search)
    lin = oracle.TfwdTable([10, 70, 300, 1000], [0.02, 0.14, 0.6, 2.0])
    for x in [0, 3, 10, 11, 69, 70, 71, 299, 301, 999, 5000]:
        assert math.isclose(oracle.tfwd(lin, x), 0.002 * x, rel_tol=1e-14, abs_tol=1e-18)
    assert math.isnan(oracle.tfwd(oracle.TfwdTable([10, 10], [1, 2]), 5))    # not increasing
    assert math.isnan(oracle.tfwd(lin, -1))


def test_waste_equations_closed_forms():
    a, M = 2e-5, 819200.0
    lin = oracle.TfwdTable([1000.0], [a * 1000.0])                           # T_fwd(x) = a x
    C, C_other = 1500.0, 90000.0
    # Eq. 1 with linear T_fwd: a C (C + C_other) M.  Catches a dropped second term.
    assert math.isclose(oracle.waste_discard(lin, C, C_other, M), a * C * (C + C_other) * M, rel_tol=1e-14)
    # Eq. 2, Eq. 3 by hand: 3 s x 1500 tokens x M; 2 x 0.25 s x 91500 tokens x M
    assert oracle.waste_preserve(3.0, 1500.0, M) == 3.0 * 1500.0 * M
    assert oracle.waste_swap(0.25, 91500.0, M) == 2.0 * 0.25 * 91500.0 * M
    # Eq. 4: first term is HALF of Eq. 1's; with a linear T_fwd the second term equals Eq. 1's for any n
    for n in (1, 2, 3, 7):
        got = oracle.waste_chunked_discard(lin, C, C_other, M, n)
        assert math.isclose(got, a * C * C * M / 2 + a * C * C_other * M, rel_tol=1e-14), n
    # with a profile that grows faster than linearly, n T(C/n) <= T(C) (the inequality of Section 4.2)
    # so Eq. 4 < Eq. 1, strictly, and more chunks never cost more
    cvx = oracle.TfwdTable([256, 512, 1024, 2048, 4096], [0.010, 0.022, 0.050, 0.120, 0.300])
    d = oracle.waste_discard(cvx, 4096, C_other, M)
    prev = None
    for n in (1, 2, 4, 8, 16):
        w = oracle.waste_chunked_discard(cvx, 4096, C_other, M, n)
        assert w < d
        assert n * oracle.tfwd(cvx, 4096 / n) <= oracle.tfwd(cvx, 4096) * (1 + 1e-15)
        assert prev is None or w <= prev * (1 + 1e-15)
        prev = w
    # n = 1 by hand: T(C) C M / 2 + T(C) C_other M
    assert math.isclose(oracle.waste_chunked_discard(cvx, 2048, 500.0, 2.0, 1), 0.12 * 2048 * 2 / 2 + 0.12 * 500 * 2,
                        rel_tol=1e-14)
    assert math.isnan(oracle.waste_chunked_discard(cvx, 2048, 500.0, 2.0, 0))


def test_chunk_size_and_count():
    assert oracle.chunk_tokens(640, 128) == 512 and oracle.chunk_tokens(100, 128) == 0
    assert oracle.chunk_count(2048, 512) == 4 and oracle.chunk_count(2049, 512) == 5 and oracle.chunk_count(0, 512) == 0
    assert oracle.chunk_count(10, 0) == -1


def test_saturation_point_of_a_profile_with_a_known_knee():
    # iteration time max(t0, a q): throughput q / t rises up to q* = t0 / a = 500 and is flat beyond
    q = np.array([64, 128, 256, 384, 480, 512, 768, 1024, 2048], dtype=np.float64)
    t = np.maximum(1e-3, 2e-6 * q)
    assert oracle.saturation_point(q, t, 0.95) == 480                        # 480 / 500 = 0.96 of the plateau
    assert oracle.saturation_point(q, t, 1.0) == 512
    assert oracle.saturation_point(q, t, 0.5) == 256
    # a profile still rising at its end saturates at its last point
    assert oracle.saturation_point([10, 20, 40], [1.0, 1.0, 1.0], 0.95) == 40
    assert oracle.saturation_point([10, 10], [1.0, 1.0], 0.95) == -1


def test_schedule_intercepted_against_a_python_restatement():
    rng = np.random.default_rng(31)
    for _ in range(200):
        n = int(rng.integers(0, 12))
        wp = rng.integers(0, 6, size=n).astype(np.float64)                  # small integers: plenty of ties
        wc = rng.integers(0, 6, size=n).astype(np.float64)
        ctx = rng.integers(0, 50, size=n).astype(np.int64)
        budget = int(rng.integers(0, 200))
        sw, act = oracle.schedule_intercepted(wp, wc, ctx, budget)
        order = sorted(range(n), key=lambda i: (-min(wp[i], wc[i]), i))
        left, want_sw = budget, np.zeros(n, dtype=np.int64)
        for i in order:
            want_sw[i] = min(int(ctx[i]), left); left -= int(want_sw[i])
        assert np.array_equal(sw, want_sw)
        assert sw.sum() == min(budget, int(ctx.sum()))
        for i in range(n):
            rest = ctx[i] - sw[i]
            assert act[i] == (0 if rest == 0 else (1 if wp[i] <= wc[i] else 2))
    # worked example: wastes min = [5, 1, 2, 9]; budget 120 goes to request 3 (30), then request 0 (90 of 100)
    sw, act = oracle.schedule_intercepted([5, 1, 9, 9], [6, 3, 2, 20], [100, 50, 70, 30], 120)
    assert list(sw) == [90, 0, 0, 30] and list(act) == [1, 1, 2, 0]
    with pytest.raises(oracle.OracleError):
        oracle.schedule_intercepted([1.0], [float("nan")], [5], 10)


# ---------------------------------------------------------------------------------------------
# Grouped-query attention: H query heads over Hkv key/value heads
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("H,Hkv", [(8, 2), (8, 8), (6, 1), (64, 8)])
def test_gqa_equals_mha_on_replicated_kv_heads(H, Hkv):
    # Replicating every K/V head G times turns the grouped problem into the multi-head one the pins above
    # cover; outputs must agree bit for bit.  Catches h % G instead of h / G, and a pool stride of H.
    rng = np.random.default_rng(H * 100 + Hkv)
    D, nb, G = 16, 24, H // Hkv
    batch = W.assemble_batch(Hkv, D, B, nb, [37, 16, 50], [1, 16, 9], rng)
    pool = W.randn_bf16(W.pool_shape(nb, Hkv, B, D), rng)
    q = W.randn_bf16((batch.total_q_rows, H, D), rng)
    got = oracle.paged_attn(pool, batch.ctx_len, batch.q_len, batch.q_start, batch.block_tables, q, 0.3)
    wide = np.repeat(pool, G, axis=2)                                        # kv head j -> query heads jG..jG+G-1
    want = oracle.paged_attn(wide, batch.ctx_len, batch.q_len, batch.q_start, batch.block_tables, q, 0.3)
    assert got.shape == (batch.total_q_rows, H, D)
    assert np.array_equal(got, want)


def test_gqa_matches_dense_numpy_with_explicit_head_map():
    rng = np.random.default_rng(55)
    H, Hkv, D, ctx, n = 6, 2, 8, 45, 12
    K = W.randn_bf16((ctx, Hkv, D), rng); V = W.randn_bf16((ctx, Hkv, D), rng); q = W.randn_bf16((n, H, D), rng)
    table = rng.permutation(6)[:3].astype(np.int32)
    pool = paged_pool_from_dense(K, V, table, B, 6)
    out = oracle.paged_attn(pool, [ctx], [n], [0], table[None, :], q, 0.25)
    head_map = [0, 0, 0, 1, 1, 1]
    Kw, Vw = W.bf16_bits_to_f64(K)[:, head_map], W.bf16_bits_to_f64(V)[:, head_map]
    want = dense_causal_attention(W.bf16_bits_to_f64(q), Kw, Vw, 0.25, ctx - n)
    assert np.abs(out - want).max() < 1e-12


def test_gqa_rejects_heads_that_do_not_divide():
    rng = np.random.default_rng(56)
    pool = W.randn_bf16(W.pool_shape(4, 3, B, 8), rng)
    q = W.randn_bf16((1, 4, 8), rng)
    with pytest.raises(oracle.OracleError):
        oracle.paged_attn(pool, [5], [1], [0], np.zeros((1, 1), dtype=np.int32), q, 1.0)


def test_stored_oracle_values_have_not_moved():
    """tests/golden/*.txt were written by tests/golden/make_golden.py from the oracle alone (the paper prints no
    worked values for this path); an edit that changes the oracle's arithmetic must show up here."""
    import importlib.util
    import os
    here = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(here, "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    for name, fn in mod.FILES.items():
        assert open(os.path.join(here, name)).read() == fn(), name


def test_split_kv_merge_reproduces_the_unsplit_row():
    """The identity the GPU path's split-KV rests on (it is not in the paper): cut a row's keys into ranges, take
    (m, l, o~) of each, merge by log-sum-exp, and the unsplit attention row comes back to 1e-13.  Partitions of one
    key, of uneven sizes, in any order; a grouped pool (query head 5 reads K/V head 1)."""
    rng = np.random.default_rng(2024)
    H, Hkv, D, ctx = 6, 2, 64, 333
    pool_bits = W.randn_bf16((32, 2, Hkv, 16, D), rng)
    table = rng.permutation(32)[: (ctx + 15) // 16].astype(np.int32)
    q_bits = W.randn_bf16((1, H, D), rng)
    scale = 1.0 / np.sqrt(D)
    want = oracle.paged_attn(pool_bits, [ctx], [1], [0], table[None, :], q_bits, scale)   # [1][H][D], the C oracle
    for head in (0, 5):
        kvh = head // (H // Hkv)
        whole = oracle.attn_partial(pool_bits, table, q_bits[0, head], scale, 0, ctx, kvh)
        assert np.allclose(whole[2] / whole[1], want[0, head], rtol=0, atol=1e-13)
        for cuts in ([0, 64, 128, 333], [0, 1, 2, 330, 333], [0, 200, 333], sorted({0, ctx} | set(rng.integers(1, ctx, 9).tolist()))):
            parts = [oracle.attn_partial(pool_bits, table, q_bits[0, head], scale, a, b, kvh) for a, b in zip(cuts, cuts[1:])]
            for order in (parts, parts[::-1]):
                assert np.allclose(oracle.merge_partials(order), want[0, head], rtol=0, atol=1e-13)
    # a wrong merge (forgetting the e^(m_p - m) factors) is caught
    parts = [oracle.attn_partial(pool_bits, table, q_bits[0, 0], scale, a, b, 0) for a, b in ((0, 100), (100, 333))]
    wrong = sum(p[2] for p in parts) / sum(p[1] for p in parts)
    assert np.abs(wrong - want[0, 0]).max() > 1e-3
