"""CPU-only checks of the C-ABI library: exported symbols, validation and launch planning.
No compute entry point is called here (no GPU in this tier)."""
import ctypes as C
import math
import os
import re

import numpy as np
import pytest

from paper_2402_01869_amd import binding as B
from paper_2402_01869_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions(header):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b([a-z_0-9]+)\s*\([^;{]*\)\s*;", text)))


def test_library_exports_every_declared_symbol():
    """infercept_hot.h is the method's contract, infercept_measure.h holds the measurement aids; together they
    declare exactly what the library exports and the binding lists."""
    method, measure = _declared_functions("infercept_hot.h"), _declared_functions("infercept_measure.h")
    assert {"kv_pool_init", "paged_attn_mixed", "kv_pack_blocks", "kv_unpack_blocks"} <= set(method)
    assert set(measure) == {"ic_prof_begin", "ic_prof_end", "ic_mfma_ceiling", "ic_hbm_ceiling", "ic_paged_read_ceiling"}
    assert not set(method) & set(measure)
    assert not [n for n in method if "ceiling" in n or "prof" in n]
    raw = C.CDLL(B.LIB_PATH)
    for n in method + measure:
        assert hasattr(raw, n), f"{n} declared in a header but not exported"
    assert set(method + measure) == set(B.EXPORTS), "binding.EXPORTS out of sync with the headers"


def test_strerror_covers_codes():
    seen = {B.strerror(c) for c in range(0, -12, -1)}
    assert len(seen) == 12 and "unknown error code" not in seen
    assert B.strerror(-99) == "unknown error code"


def _pool(cfg=None, ptr=0x10000, nbytes=None):
    cfg = cfg or B.make_cfg(64, 4, 64)
    bb = cfg.block_size * 2 * cfg.num_kv_heads * cfg.head_dim * 2
    return B.KvPool(cfg, ptr, cfg.num_blocks * bb if nbytes is None else nbytes)


def test_pool_init_validation():
    # kv_pool_init touches no GPU state, so a made-up (aligned) address is enough on the CPU
    p = _pool()
    assert p.block_bytes == 16 * 2 * 4 * 64 * 2
    p.close()
    for kw, code in [(dict(cfg=B.make_cfg(64, 4, 96)), B.IC_EUNSUPPORTED),
                     (dict(cfg=B.make_cfg(64, 4, 64, block_size=32)), B.IC_EUNSUPPORTED),
                     (dict(cfg=B.make_cfg(64, 8, 64, num_kv_heads=3)), B.IC_EINVAL),      # heads must divide
                     (dict(cfg=B.make_cfg(64, 4, 64, num_kv_heads=8)), B.IC_EINVAL),
                     (dict(cfg=B.make_cfg(64, 4, 64, dtype=1)), B.IC_EUNSUPPORTED),
                     (dict(cfg=B.make_cfg(0, 4, 64)), B.IC_EINVAL),
                     (dict(ptr=0x10008), B.IC_EALIGN),
                     (dict(ptr=0), B.IC_ENULL),
                     (dict(nbytes=63 * 16384), B.IC_ESIZE)]:
        with pytest.raises(B.InferceptError) as e:
            _pool(**kw)
        assert e.value.code == code, kw


def test_check_batch_codes():
    cfg = B.make_cfg(64, 4, 64)
    b = W.make_batch(W.TINY)
    ok = B.HostDesc.from_batch(b)
    assert B.check_batch(cfg, ok) == B.IC_OK

    def desc(**kw):
        a = dict(ctx_len=b.ctx_len.copy(), q_len=b.q_len.copy(), q_start=b.q_start.copy(),
                 block_tables=b.block_tables.copy(), scale=b.scale, total_q_rows=b.total_q_rows)
        a.update(kw)
        return B.HostDesc(**a)

    bt = b.block_tables.copy(); bt[2, 1] = 64
    assert B.check_batch(cfg, desc(block_tables=bt)) == B.IC_ERANGE
    bt = b.block_tables.copy(); bt[0, 0] = -1
    assert B.check_batch(cfg, desc(block_tables=bt)) == B.IC_ERANGE
    # entries past ceil(ctx/16) are ignored, whatever they hold
    bt = b.block_tables.copy(); bt[0, -1] = 10 ** 6 if b.ctx_len[0] <= 16 * (bt.shape[1] - 1) else bt[0, -1]
    assert B.check_batch(cfg, desc(block_tables=bt)) == B.IC_OK
    c = b.ctx_len.copy(); c[1] = 0
    assert B.check_batch(cfg, desc(ctx_len=c)) == B.IC_EINVAL
    q = b.q_len.copy(); q[0] = 0
    assert B.check_batch(cfg, desc(q_len=q)) == B.IC_EINVAL
    q = b.q_len.copy(); q[1] = b.ctx_len[1] + 1
    assert B.check_batch(cfg, desc(q_len=q, total_q_rows=10 ** 4)) == B.IC_EINVAL
    qs = b.q_start.copy(); qs[3] = qs[2] + 1
    assert B.check_batch(cfg, desc(q_start=qs)) == B.IC_EOVERLAP
    qs = b.q_start.copy(); qs[3] = b.total_q_rows - 1
    assert B.check_batch(cfg, desc(q_start=qs)) == B.IC_EOVERLAP
    assert B.check_batch(cfg, desc(block_tables=b.block_tables[:, :2])) == B.IC_ESIZE
    assert B.check_batch(cfg, desc(scale=float("nan"))) == B.IC_EINVAL
    assert B.check_batch(cfg, desc(scale=-1.0)) == B.IC_EINVAL
    assert B.check_batch(cfg, desc(scale=0.0)) == B.IC_EINVAL      # the kernels need a positive factor
    assert B.check_batch(cfg, desc(scale=float("inf"))) == B.IC_EINVAL
    # rows may leave gaps in the packed array
    assert B.check_batch(cfg, desc(total_q_rows=b.total_q_rows + 5)) == B.IC_OK


def test_check_ids_codes():
    cfg = B.make_cfg(100, 4, 64)
    assert B.check_ids(cfg, [1, 5, 5], False) == B.IC_OK
    assert B.check_ids(cfg, [1, 5, 5], True) == B.IC_EDUP
    assert B.check_ids(cfg, [0, 99], True) == B.IC_OK
    assert B.check_ids(cfg, [100], False) == B.IC_ERANGE
    assert B.check_ids(cfg, [-1], False) == B.IC_ERANGE
    assert B.check_ids(cfg, [], True) == B.IC_OK


def test_plan_counts_and_workspace():
    p = _pool()
    b = W.make_batch(W.TINY)
    d = B.HostDesc.from_batch(b)
    base = p.plan_query(d)
    assert base["decode_rows"] == 2 and base["span_rows"] == int(b.q_len[2:].sum())
    # rows of a span that see fewer than 64 keys are vector row items; the rest of the span is one tile
    few = [min(int(n), max(0, 63 - int(c - n))) for c, n in zip(b.ctx_len[2:], b.q_len[2:])]
    assert base["row_items"] == 2 + sum(few) and base["partial_slots"] == 0 and base["merge_rows"] == 0
    assert base["tile_items"] == sum(1 for f, n in zip(few, b.q_len[2:]) if f < n)
    p.set_tuning(mfma_min_keys=1)             # no such routing: every span row on the matrix cores
    alltile = p.plan_query(d)
    assert alltile["row_items"] == 2 and alltile["tile_items"] == 2   # one tile per 32-row span
    p.set_tuning()
    assert base["table_entries"] == int(sum(-(-int(c) // 16) for c in b.ctx_len))
    w0 = p.workspace_bytes(d)
    assert w0 > 0 and w0 % 256 == 0
    # forcing 64-key partitions splits every context longer than 64 keys
    p.set_tuning(64, 64, 0)
    split = p.plan_query(d)
    want_row_items = sum(-(-int(c) // 64) for c in b.ctx_len[:2]) + sum(few)
    assert split["row_items"] == want_row_items
    assert split["partial_slots"] > 0 and split["merge_rows"] > 0
    assert p.workspace_bytes(d) > w0
    # spans row by row: one work item per (row, partition)
    p.set_tuning(0, 0, 1)
    rows = p.plan_query(d)
    assert rows["tile_items"] == 0 and rows["row_items"] == b.total_q_rows
    with pytest.raises(B.InferceptError):
        p.set_tuning(-1, 0, 0)
    with pytest.raises(B.InferceptError):
        p.set_tuning(0, 0, 3)
    with pytest.raises(B.InferceptError):
        p.set_tuning(mfma_min_keys=65)
    bad = B.HostDesc(b.ctx_len, b.q_len + 1000, b.q_start, b.block_tables, b.scale)
    assert p.workspace_bytes(bad) == 0
    p.close()


def test_full_size_plans_are_sane():
    """Plans of the benchmark configurations: every key of every row is covered exactly once."""
    for cfg in (W.GPTJ_DECODE, W.MIXED_13B, W.LONG_CTX):
        b = W.make_batch(cfg)
        p = _pool(B.make_cfg(cfg.pool_blocks, cfg.num_heads, cfg.head_dim))
        d = B.HostDesc.from_batch(b, flags=B.IC_FLAG_TRUSTED)
        info = p.plan_query(d)
        assert info["decode_rows"] == cfg.n_decode and info["span_rows"] == cfg.n_span * cfg.span_len
        assert info["table_entries"] == int(sum(-(-int(c) // 16) for c in b.ctx_len))
        part = 4096
        assert info["row_items"] == int(sum(-(-int(c) // part) for c in b.ctx_len[:cfg.n_decode]))
        assert info["tile_items"] >= cfg.n_span * (cfg.span_len // 256)
        assert 0 < p.workspace_bytes(d) < (4 << 30)
        p.close()


# ---------------------------------------------------------------------------------------------
# Layer-pipelined swap: host-side validation and the swap-limit arithmetic (no GPU touched)
# ---------------------------------------------------------------------------------------------
def _swapper(L=3, max_blocks=8, stages=2, staging_ptr=0x4000000, staging_bytes=None, pools=None):
    pools = pools or [_pool(ptr=0x100000 * (l + 1)) for l in range(L)]
    bb = pools[0].block_bytes
    nbytes = stages * max_blocks * bb if staging_bytes is None else staging_bytes
    return B.LayerSwapper(pools, max_blocks, staging_ptr, nbytes, stages), pools


def test_swapper_create_validation():
    sw, pools = _swapper()
    assert B.LayerSwapper.staging_bytes(pools[0], 3, 8, 2) == 2 * 8 * pools[0].block_bytes
    sw.close()
    bad = [(dict(stages=1), B.IC_EINVAL), (dict(stages=9), B.IC_EINVAL), (dict(max_blocks=0), B.IC_EINVAL),
           (dict(max_blocks=65), B.IC_EINVAL),                       # more than the pool holds
           (dict(staging_ptr=0x4000008), B.IC_EALIGN), (dict(staging_ptr=0), B.IC_ENULL),
           (dict(staging_bytes=2 * 8 * 16384 - 1), B.IC_ESIZE),
           (dict(staging_ptr=0x100000 + 4096), B.IC_EINVAL),         # staging inside layer 0's pool
           (dict(pools=[_pool(ptr=0x100000), _pool(cfg=B.make_cfg(64, 4, 128), ptr=0x900000)]), B.IC_EINVAL)]
    for kw, code in bad:
        with pytest.raises(B.InferceptError) as e:
            _swapper(**kw)
        assert e.value.code == code, kw


def test_swapper_call_validation_happens_before_any_gpu_work():
    sw, pools = _swapper()
    host, stride = 0x7000000, 8 * pools[0].block_bytes
    for fn in (sw.swap_out, sw.swap_in):
        assert fn([], host, stride, check=False) == B.IC_OK                     # n = 0: nothing to do
        assert fn(list(range(9)), host, stride, check=False) == B.IC_EINVAL     # more than max_blocks
        assert fn([1, 64], host, stride, check=False) == B.IC_ERANGE
        assert fn([1, -1], host, stride, check=False) == B.IC_ERANGE
        assert fn([1, 2], 0, stride, check=False) == B.IC_ENULL
        assert fn([1, 2, 3], host, 2 * pools[0].block_bytes, check=False) == B.IC_ESIZE
        assert fn([1, 2], host + 4, stride, check=False) == B.IC_EALIGN
    assert sw.swap_in([5, 5], host, stride, check=False) == B.IC_EDUP            # order-dependent result
    assert sw.wait_layer(B.IC_SWAP_IN, 2) == B.IC_OK                             # nothing queued: no-op
    with pytest.raises(B.InferceptError):
        sw.wait_layer(B.IC_SWAP_IN, 3)
    with pytest.raises(B.InferceptError):
        sw.sync_layer(2, 0)
    sw.sync()
    sw.close()


def test_swap_limit_and_schedule_match_the_oracle():
    import oracle
    rng = np.random.default_rng(11)
    for _ in range(500):
        t = float(rng.uniform(0, 0.3)); bw = float(rng.uniform(1e9, 2e11)); m = float(rng.integers(512, 8 << 20))
        assert B.swap_limit_tokens(t, bw, m) == oracle.swap_limit_tokens(t, bw, m)
    for args in [(0.0, 1e9, 1024.0), (0.5, 2.0 ** 30, 2.0 ** 20), (-1.0, 1e9, 1.0), (1.0, 0.0, 1.0), (1.0, 1.0, 0.0),
                 (float("nan"), 1e9, 1.0), (1e30, 1e30, 1e-30)]:
        assert B.swap_limit_tokens(*args) == oracle.swap_limit_tokens(*args), args
    for _ in range(200):
        total = int(rng.integers(0, 300)); bs = int(rng.choice([1, 16, 32]))
        limits = rng.integers(0, 50 * bs, size=int(rng.integers(0, 25))).astype(np.int64)
        got, want = B.swap_schedule(total, bs, limits), oracle.swap_schedule(total, bs, limits)
        assert got[0] == want[0] and np.array_equal(got[1], want[1])
    assert B.swap_schedule(5, 16, [32, -1])[0] == oracle.swap_schedule(5, 16, [32, -1])[0] == -1
    assert B.swap_schedule(-1, 16, [32])[0] == -1 and B.swap_schedule(1, 0, [32])[0] == -1


def test_kv_write_span_validation_happens_before_any_gpu_work():
    p = _pool()
    b = W.make_batch(W.TINY)
    ok = B.HostDesc.from_batch(b)
    k = v = 0x9000000
    assert p.kv_write_span(ok, 0, v, check=False) == B.IC_ENULL
    assert p.kv_write_span(ok, k, v + 8, check=False) == B.IC_EALIGN
    bt = b.block_tables.copy(); bt[2, 0] = 64
    bad = B.HostDesc(b.ctx_len, b.q_len, b.q_start, bt, b.scale, b.total_q_rows)
    assert p.kv_write_span(bad, k, v, check=False) == B.IC_ERANGE
    # two sequences whose new tokens land on one slot: the result would depend on the write order
    s0, s1 = [s for s in range(b.num_seqs) if b.q_len[s] == 1][:2]
    ctx = b.ctx_len.copy(); ctx[s1] = ctx[s0]
    bt = b.block_tables.copy(); bt[s1] = bt[s0]
    dup = B.HostDesc(ctx, b.q_len, b.q_start, bt, b.scale, b.total_q_rows)
    assert p.kv_write_span(dup, k, v, check=False) == B.IC_EDUP
    p.close()


# ---------------------------------------------------------------------------------------------
# Waste model, chunk sizing, saturation point and interception schedule against the oracle
# ---------------------------------------------------------------------------------------------
def _close(a, b):
    """Library and oracle evaluate the same fp64 expressions in the same order: the doubles must be identical."""
    if math.isnan(a) or math.isnan(b):
        return math.isnan(a) and math.isnan(b)
    return a == b


def test_waste_model_matches_the_oracle():
    import oracle
    rng = np.random.default_rng(41)
    for _ in range(300):
        n = int(rng.integers(1, 8))
        tok = np.cumsum(rng.integers(1, 2000, size=n)).astype(np.float64)
        sec = np.cumsum(rng.uniform(1e-4, 5e-2, size=n))
        tb, to = B.TfwdTable(tok, sec), oracle.TfwdTable(tok, sec)
        xs = list(rng.uniform(0, tok[-1] * 2, size=6)) + list(tok) + [0.0]
        for x in xs:
            assert _close(tb(x), oracle.tfwd(to, x)), (tok, sec, x)
        Cc, Co, M = float(rng.integers(1, 8000)), float(rng.integers(0, 200000)), float(rng.integers(1024, 1 << 21))
        assert _close(B.waste_discard(tb, Cc, Co, M), oracle.waste_discard(to, Cc, Co, M))
        for k in (1, 2, 5, 16):
            assert _close(B.waste_chunked_discard(tb, Cc, Co, M, k), oracle.waste_chunked_discard(to, Cc, Co, M, k))
        ti = float(rng.uniform(0, 30))
        assert B.waste_preserve(ti, Cc, M) == oracle.waste_preserve(ti, Cc, M)
        assert B.waste_swap(ti, Cc + Co, M) == oracle.waste_swap(ti, Cc + Co, M)
    bad_b, bad_o = B.TfwdTable([5, 5], [1, 2]), oracle.TfwdTable([5, 5], [1, 2])
    assert math.isnan(bad_b(1.0)) and math.isnan(oracle.tfwd(bad_o, 1.0))
    assert math.isnan(B.waste_chunked_discard(B.TfwdTable([5], [1]), 10, 10, 1, 0))
    assert math.isnan(B.TfwdTable([5], [1])(-1.0))
    for S, r in [(640, 128), (100, 128), (0, 0), (512, 512)]:
        assert B.chunk_tokens(S, r) == oracle.chunk_tokens(S, r)
    for Cc, ch in [(2048, 512), (2049, 512), (0, 512), (1, 1), (10, 0), (-1, 5)]:
        assert B.chunk_count(Cc, ch) == oracle.chunk_count(Cc, ch)


def test_saturation_point_and_schedule_match_the_oracle():
    import oracle
    rng = np.random.default_rng(42)
    for _ in range(200):
        n = int(rng.integers(1, 12))
        q = np.cumsum(rng.integers(1, 600, size=n)).astype(np.float64)
        t = np.maximum(rng.uniform(5e-4, 2e-3), rng.uniform(1e-6, 4e-6) * q) * rng.uniform(0.97, 1.03, size=n)
        for frac in (0.5, 0.9, 0.95, 1.0):
            assert B.saturation_point(q, t, frac) == oracle.saturation_point(q, t, frac)
    assert B.saturation_point([10, 10], [1, 1]) == oracle.saturation_point([10, 10], [1, 1]) == -1
    assert B.saturation_point([10, 20], [1, 1], 1.5) == -1
    for _ in range(300):
        n = int(rng.integers(0, 14))
        wp = rng.integers(0, 5, size=n).astype(np.float64) * rng.choice([1.0, 0.5])
        wc = rng.integers(0, 5, size=n).astype(np.float64)
        ctx = rng.integers(0, 80, size=n).astype(np.int64)
        budget = int(rng.integers(0, 300))
        rc, sw, act = B.schedule_intercepted(wp, wc, ctx, budget)
        osw, oact = oracle.schedule_intercepted(wp, wc, ctx, budget)
        assert rc == B.IC_OK and np.array_equal(sw, osw) and np.array_equal(act, oact)
    assert B.schedule_intercepted([1.0], [float("nan")], [5], 10)[0] == B.IC_EINVAL
    assert B.schedule_intercepted([1.0], [1.0], [-5], 10)[0] == B.IC_EINVAL
    assert B.schedule_intercepted([1.0], [1.0], [5], -1)[0] == B.IC_EINVAL


def test_kernel_register_budgets():
    """The side-by-side launch of the mixed batch needs, per SIMD, two waves of the persistent tile kernel
    and one of the slim row kernel resident together: 2 x 216 + 80 = 512 registers per lane; in a grouped pool
    the slim group kernel takes the row kernel's place with 96, so the tile kernel may use 208 there; head_dim 256
    pairs a 208-register tile kernel of 16-row waves with a 96-register row kernel.  Read the compiler's resource
    report for these kernels and for spills in the MFMA kernels."""
    import shutil
    import subprocess
    import tempfile
    if not shutil.which("hipcc"):
        pytest.skip("hipcc not on PATH")
    csrc = os.path.join(ROOT, "paper_2402_01869_amd", "csrc")
    usage = {}
    with tempfile.TemporaryDirectory() as tmp:
        for src in ("attn_tile.hip", "attn_row.hip", "attn_group_slim.hip"):
            r = subprocess.run(["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature",
                                "-Xclang", "-packed-fp32-ops", "-Rpass-analysis=kernel-resource-usage", "-c",
                                os.path.join(csrc, src), "-o", os.path.join(tmp, src + ".o")],
                               capture_output=True, text=True)
            assert r.returncode == 0, r.stderr[-2000:]
            name = None
            for line in r.stderr.splitlines():
                m = re.search(r"Function Name: (\S+)", line)
                if m:
                    name = m.group(1); usage[name] = {}
                m = re.search(r"\s(VGPRs|VGPRs Spill|ScratchSize \[bytes/lane\]): (\d+)", line)
                if m and name:
                    usage[name][m.group(1)] = int(m.group(2))
    def find(kernel, dim):
        hits = [u for n, u in usage.items() if kernel in n and f"ILi{dim}E" in n]
        assert len(hits) >= 1, (kernel, dim, list(usage))   # builds that differ in name only: the worst of them
        return {k: max(h[k] for h in hits) for k in hits[0]}
    for dim in (64, 128):
        assert find("tile_persist_kernel", dim)["VGPRs"] <= 216
        assert find("row_persist_slim_kernel", dim)["VGPRs"] <= 80
    # head_dim 256: 16-row waves, 2 x 208 + 96
    assert find("tile_persist_kernel", 256)["VGPRs"] <= 208 and find("row_persist_slim_kernel", 256)["VGPRs"] <= 96
    slim = [u for n, u in usage.items() if "group_slim_kernel" in n]
    assert len(slim) == 1 and slim[0]["VGPRs"] <= 96 and 2 * find("tile_persist_kernel", 128)["VGPRs"] + 96 <= 512
    for dim in (64, 128, 256):
        assert find("tile_attn_kernel", dim)["VGPRs Spill"] == 0
    for dim in (64, 128):
        assert find("tile_persist_kernel", dim)["VGPRs Spill"] == 0


def test_mfma_ceiling_rejects_bad_arguments_before_any_launch():
    """Validation happens on the host: these calls return before touching the GPU (none is present here)."""
    ok_ops, ok_sink = 0x1000, 0x2000   # never dereferenced: every call below fails validation first
    assert B.mfma_ceiling(0, B.IC_CEILING_OPERAND_BYTES, ok_sink, B.IC_CEILING_SINK_BYTES, 10)[0] == B.IC_ENULL
    assert B.mfma_ceiling(ok_ops, B.IC_CEILING_OPERAND_BYTES, 0, B.IC_CEILING_SINK_BYTES, 10)[0] == B.IC_ENULL
    assert B.mfma_ceiling(ok_ops, B.IC_CEILING_OPERAND_BYTES, ok_sink, B.IC_CEILING_SINK_BYTES, 0)[0] == B.IC_EINVAL
    assert B.mfma_ceiling(ok_ops, B.IC_CEILING_OPERAND_BYTES - 1, ok_sink, B.IC_CEILING_SINK_BYTES, 10)[0] == B.IC_ESIZE
    assert B.mfma_ceiling(ok_ops, B.IC_CEILING_OPERAND_BYTES, ok_sink, B.IC_CEILING_SINK_BYTES - 1, 10)[0] == B.IC_ESIZE
    assert B.mfma_ceiling(ok_ops + 8, B.IC_CEILING_OPERAND_BYTES, ok_sink, B.IC_CEILING_SINK_BYTES, 10)[0] == B.IC_EALIGN


def _check_plan_covers_every_row_once(pool, batch, desc, min_keys=64):
    """Every (query row, visible key) pair is handled by exactly one work item; partial slots are distinct and every
    split row has a merge item naming them; tables, row destinations and alignment are as the kernels assume."""
    P = pool.plan_image(desc)
    assert not P["counters"].any()
    # compact block tables
    off = 0
    for s in range(batch.num_seqs):
        nb = (int(batch.ctx_len[s]) + 15) // 16
        assert P["bt_off"][s] == off
        assert np.array_equal(P["bt_flat"][off:off + nb], batch.block_tables[s, :nb])
        off += nb
    rows = int(desc.struct.total_q_rows)
    klen = np.zeros(rows, dtype=np.int64)          # keys visible to each query row; 0 = nobody's row
    want_dst = np.full(rows, -1, dtype=np.int64)
    for s in range(batch.num_seqs):
        c, n, r0 = int(batch.ctx_len[s]), int(batch.q_len[s]), int(batch.q_start[s])
        for i in range(n):
            t = c - n + i
            klen[r0 + i] = t + 1
            want_dst[r0 + i] = int(batch.block_tables[s, t // 16]) * 16 + t % 16
    assert np.array_equal(P["row_dst"], want_dst)
    ranges = [[] for _ in range(rows)]             # per row: (k_begin, k_end_visible, slot)
    n_vec = P["n_vector_row_items"]
    assert 0 <= n_vec <= P["n_row_items"]
    if batch.kv_heads == batch.num_heads:
        assert n_vec == P["n_row_items"]           # only grouped pools have a group kernel
    for idx, (seq, qrow, kb, ke, slot, p0, p1, p2) in enumerate(P["row_items"].tolist()):
        assert kb % 16 == 0 and 0 <= kb < ke <= klen[qrow] and ke - kb <= P["row_part_tokens"] and p0 == p1 == p2 == 0
        assert batch.q_start[seq] <= qrow < batch.q_start[seq] + batch.q_len[seq]
        if idx >= n_vec:                           # matrix-core decode rows: never a row of a handful of keys
            assert klen[qrow] >= min_keys and batch.q_len[seq] == 1
        ranges[qrow].append((kb, ke, slot))
    for seq, qrow0, n_rows, pos0, kb, ke, slot0, nparts in P["tile_items"].tolist():
        assert kb % 64 == 0 and 1 <= n_rows <= P["tile_query_rows"] and nparts >= 1
        assert pos0 + 1 >= min_keys                # the tile's first row already sees min_keys keys
        assert pos0 == int(batch.ctx_len[seq] - batch.q_len[seq]) + (qrow0 - int(batch.q_start[seq]))
        part = P["row_part_tokens"] if batch.q_len[seq] == 1 else P["span_part_tokens"]   # decode rows as one-row tiles
        assert kb < ke <= pos0 + n_rows and ke - kb <= part
        for r in range(n_rows):
            vis_end = min(ke, pos0 + r + 1)
            # a row whose position lies before this partition has nothing to do in it, but still owns a slot there
            ranges[qrow0 + r].append((kb, max(vis_end, kb), -1 if slot0 < 0 else slot0 + r * nparts))
    merges = {int(q): (int(s0), int(np_)) for q, s0, np_, pad in P["merge_items"].tolist()}
    assert len(merges) == P["n_merge_items"]
    seen_slots = set()
    for r in range(rows):
        if klen[r] == 0:
            assert not ranges[r]
            continue
        parts = sorted(ranges[r])
        assert parts[0][0] == 0
        end = 0
        for kb, ke, slot in parts:
            if ke == kb:
                assert kb >= klen[r], (r, parts)   # an empty partition lies wholly beyond the row's position
                continue
            assert kb == end, (r, parts)           # contiguous, no overlap
            end = ke
        assert end == klen[r], (r, parts, klen[r])
        if len(parts) == 1:
            assert parts[0][2] == -1 and r not in merges
        else:
            slots = sorted(p[2] for p in parts)
            s0, np_ = merges[r]
            assert slots == list(range(s0, s0 + np_)), (r, slots, merges[r])
            assert not (seen_slots & set(slots))
            seen_slots |= set(slots)
    assert seen_slots == set(range(P["partial_slots"]))


@pytest.mark.parametrize("H,Hkv,D", [(4, 4, 64), (5, 5, 128), (2, 2, 256), (8, 2, 128), (64, 8, 128), (6, 2, 64)])
def test_launch_plan_covers_every_row_and_key_exactly_once(H, Hkv, D):
    """ic_plan_image on random batches and tunings (host only): decode rows and spans, split and unsplit, spans as
    rows or tiles, grouped pools with decode rows as group items or one-row tiles, gaps in the row space."""
    rng = np.random.default_rng(1000 * H + 10 * Hkv + D)
    for trial in range(6):
        n_seq = int(rng.integers(1, 9))
        ctx = rng.integers(1, 1500, size=n_seq).tolist()
        qlen = [1 if rng.random() < 0.5 else int(rng.integers(1, c + 1)) for c in ctx]
        if trial == 0:
            ctx, qlen = [700, 5000, 64, 1], [300, 1, 64, 1]
        batch = W.assemble_batch(H, D, 16, 2048, ctx, qlen, rng, num_kv_heads=Hkv)
        total = batch.total_q_rows
        if trial % 2:   # leave rows nobody owns between the sequences
            batch.q_start = (batch.q_start + 3 * np.arange(batch.num_seqs)).astype(np.int32)
            total += 3 * batch.num_seqs + 5
        cfg = B.make_cfg(2048, H, D, num_kv_heads=Hkv)
        pool = B.KvPool(cfg, 0x10000, 2048 * 16 * 2 * Hkv * D * 2)   # the base address is never dereferenced here
        desc = B.HostDesc(batch.ctx_len, batch.q_len, batch.q_start, batch.block_tables, batch.scale, total)
        for tn in (dict(), dict(decode_part_tokens=64, span_part_tokens=64), dict(span_kernel=1, decode_part_tokens=128),
                   dict(span_kernel=2, decode_part_tokens=256, span_part_tokens=128), dict(span_part_tokens=1 << 20),
                   dict(mfma_min_keys=1), dict(mfma_min_keys=17, span_kernel=2, decode_part_tokens=64)):
            pool.set_tuning(**tn)
            _check_plan_covers_every_row_once(pool, batch, desc, tn.get("mfma_min_keys", 64))
        pool.close()


def test_hbm_ceiling_rejects_bad_arguments_before_any_launch():
    a, b = 0x100000, 0x900000   # never dereferenced: every call below fails validation first
    assert B.hbm_ceiling(0, b, 1 << 20, 0, 1)[0] == B.IC_ENULL
    assert B.hbm_ceiling(a, 0, 1 << 20, 1, 1)[0] == B.IC_ENULL
    assert B.hbm_ceiling(a, b, 1024, 0, 1)[0] == B.IC_EINVAL          # not a multiple of 8 KiB
    assert B.hbm_ceiling(a, b, 1 << 20, 2, 1)[0] == B.IC_EINVAL         # unknown mode
    assert B.hbm_ceiling(a, b, 1 << 20, 1, 0)[0] == B.IC_EINVAL         # no repetitions
    assert B.hbm_ceiling(a + 4, b, 1 << 20, 1, 1)[0] == B.IC_EALIGN
    assert B.hbm_ceiling(a, a + (1 << 19), 1 << 20, 1, 1)[0] == B.IC_EINVAL   # overlapping copy


def test_paged_read_ceiling_rejects_bad_arguments_before_any_launch():
    pool = B.KvPool(B.make_cfg(64, 4, 64), 0x10000, 64 * 16 * 2 * 4 * 64 * 2)   # base never dereferenced
    assert pool.paged_read_ceiling([0, 1], 0, 1, check=False)[0] == B.IC_ENULL
    assert pool.paged_read_ceiling([0, 64], 0x2000, 1, check=False)[0] == B.IC_ERANGE
    assert pool.paged_read_ceiling([0, 1], 0x2000, 0, check=False)[0] == B.IC_EINVAL
    assert pool.paged_read_ceiling([0, 1], 0x2008, 1, check=False)[0] == B.IC_EALIGN
    pool.close()
