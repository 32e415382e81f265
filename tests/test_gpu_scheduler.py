"""The scheduler's arithmetic on a MEASURED T_fwd profile: the attention call is timed through the C ABI for a decode
batch plus a growing number of recomputation chunks (Section 4.2), and the profile is fed to the library's saturation
point, chunk sizing, waste model (Eq. 1, 4, 5) and interception schedule (Section 4.3) and to the oracle's: integers
must be identical and doubles bit-identical."""
import time

import numpy as np
import pytest
import torch

import oracle
from paper_2402_01869_amd import binding as B
from paper_2402_01869_amd import workloads as W
from gpu_common import DEV, to_dev_bits

pytestmark = pytest.mark.gpu


def _bits(x: float) -> int:
    return int(np.float64(x).view(np.uint64))


def test_measured_profile_through_saturation_point_chunks_waste_and_schedule():
    H, D, blocks = 40, 128, 16384                                    # 13B-shaped layer, 5 GiB pool
    rng = np.random.default_rng(20240201)
    pool_t = torch.empty(W.pool_shape(blocks, H, 16, D), dtype=torch.bfloat16, device=DEV)
    W.fill_pool_device_normal(pool_t, 7)
    pool = B.KvPool.from_tensor(pool_t, H, D)
    dec_ctx = rng.integers(256, 2049, size=32).tolist()
    stream = torch.cuda.current_stream().cuda_stream
    q_tokens, seconds = [], []
    for n_span in (0, 1, 2, 4, 8, 16):
        ctx = dec_ctx + rng.integers(1024, 2049, size=n_span).tolist()
        qlen = [1] * 32 + [256] * n_span
        batch = W.assemble_batch(H, D, 16, blocks, ctx, qlen, np.random.default_rng(n_span))
        desc = B.HostDesc.from_batch(batch)
        q = to_dev_bits(W.randn_bf16((batch.total_q_rows, H, D), rng))
        out = torch.empty_like(q)
        ws = torch.empty(pool.workspace_bytes(desc), dtype=torch.uint8, device=DEV)
        for timed in (False, True):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(20):
                pool.paged_attn_mixed(desc, q.data_ptr(), out.data_ptr(), ws.data_ptr(), ws.numel(), stream)
            torch.cuda.synchronize()
        q_tokens.append(float(batch.total_q_rows))
        seconds.append((time.perf_counter() - t0) / 20)
        print(f"profile point: {n_span} chunks, {batch.total_q_rows} query tokens, {seconds[-1] * 1e3:.4f} ms", flush=True)
    pool.close()
    assert all(s > 0 for s in seconds)

    # saturation point and chunk sizing (Section 4.2)
    for frac in (0.5, 0.8, 0.95, 1.0):
        assert B.saturation_point(q_tokens, seconds, frac) == oracle.saturation_point(q_tokens, seconds, frac)
    S = B.saturation_point(q_tokens, seconds, 0.95)
    assert S in [int(x) for x in q_tokens]
    running = 32
    chunk = B.chunk_tokens(S, running)
    assert chunk == oracle.chunk_tokens(S, running) == max(0, S - running)
    # T_fwd for the waste model: time ADDED to the iteration against recomputed tokens (made strictly usable:
    # timing noise can make a point dip below its predecessor, which the piecewise-linear model accepts)
    tok = [t - q_tokens[0] for t in q_tokens[1:]]
    sec = [max(s - seconds[0], 0.0) for s in seconds[1:]]
    tb, to = B.TfwdTable(tok, sec), oracle.TfwdTable(tok, sec)
    M = float(2 * H * D * 2)
    C_other = float(sum(dec_ctx))
    wp, wc, ctxs = [], [], []
    for C in (300.0, 753.0, 1422.0, 2185.0, 5000.0):               # Table 1's range of context lengths and beyond
        for x in (C, C / 3.0, 0.0, 1.0):
            assert _bits(tb(x)) == _bits(oracle.tfwd(to, x)), (C, x)
        n_chunks = B.chunk_count(int(C), max(chunk, 1))
        assert n_chunks == oracle.chunk_count(int(C), max(chunk, 1)) >= 1
        a, b = B.waste_discard(tb, C, C_other, M), oracle.waste_discard(to, C, C_other, M)
        assert _bits(a) == _bits(b), (C, a, b)
        for k in {1, n_chunks, 7}:
            a, b = B.waste_chunked_discard(tb, C, C_other, M, k), oracle.waste_chunked_discard(to, C, C_other, M, k)
            assert _bits(a) == _bits(b), (C, k, a, b)
        t_int = 0.05 * C / 300.0                                    # an interception that lasts longer for longer contexts
        assert _bits(B.waste_preserve(t_int, C, M)) == _bits(oracle.waste_preserve(t_int, C, M))
        wp.append(B.waste_preserve(t_int, C, M))
        wc.append(B.waste_chunked_discard(tb, C, C_other, M, n_chunks))
        ctxs.append(int(C))
    # interception schedule (Section 4.3, Eq. 5) on those wastes, for budgets that cover none, some and all requests
    for budget in (0, 500, 2000, 4000, 20000):
        rc, sw, act = B.schedule_intercepted(wp, wc, ctxs, budget)
        osw, oact = oracle.schedule_intercepted(wp, wc, ctxs, budget)
        assert rc == B.IC_OK and np.array_equal(sw, osw) and np.array_equal(act, oact), budget
        assert int(sw.sum()) == min(budget, sum(ctxs))
    # swap limit of Section 4.1 with the measured iteration time
    for bw in (25e9, 55e9):
        assert B.swap_limit_tokens(seconds[0], bw, M) == oracle.swap_limit_tokens(seconds[0], bw, M)
