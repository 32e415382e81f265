"""ctypes front-end of the plain-C fp64 oracle: TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this
package; the product path (paper_2402_01869_amd) never does and shares no code with it.

paged_attn / paged_attn_items : textbook causal scaled-dot-product attention read through
    block tables (paper Sections 3.1, 4.2 and 4.3), fp64, bf16 bit patterns in.
pack_blocks / unpack_blocks   : the swap gather / scatter of Section 3.2 as memcpy loops.
kv_append                     : a chunk's own keys / values written into the paged cache (Sections 4.2, 4.3).
tfwd / waste_* / chunk_* / saturation_point / schedule_intercepted : the GPU-memory-waste model
    (Eq. 1-5), the saturation point and the interception schedule (Sections 3.2, 4.2, 4.3).
swap_out_layers / swap_in_layers / swap_limit_tokens / swap_schedule : what the layer-by-layer,
    chunked swap of Section 4.1 leaves behind, its swap limit N_i and the split over iterations.
attn_partial / merge_partials : the split-KV identity the GPU path relies on (not in the paper): a row's keys cut
    into ranges, each giving (m, l, o~), merged by log-sum-exp; written out in numpy to pin the FORMULA.
Every function is pinned by tests/test_oracle_pins.py; none is "parity unpinned".
"""
from __future__ import annotations

import ctypes as C
from typing import Optional

import numpy as np

from .build import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(_build())
        i32p, u16p, u8p, f64p = (C.POINTER(C.c_int32), C.POINTER(C.c_uint16),
                                 C.POINTER(C.c_uint8), C.POINTER(C.c_double))
        _lib.oracle_paged_attn_items.argtypes = [
            u16p, C.c_int64, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, i32p, i32p, i32p, i32p, C.c_int,
            u16p, C.c_double, C.c_int64, i32p, i32p, f64p]
        _lib.oracle_paged_attn_items.restype = C.c_int
        _lib.oracle_paged_attn.argtypes = [
            u16p, C.c_int64, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, i32p, i32p, i32p, i32p, C.c_int,
            u16p, C.c_double, f64p]
        _lib.oracle_paged_attn.restype = C.c_int
        _lib.oracle_pack_blocks.argtypes = [u8p, C.c_int64, C.c_int64, i32p, C.c_int64, u8p]
        _lib.oracle_pack_blocks.restype = C.c_int
        _lib.oracle_unpack_blocks.argtypes = [u8p, C.c_int64, C.c_int64, i32p, C.c_int64, u8p]
        _lib.oracle_unpack_blocks.restype = C.c_int
        _lib.oracle_num_threads.restype = C.c_int
        _lib.oracle_kv_append.argtypes = [u16p, C.c_int64, C.c_int, C.c_int, C.c_int, C.c_int, i32p, i32p, i32p,
                                          i32p, C.c_int, u16p, u16p]
        _lib.oracle_kv_append.restype = C.c_int
        vpp, i64p = C.POINTER(C.c_void_p), C.POINTER(C.c_int64)
        dbl = C.c_double
        _lib.oracle_tfwd.argtypes, _lib.oracle_tfwd.restype = [f64p, f64p, C.c_int, dbl], dbl
        _lib.oracle_waste_discard.argtypes = [f64p, f64p, C.c_int, dbl, dbl, dbl]
        _lib.oracle_waste_discard.restype = dbl
        _lib.oracle_waste_preserve.argtypes, _lib.oracle_waste_preserve.restype = [dbl, dbl, dbl], dbl
        _lib.oracle_waste_swap.argtypes, _lib.oracle_waste_swap.restype = [dbl, dbl, dbl], dbl
        _lib.oracle_waste_chunked_discard.argtypes = [f64p, f64p, C.c_int, dbl, dbl, dbl, C.c_int]
        _lib.oracle_waste_chunked_discard.restype = dbl
        _lib.oracle_chunk_tokens.argtypes, _lib.oracle_chunk_tokens.restype = [C.c_int64, C.c_int64], C.c_int64
        _lib.oracle_chunk_count.argtypes, _lib.oracle_chunk_count.restype = [C.c_int64, C.c_int64], C.c_int64
        _lib.oracle_saturation_point.argtypes = [f64p, f64p, C.c_int, dbl]
        _lib.oracle_saturation_point.restype = C.c_int64
        _lib.oracle_schedule_intercepted.argtypes = [C.c_int, f64p, f64p, i64p, C.c_int64, i64p, i32p]
        _lib.oracle_schedule_intercepted.restype = C.c_int
        _lib.oracle_swap_out_layers.argtypes = [vpp, C.c_int64, C.c_int64, C.c_int64, i32p, C.c_int64, u8p, C.c_int64]
        _lib.oracle_swap_out_layers.restype = C.c_int
        _lib.oracle_swap_in_layers.argtypes = [vpp, C.c_int64, C.c_int64, C.c_int64, i32p, C.c_int64, u8p, C.c_int64]
        _lib.oracle_swap_in_layers.restype = C.c_int
        _lib.oracle_swap_limit_tokens.argtypes = [C.c_double, C.c_double, C.c_double]
        _lib.oracle_swap_limit_tokens.restype = C.c_int64
        _lib.oracle_swap_schedule.argtypes = [C.c_int64, C.c_int64, i64p, C.c_int64, i64p]
        _lib.oracle_swap_schedule.restype = C.c_int64
    return _lib


def _p(a: np.ndarray, ctype):
    return a.ctypes.data_as(C.POINTER(ctype))


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


class OracleError(RuntimeError):
    pass


def _check(rc: int) -> None:
    if rc == -1:
        raise MemoryError("oracle: allocation failed")
    if rc == -2:
        raise OracleError("oracle: invalid descriptor or block id")
    if rc == -3:
        raise OracleError("oracle: duplicate destination (block id or cache slot)")
    if rc != 0:
        raise OracleError(f"oracle: error {rc}")


def paged_attn_items(pool_bits, ctx_len, q_len, q_start, block_tables, q_bits, scale,
                     item_seq, item_row) -> np.ndarray:
    """Attention for the listed (sequence, row-in-span) pairs -> fp64 [n_items][H][D].

    pool_bits uint16 [blocks][2][H][B][D]; q_bits uint16 [rows][H][D]; block_tables int32
    [num_seqs][max_blocks] (unused entries may hold anything).
    """
    pool_bits = _c(pool_bits, np.uint16)
    nblk, two, Hkv, B, D = pool_bits.shape
    assert two == 2
    ctx_len, q_len, q_start = _c(ctx_len, np.int32), _c(q_len, np.int32), _c(q_start, np.int32)
    block_tables = _c(block_tables, np.int32)
    q_bits = _c(q_bits, np.uint16)
    assert q_bits.ndim == 3 and q_bits.shape[2] == D
    H = int(q_bits.shape[1])          # query heads; the pool holds Hkv <= H key/value heads
    item_seq, item_row = _c(item_seq, np.int32), _c(item_row, np.int32)
    n = item_seq.shape[0]
    out = np.empty((n, H, D), dtype=np.float64)
    rc = lib().oracle_paged_attn_items(
        _p(pool_bits, C.c_uint16), nblk, B, H, Hkv, D, ctx_len.shape[0], _p(ctx_len, C.c_int32),
        _p(q_len, C.c_int32), _p(q_start, C.c_int32), _p(block_tables, C.c_int32),
        block_tables.shape[1], _p(q_bits, C.c_uint16), float(scale), n,
        _p(item_seq, C.c_int32), _p(item_row, C.c_int32), _p(out, C.c_double))
    _check(rc)
    return out


def paged_attn(pool_bits, ctx_len, q_len, q_start, block_tables, q_bits, scale,
               total_q_rows: Optional[int] = None) -> np.ndarray:
    """Attention for every row of the batch -> fp64 [total_q_rows][H][D]."""
    pool_bits = _c(pool_bits, np.uint16)
    nblk, two, Hkv, B, D = pool_bits.shape
    assert two == 2
    ctx_len, q_len, q_start = _c(ctx_len, np.int32), _c(q_len, np.int32), _c(q_start, np.int32)
    block_tables = _c(block_tables, np.int32)
    q_bits = _c(q_bits, np.uint16)
    H = int(q_bits.shape[1])
    rows = int(q_bits.shape[0]) if total_q_rows is None else int(total_q_rows)
    out = np.full((rows, H, D), np.nan, dtype=np.float64)
    rc = lib().oracle_paged_attn(
        _p(pool_bits, C.c_uint16), nblk, B, H, Hkv, D, ctx_len.shape[0], _p(ctx_len, C.c_int32),
        _p(q_len, C.c_int32), _p(q_start, C.c_int32), _p(block_tables, C.c_int32),
        block_tables.shape[1], _p(q_bits, C.c_uint16), float(scale), _p(out, C.c_double))
    _check(rc)
    return out


def _bf16_to_f64(bits: np.ndarray) -> np.ndarray:
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def attn_partial(pool_bits, table, q_row_bits, scale, k_begin: int, k_end: int, kv_head: int):
    """Split-KV partial of ONE query row of one head over keys [k_begin, k_end) of a paged sequence:
    m = max_t s_t, l = sum_t e^(s_t - m), o~ = sum_t e^(s_t - m) v_t, with s_t = scale * q . k_t (fp64).
    pool_bits uint16 [blocks][2][Hkv][B][D]; table = the sequence's block ids; q_row_bits uint16 [D]."""
    B = pool_bits.shape[3]
    q = _bf16_to_f64(q_row_bits)
    s, v = [], []
    for t in range(int(k_begin), int(k_end)):
        blk, slot = int(table[t // B]), t % B
        s.append(float(scale) * float(np.dot(q, _bf16_to_f64(pool_bits[blk, 0, kv_head, slot]))))
        v.append(_bf16_to_f64(pool_bits[blk, 1, kv_head, slot]))
    s = np.array(s)
    m = float(s.max())
    w = np.exp(s - m)
    return m, float(w.sum()), (w[:, None] * np.array(v)).sum(axis=0)


def merge_partials(parts):
    """Merge of split-KV partials [(m_p, l_p, o~_p), ...]: m = max_p m_p, l = sum_p l_p e^(m_p - m),
    o = sum_p o~_p e^(m_p - m) / l."""
    m = max(p[0] for p in parts)
    l = sum(p[1] * np.exp(p[0] - m) for p in parts)
    o = sum(p[2] * np.exp(p[0] - m) for p in parts)
    return o / l


def attn_batch(batch, pool_bits, q_bits) -> np.ndarray:
    """Convenience: paged_attn on a workloads.Batch-like object (duck-typed, nothing imported)."""
    return paged_attn(pool_bits, batch.ctx_len, batch.q_len, batch.q_start, batch.block_tables,
                      q_bits, batch.scale, batch.total_q_rows)


def pack_blocks(pool_bytes: np.ndarray, ids) -> np.ndarray:
    """staging[i] = pool[ids[i]] as raw bytes; pool_bytes is uint8 [blocks][block_bytes]."""
    pool_bytes = _c(pool_bytes, np.uint8)
    ids = _c(ids, np.int32)
    nblk, bb = pool_bytes.shape
    staging = np.empty((ids.shape[0], bb), dtype=np.uint8)
    _check(lib().oracle_pack_blocks(_p(pool_bytes, C.c_uint8), nblk, bb, _p(ids, C.c_int32),
                                    ids.shape[0], _p(staging, C.c_uint8)))
    return staging


def unpack_blocks(pool_bytes: np.ndarray, ids, staging: np.ndarray) -> None:
    """pool[ids[i]] = staging[i], in place; ids must be distinct."""
    assert pool_bytes.dtype == np.uint8 and pool_bytes.flags.c_contiguous
    ids = _c(ids, np.int32)
    staging = _c(staging, np.uint8)
    nblk, bb = pool_bytes.shape
    assert staging.shape == (ids.shape[0], bb)
    _check(lib().oracle_unpack_blocks(_p(pool_bytes, C.c_uint8), nblk, bb, _p(ids, C.c_int32),
                                      ids.shape[0], _p(staging, C.c_uint8)))


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def kv_append(pool_bits: np.ndarray, ctx_len, q_len, q_start, block_tables, k_new, v_new) -> None:
    """Write rows of k_new / v_new (uint16 [rows][H][D]) into pool_bits (uint16 [blocks][2][H][B][D]) in place:
    row q_start[s] + i goes to logical position ctx_len[s] - q_len[s] + i of sequence s."""
    assert pool_bits.dtype == np.uint16 and pool_bits.flags.c_contiguous
    nblk, two, H, B, D = pool_bits.shape
    assert two == 2
    ctx_len, q_len, q_start = _c(ctx_len, np.int32), _c(q_len, np.int32), _c(q_start, np.int32)
    block_tables = _c(block_tables, np.int32)
    k_new, v_new = _c(k_new, np.uint16), _c(v_new, np.uint16)
    assert k_new.shape == v_new.shape and k_new.shape[1:] == (H, D)
    assert int((q_start + q_len).max()) <= k_new.shape[0]
    _check(lib().oracle_kv_append(_p(pool_bits, C.c_uint16), nblk, B, H, D, ctx_len.shape[0],
                                  _p(ctx_len, C.c_int32), _p(q_len, C.c_int32), _p(q_start, C.c_int32),
                                  _p(block_tables, C.c_int32), block_tables.shape[1],
                                  _p(k_new, C.c_uint16), _p(v_new, C.c_uint16)))


def _layer_ptrs(pools):
    for a in pools:
        assert a.dtype == np.uint8 and a.flags.c_contiguous and a.shape == pools[0].shape
    return (C.c_void_p * len(pools))(*[a.ctypes.data for a in pools])


def swap_out_layers(pools, ids, layer_stride: Optional[int] = None) -> np.ndarray:
    """host[l][i] = pools[l][ids[i]] for every layer l; pools: list of uint8 [blocks][block_bytes].

    Returns uint8 [L][layer_stride]; bytes past n * block_bytes of a layer are left 0xEE."""
    ids = _c(ids, np.int32)
    nblk, bb = pools[0].shape
    stride = ids.shape[0] * bb if layer_stride is None else int(layer_stride)
    host = np.full((len(pools), stride), 0xEE, dtype=np.uint8)
    _check(lib().oracle_swap_out_layers(_layer_ptrs(pools), len(pools), nblk, bb, _p(ids, C.c_int32),
                                        ids.shape[0], _p(host, C.c_uint8), stride))
    return host


def swap_in_layers(pools, ids, host: np.ndarray) -> None:
    """pools[l][ids[i]] = host[l][i], in place; host uint8 [L][layer_stride]; ids distinct."""
    ids = _c(ids, np.int32)
    nblk, bb = pools[0].shape
    assert host.dtype == np.uint8 and host.flags.c_contiguous and host.shape[0] == len(pools)
    _check(lib().oracle_swap_in_layers(_layer_ptrs(pools), len(pools), nblk, bb, _p(ids, C.c_int32),
                                       ids.shape[0], _p(host, C.c_uint8), host.shape[1]))


def swap_limit_tokens(t_fwd: float, bandwidth: float, token_bytes: float) -> int:
    """Swap limit N_i: tokens whose movement at `bandwidth` bytes/s takes t_fwd seconds, rounded down."""
    return int(lib().oracle_swap_limit_tokens(float(t_fwd), float(bandwidth), float(token_bytes)))


def swap_schedule(total_blocks: int, block_size: int, limits) -> tuple:
    """Blocks moved per iteration under per-iteration token limits -> (iterations used, int64 array)."""
    limits = _c(limits, np.int64)
    out = np.zeros(limits.shape[0], dtype=np.int64)
    used = int(lib().oracle_swap_schedule(int(total_blocks), int(block_size), _p(limits, C.c_int64),
                                          limits.shape[0], _p(out, C.c_int64)))
    return used, out


class TfwdTable:
    """Profiled T_fwd: (tokens, seconds) points, tokens strictly increasing."""

    def __init__(self, tokens, seconds):
        self.tokens, self.seconds = _c(tokens, np.float64), _c(seconds, np.float64)
        assert self.tokens.shape == self.seconds.shape and self.tokens.ndim == 1

    def args(self):
        return _p(self.tokens, C.c_double), _p(self.seconds, C.c_double), int(self.tokens.shape[0])


def tfwd(table: TfwdTable, x: float) -> float:
    return float(lib().oracle_tfwd(*table.args(), float(x)))


def waste_discard(table: TfwdTable, C_tokens, C_other, M) -> float:
    return float(lib().oracle_waste_discard(*table.args(), float(C_tokens), float(C_other), float(M)))


def waste_preserve(T_int, C_tokens, M) -> float:
    return float(lib().oracle_waste_preserve(float(T_int), float(C_tokens), float(M)))


def waste_swap(T_swap, C_batch, M) -> float:
    return float(lib().oracle_waste_swap(float(T_swap), float(C_batch), float(M)))


def waste_chunked_discard(table: TfwdTable, C_tokens, C_other, M, n_chunks: int) -> float:
    return float(lib().oracle_waste_chunked_discard(*table.args(), float(C_tokens), float(C_other), float(M),
                                                    int(n_chunks)))


def chunk_tokens(S: int, running: int) -> int:
    return int(lib().oracle_chunk_tokens(int(S), int(running)))


def chunk_count(C_tokens: int, chunk: int) -> int:
    return int(lib().oracle_chunk_count(int(C_tokens), int(chunk)))


def saturation_point(q_tokens, seconds, frac: float = 0.95) -> int:
    q, t = _c(q_tokens, np.float64), _c(seconds, np.float64)
    return int(lib().oracle_saturation_point(_p(q, C.c_double), _p(t, C.c_double), int(q.shape[0]), float(frac)))


def schedule_intercepted(waste_preserve_, waste_chunkd, ctx_tokens, budget: int):
    """-> (swap_tokens int64 [n], action int32 [n]: 0 nothing left, 1 preserve, 2 discard)."""
    wp, wc = _c(waste_preserve_, np.float64), _c(waste_chunkd, np.float64)
    ct = _c(ctx_tokens, np.int64)
    n = int(ct.shape[0])
    sw, act = np.zeros(n, dtype=np.int64), np.zeros(n, dtype=np.int32)
    rc = lib().oracle_schedule_intercepted(n, _p(wp, C.c_double), _p(wc, C.c_double), _p(ct, C.c_int64), int(budget),
                                           _p(sw, C.c_int64), _p(act, C.c_int32))
    if rc != 0:
        raise OracleError("oracle: bad schedule arguments")
    return sw, act
