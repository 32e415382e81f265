"""Thin ctypes binding of libinfercept_hot.so: argument marshalling only.

Function names and argument order follow include/infercept_hot.h.  Every step of the hot path
runs inside the library's HIP kernels; there is no fallback: if the library is not built, or an
entry point fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("INFERCEPT_HOT_LIB") or os.path.join(_HERE, "libinfercept_hot.so")

IC_OK = 0
IC_ENULL, IC_EINVAL, IC_ERANGE, IC_ESIZE, IC_EALIGN = -1, -2, -3, -4, -5
IC_EDUP, IC_EUNSUPPORTED, IC_EOVERLAP, IC_EHIP, IC_ENOMEM, IC_ELIMIT = -6, -7, -8, -9, -10, -11
IC_STATIC_PACK_MAX_BLOCKS = 65536
IC_FLAG_TRUSTED = 1
IC_K_ROW, IC_K_TILE, IC_K_MERGE, IC_K_PACK, IC_K_UNPACK, IC_K_UPLOAD, IC_K_APPEND, IC_K_GROUP, IC_K_COUNT = range(9)
KERNEL_NAMES = ("row", "tile", "merge", "pack", "unpack", "upload", "append", "group")

EXPORTS = (
    "ic_strerror", "kv_pool_init", "kv_pool_destroy", "kv_block_bytes",
    "paged_attn_mixed_workspace_bytes", "paged_attn_mixed", "ic_check_batch", "ic_pool_set_tuning",
    "ic_plan_query", "kv_pack_blocks", "kv_unpack_blocks", "ic_check_ids", "ic_prof_begin",
    "ic_prof_end",
    "ic_swapper_staging_bytes", "ic_swapper_create", "ic_swapper_destroy", "kv_swap_out_layers",
    "kv_swap_in_layers", "ic_swapper_wait_layer", "ic_swapper_sync_layer", "ic_swapper_sync",
    "ic_host_alloc", "ic_host_free", "ic_swap_limit_tokens", "ic_swap_schedule", "kv_write_span",
    "ic_tfwd_eval", "ic_waste_discard", "ic_waste_preserve", "ic_waste_swap", "ic_waste_chunked_discard",
    "ic_chunk_tokens", "ic_chunk_count", "ic_saturation_point", "ic_schedule_intercepted",
    "paged_attn_plan_create", "paged_attn_planned", "paged_attn_plan_destroy", "kv_write_span_planned",
    "ic_mfma_ceiling", "ic_plan_image", "ic_hbm_ceiling", "ic_paged_read_ceiling", "kv_pack_blocks_static",
)
IC_CEILING_OPERAND_BYTES = 1 << 20
IC_CEILING_SINK_BYTES = 256 * 512 * 4 + 256 * 16
IC_ACT_NONE, IC_ACT_PRESERVE, IC_ACT_DISCARD = 0, 1, 2
IC_SWAP_OUT, IC_SWAP_IN = 0, 1


class PoolCfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("num_blocks", "block_size", "num_heads", "num_kv_heads", "head_dim", "dtype", "layout")]


class BatchDesc(C.Structure):
    _fields_ = [("num_seqs", C.c_int32),
                ("ctx_len", C.POINTER(C.c_int32)),
                ("q_len", C.POINTER(C.c_int32)),
                ("q_start", C.POINTER(C.c_int32)),
                ("block_tables", C.POINTER(C.c_int32)),
                ("max_blocks_per_seq", C.c_int32),
                ("total_q_rows", C.c_int32),
                ("scale", C.c_float),
                ("flags", C.c_uint32)]


class Tuning(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("decode_part_tokens", "span_part_tokens", "span_kernel", "row_variant",
                                         "serial_spans", "row_launch", "row_slots", "mfma_min_keys")] + [("reserved", C.c_int32 * 1)]


class PlanInfo(C.Structure):
    _fields_ = [("decode_rows", C.c_int32), ("span_rows", C.c_int32), ("row_items", C.c_int32),
                ("tile_items", C.c_int32), ("partial_slots", C.c_int32), ("merge_rows", C.c_int32),
                ("table_entries", C.c_int64)]


class PlanLayout(C.Structure):
    _fields_ = ([(n, C.c_int64) for n in ("image_bytes", "off_counters", "off_bt_off", "off_bt_flat", "off_row_items",
                                          "off_tile_items", "off_merge_items", "off_row_dst")] +
                [(n, C.c_int32) for n in ("row_part_tokens", "span_part_tokens", "tile_query_rows", "tile_head_shift",
                                          "n_row_items", "n_tile_items", "n_merge_items", "n_vector_row_items")])


class ProfStats(C.Structure):
    _fields_ = [("launches", C.c_int32 * IC_K_COUNT), ("total_ms", C.c_float * IC_K_COUNT),
                ("min_ms", C.c_float * IC_K_COUNT), ("max_ms", C.c_float * IC_K_COUNT)]


class SwapperCfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("num_layers", "max_blocks", "num_stages", "reserved")]


class TfwdTableC(C.Structure):
    _fields_ = [("n", C.c_int32), ("tokens", C.POINTER(C.c_double)), ("seconds", C.POINTER(C.c_double))]


class InferceptError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} ({code})")


_lib = None


def lib():
    """Load the HIP library; fails loudly if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2402_01869_amd.build` "
                              "(there is no CPU fallback)")
        # The library must share ONE HIP runtime with the process that owns the device memory it is
        # handed.  PyTorch ships its own copy of the runtime under the same SONAME: loaded first, it
        # is the one this library binds to; loaded second, the process would hold two runtimes that
        # do not know each other's allocations.
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        L = C.CDLL(LIB_PATH)
        vp, i32p = C.c_void_p, C.POINTER(C.c_int32)
        L.ic_strerror.argtypes, L.ic_strerror.restype = [C.c_int], C.c_char_p
        L.kv_pool_init.argtypes = [C.POINTER(PoolCfg), vp, C.c_size_t, C.POINTER(vp)]
        L.kv_pool_destroy.argtypes = [vp]
        L.kv_block_bytes.argtypes, L.kv_block_bytes.restype = [vp], C.c_size_t
        L.paged_attn_mixed_workspace_bytes.argtypes = [vp, C.POINTER(BatchDesc)]
        L.paged_attn_mixed_workspace_bytes.restype = C.c_size_t
        L.paged_attn_mixed.argtypes = [vp, C.POINTER(BatchDesc), vp, vp, vp, C.c_size_t, vp]
        L.kv_write_span.argtypes = [vp, C.POINTER(BatchDesc), vp, vp, vp]
        L.paged_attn_plan_create.argtypes = [vp, C.POINTER(BatchDesc), vp, C.c_size_t, vp, C.POINTER(vp)]
        L.paged_attn_planned.argtypes = [vp, vp, vp, vp, vp]
        L.kv_write_span_planned.argtypes = [vp, vp, vp, vp, vp]
        L.paged_attn_plan_destroy.argtypes = [vp]
        L.ic_check_batch.argtypes = [C.POINTER(PoolCfg), C.POINTER(BatchDesc)]
        L.ic_pool_set_tuning.argtypes = [vp, C.POINTER(Tuning)]
        L.ic_plan_query.argtypes = [vp, C.POINTER(BatchDesc), C.POINTER(PlanInfo)]
        L.kv_pack_blocks.argtypes = [vp, i32p, C.c_int32, vp, C.c_size_t, vp]
        L.kv_unpack_blocks.argtypes = [vp, i32p, C.c_int32, vp, C.c_size_t, vp]
        L.kv_pack_blocks_static.argtypes = [vp, i32p, C.c_int32, vp, C.c_size_t, vp]
        L.ic_check_ids.argtypes = [C.POINTER(PoolCfg), i32p, C.c_int32, C.c_int]
        L.ic_prof_begin.argtypes = [vp, C.c_int32]
        L.ic_prof_end.argtypes = [vp, C.POINTER(ProfStats)]
        i64p = C.POINTER(C.c_int64)
        L.ic_swapper_staging_bytes.argtypes = [C.POINTER(SwapperCfg), vp]
        L.ic_swapper_staging_bytes.restype = C.c_size_t
        L.ic_swapper_create.argtypes = [C.POINTER(SwapperCfg), C.POINTER(vp), vp, C.c_size_t, C.POINTER(vp)]
        L.ic_swapper_destroy.argtypes = [vp]
        L.kv_swap_out_layers.argtypes = [vp, i32p, C.c_int32, vp, C.c_size_t, vp]
        L.kv_swap_in_layers.argtypes = [vp, i32p, C.c_int32, vp, C.c_size_t, vp]
        L.ic_swapper_wait_layer.argtypes = [vp, C.c_int32, C.c_int32, vp]
        L.ic_swapper_sync_layer.argtypes = [vp, C.c_int32, C.c_int32]
        L.ic_swapper_sync.argtypes = [vp]
        L.ic_host_alloc.argtypes, L.ic_host_alloc.restype = [C.c_size_t], vp
        L.ic_host_free.argtypes = [vp]
        L.ic_swap_limit_tokens.argtypes = [C.c_double, C.c_double, C.c_double]
        L.ic_swap_limit_tokens.restype = C.c_int64
        L.ic_swap_schedule.argtypes = [C.c_int64, C.c_int32, i64p, C.c_int64, i64p]
        L.ic_swap_schedule.restype = C.c_int64
        dbl, f64p, tp = C.c_double, C.POINTER(C.c_double), C.POINTER(TfwdTableC)
        L.ic_tfwd_eval.argtypes, L.ic_tfwd_eval.restype = [tp, dbl], dbl
        L.ic_waste_discard.argtypes, L.ic_waste_discard.restype = [tp, dbl, dbl, dbl], dbl
        L.ic_waste_preserve.argtypes, L.ic_waste_preserve.restype = [dbl, dbl, dbl], dbl
        L.ic_waste_swap.argtypes, L.ic_waste_swap.restype = [dbl, dbl, dbl], dbl
        L.ic_waste_chunked_discard.argtypes = [tp, dbl, dbl, dbl, C.c_int32]
        L.ic_waste_chunked_discard.restype = dbl
        L.ic_chunk_tokens.argtypes, L.ic_chunk_tokens.restype = [C.c_int64, C.c_int64], C.c_int64
        L.ic_chunk_count.argtypes, L.ic_chunk_count.restype = [C.c_int64, C.c_int64], C.c_int64
        L.ic_saturation_point.argtypes, L.ic_saturation_point.restype = [f64p, f64p, C.c_int32, dbl], C.c_int64
        L.ic_schedule_intercepted.argtypes = [C.c_int32, f64p, f64p, i64p, C.c_int64, i64p, i32p]
        other = ("ic_tfwd_eval", "ic_waste_discard", "ic_waste_preserve", "ic_waste_swap", "ic_waste_chunked_discard",
                 "ic_chunk_tokens", "ic_chunk_count", "ic_saturation_point", "ic_strerror", "kv_block_bytes", "paged_attn_mixed_workspace_bytes", "ic_swapper_staging_bytes",
                 "ic_host_alloc", "ic_swap_limit_tokens", "ic_swap_schedule")
        for name in EXPORTS:
            if name not in other:
                getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().ic_strerror(int(code)).decode()


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(C.POINTER(C.c_int32))


def make_cfg(num_blocks, num_heads, head_dim, block_size=16, num_kv_heads=None, dtype=0, layout=0) -> PoolCfg:
    return PoolCfg(int(num_blocks), int(block_size), int(num_heads),
                   int(num_heads if num_kv_heads is None else num_kv_heads), int(head_dim), dtype, layout)


class HostDesc:
    """Keeps the numpy arrays of a batch descriptor alive next to the ctypes struct."""

    def __init__(self, ctx_len, q_len, q_start, block_tables, scale, total_q_rows=None, flags=0):
        self.ctx_len, self.q_len, self.q_start = _i32(ctx_len), _i32(q_len), _i32(q_start)
        self.block_tables = _i32(block_tables)
        if self.block_tables.ndim != 2:
            raise ValueError("block_tables must be [num_seqs][max_blocks_per_seq]")
        rows = int(self.q_len.sum()) if total_q_rows is None else int(total_q_rows)
        self.struct = BatchDesc(int(self.ctx_len.shape[0]), _ptr(self.ctx_len), _ptr(self.q_len),
                                _ptr(self.q_start), _ptr(self.block_tables),
                                int(self.block_tables.shape[1]), rows, float(scale), int(flags))

    @classmethod
    def from_batch(cls, batch, flags=0):
        return cls(batch.ctx_len, batch.q_len, batch.q_start, batch.block_tables, batch.scale,
                   batch.total_q_rows, flags)


def check_batch(cfg: PoolCfg, desc: HostDesc) -> int:
    return int(lib().ic_check_batch(C.byref(cfg), C.byref(desc.struct)))


def check_ids(cfg: PoolCfg, ids, require_distinct: bool) -> int:
    ids = _i32(ids)
    return int(lib().ic_check_ids(C.byref(cfg), _ptr(ids), int(ids.shape[0]), int(require_distinct)))


class KvPool:
    """kv_pool_init / kv_pool_destroy wrapper.  `dev_ptr` is caller-owned device memory."""

    def __init__(self, cfg: PoolCfg, dev_ptr: int, pool_bytes: int):
        self.cfg = cfg
        self._h = C.c_void_p()
        rc = lib().kv_pool_init(C.byref(cfg), C.c_void_p(dev_ptr), int(pool_bytes), C.byref(self._h))
        if rc != IC_OK:
            raise InferceptError(rc, "kv_pool_init")

    @classmethod
    def from_tensor(cls, pool_t, num_heads, head_dim, block_size=16, num_kv_heads=None):
        """pool_t: a contiguous torch device tensor holding [blocks][2][Hkv][B][D] bf16 (Hkv = num_kv_heads,
        num_heads if not given)."""
        nbytes = pool_t.numel() * pool_t.element_size()
        hkv = num_heads if num_kv_heads is None else num_kv_heads
        bb = block_size * 2 * hkv * head_dim * 2
        obj = cls(make_cfg(nbytes // bb, num_heads, head_dim, block_size, hkv), pool_t.data_ptr(), nbytes)
        obj._keep = pool_t
        return obj

    def close(self):
        if self._h:
            lib().kv_pool_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def block_bytes(self) -> int:
        return int(lib().kv_block_bytes(self._h))

    def set_tuning(self, decode_part_tokens=0, span_part_tokens=0, span_kernel=0, row_variant=0, serial_spans=0,
                   row_launch=0, row_slots=0, mfma_min_keys=0):
        t = Tuning(int(decode_part_tokens), int(span_part_tokens), int(span_kernel), int(row_variant),
                   int(serial_spans), int(row_launch), int(row_slots), int(mfma_min_keys), (C.c_int32 * 1)(0))
        rc = lib().ic_pool_set_tuning(self._h, C.byref(t))
        if rc != IC_OK:
            raise InferceptError(rc, "ic_pool_set_tuning")

    def plan_query(self, desc: HostDesc) -> dict:
        info = PlanInfo()
        rc = lib().ic_plan_query(self._h, C.byref(desc.struct), C.byref(info))
        if rc != IC_OK:
            raise InferceptError(rc, "ic_plan_query")
        return {n: int(getattr(info, n)) for n, _ in PlanInfo._fields_}

    def plan_image(self, desc: HostDesc) -> dict:
        """ic_plan_image: the launch plan as numpy arrays (host only, no GPU): layout fields plus `bt_off`, `bt_flat`,
        `row_items` [n][8], `tile_items` [n][8], `merge_items` [n][4], `row_dst`, `counters`."""
        lay = PlanLayout()
        rc = lib().ic_plan_image(self._h, C.byref(desc.struct), None, C.c_size_t(0), C.byref(lay))
        if rc != IC_OK:
            raise InferceptError(rc, "ic_plan_image")
        img = np.zeros(int(lay.image_bytes) // 4, dtype=np.int32)
        rc = lib().ic_plan_image(self._h, C.byref(desc.struct), img.ctypes.data_as(C.c_void_p),
                                 C.c_size_t(img.nbytes), C.byref(lay))
        if rc != IC_OK:
            raise InferceptError(rc, "ic_plan_image")
        out = {n: int(getattr(lay, n)) for n, _ in PlanLayout._fields_ if n != "reserved"}
        info = self.plan_query(desc)
        sec = lambda off, count: img[off // 4: off // 4 + count]
        out["counters"] = sec(out["off_counters"], 16)
        out["bt_off"] = sec(out["off_bt_off"], int(desc.struct.num_seqs))
        out["bt_flat"] = sec(out["off_bt_flat"], info["table_entries"])
        out["row_items"] = sec(out["off_row_items"], 8 * out["n_row_items"]).reshape(-1, 8)
        out["tile_items"] = sec(out["off_tile_items"], 8 * out["n_tile_items"]).reshape(-1, 8)
        out["merge_items"] = sec(out["off_merge_items"], 4 * out["n_merge_items"]).reshape(-1, 4)
        out["row_dst"] = sec(out["off_row_dst"], int(desc.struct.total_q_rows))
        out["partial_slots"] = info["partial_slots"]
        return out

    def paged_read_ceiling(self, ids, dev_sink: int, reps: int = 1, stream: int = 0, check: bool = True):
        """ic_paged_read_ceiling: GB/s of a compute-free read of the listed blocks, tile by tile (rc, GB/s if not check)."""
        ids = _i32(ids)
        g = C.c_double(0.0)
        rc = lib().ic_paged_read_ceiling(self._h, _ptr(ids), int(ids.shape[0]), C.c_void_p(dev_sink), C.c_int32(reps),
                                         C.c_void_p(stream), C.byref(g))
        if check and rc != IC_OK:
            raise InferceptError(rc, "ic_paged_read_ceiling")
        return g.value if check else (int(rc), g.value)

    def workspace_bytes(self, desc: HostDesc) -> int:
        return int(lib().paged_attn_mixed_workspace_bytes(self._h, C.byref(desc.struct)))

    def paged_attn_mixed(self, desc: HostDesc, q_ptr: int, out_ptr: int, ws_ptr: int, ws_bytes: int,
                         stream: int = 0, check: bool = True) -> int:
        rc = lib().paged_attn_mixed(self._h, C.byref(desc.struct), C.c_void_p(q_ptr), C.c_void_p(out_ptr),
                                    C.c_void_p(ws_ptr), int(ws_bytes), C.c_void_p(stream))
        if check and rc != IC_OK:
            raise InferceptError(rc, "paged_attn_mixed")
        return int(rc)

    def plan_create(self, desc: HostDesc, ws_ptr: int, ws_bytes: int, stream: int = 0) -> "AttnPlan":
        h = C.c_void_p()
        rc = lib().paged_attn_plan_create(self._h, C.byref(desc.struct), C.c_void_p(ws_ptr), int(ws_bytes),
                                          C.c_void_p(stream), C.byref(h))
        if rc != IC_OK:
            raise InferceptError(rc, "paged_attn_plan_create")
        return AttnPlan(h)

    def paged_attn_planned(self, plan: "AttnPlan", q_ptr: int, out_ptr: int, stream: int = 0, check: bool = True) -> int:
        rc = lib().paged_attn_planned(self._h, plan._h, C.c_void_p(q_ptr), C.c_void_p(out_ptr), C.c_void_p(stream))
        if check and rc != IC_OK:
            raise InferceptError(rc, "paged_attn_planned")
        return int(rc)

    def kv_write_span_planned(self, plan: "AttnPlan", k_ptr: int, v_ptr: int, stream: int = 0, check: bool = True) -> int:
        rc = lib().kv_write_span_planned(self._h, plan._h, C.c_void_p(k_ptr), C.c_void_p(v_ptr), C.c_void_p(stream))
        if check and rc != IC_OK:
            raise InferceptError(rc, "kv_write_span_planned")
        return int(rc)

    def kv_write_span(self, desc: HostDesc, k_ptr: int, v_ptr: int, stream: int = 0, check: bool = True) -> int:
        rc = lib().kv_write_span(self._h, C.byref(desc.struct), C.c_void_p(k_ptr), C.c_void_p(v_ptr), C.c_void_p(stream))
        if check and rc != IC_OK:
            raise InferceptError(rc, "kv_write_span")
        return int(rc)

    def kv_pack_blocks(self, ids, staging_ptr: int, staging_bytes: int, stream: int = 0, check: bool = True) -> int:
        ids = _i32(ids)
        rc = lib().kv_pack_blocks(self._h, _ptr(ids), int(ids.shape[0]), C.c_void_p(staging_ptr),
                                  int(staging_bytes), C.c_void_p(stream))
        if check and rc != IC_OK:
            raise InferceptError(rc, "kv_pack_blocks")
        return int(rc)

    def kv_pack_blocks_static(self, ids, staging_ptr: int, staging_bytes: int, stream: int = 0, check: bool = True) -> int:
        """kv_pack_blocks without any allocation: the id list goes to a fixed array in the library's device image."""
        ids = _i32(ids)
        rc = lib().kv_pack_blocks_static(self._h, _ptr(ids), int(ids.shape[0]), C.c_void_p(staging_ptr),
                                         int(staging_bytes), C.c_void_p(stream))
        if check and rc != IC_OK:
            raise InferceptError(rc, "kv_pack_blocks_static")
        return int(rc)

    def kv_unpack_blocks(self, ids, staging_ptr: int, staging_bytes: int, stream: int = 0, check: bool = True) -> int:
        ids = _i32(ids)
        rc = lib().kv_unpack_blocks(self._h, _ptr(ids), int(ids.shape[0]), C.c_void_p(staging_ptr),
                                    int(staging_bytes), C.c_void_p(stream))
        if check and rc != IC_OK:
            raise InferceptError(rc, "kv_unpack_blocks")
        return int(rc)

    def prof_begin(self, max_launches: int = 4096):
        rc = lib().ic_prof_begin(self._h, int(max_launches))
        if rc != IC_OK:
            raise InferceptError(rc, "ic_prof_begin")

    def prof_end(self) -> dict:
        st = ProfStats()
        rc = lib().ic_prof_end(self._h, C.byref(st))
        if rc != IC_OK:
            raise InferceptError(rc, "ic_prof_end")
        return {KERNEL_NAMES[k]: {"launches": int(st.launches[k]), "total_ms": float(st.total_ms[k]),
                                 "min_ms": float(st.min_ms[k]), "max_ms": float(st.max_ms[k])}
                for k in range(IC_K_COUNT)}


def swap_limit_tokens(t_fwd_s: float, link_bytes_per_s: float, token_bytes: float) -> int:
    """Swap limit N_i: tokens whose swap takes as long as a forward pass of t_fwd_s seconds."""
    return int(lib().ic_swap_limit_tokens(float(t_fwd_s), float(link_bytes_per_s), float(token_bytes)))


def swap_schedule(total_blocks: int, block_size: int, limits):
    """Blocks to move in each iteration under per-iteration token limits -> (iterations used, int64 array)."""
    lim = np.ascontiguousarray(limits, dtype=np.int64)
    out = np.zeros(lim.shape[0], dtype=np.int64)
    i64p = C.POINTER(C.c_int64)
    used = int(lib().ic_swap_schedule(int(total_blocks), int(block_size), lim.ctypes.data_as(i64p),
                                      lim.shape[0], out.ctypes.data_as(i64p)))
    return used, out


class AttnPlan:
    """Handle of a planned batch (descriptor image resident in the caller's workspace)."""

    def __init__(self, handle):
        self._h = handle

    def close(self):
        if self._h:
            lib().paged_attn_plan_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class PinnedBuffer:
    """Pinned host memory from the library, viewed as a numpy uint8 array."""

    def __init__(self, nbytes: int):
        self.nbytes = int(nbytes)
        self.ptr = lib().ic_host_alloc(self.nbytes)
        if not self.ptr:
            raise MemoryError(f"ic_host_alloc({self.nbytes}) failed")
        self.array = np.ctypeslib.as_array((C.c_uint8 * self.nbytes).from_address(self.ptr))

    def close(self):
        if self.ptr:
            self.array = None
            lib().ic_host_free(C.c_void_p(self.ptr))
            self.ptr = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class LayerSwapper:
    """Layer-pipelined swap of listed blocks between L same-shaped pools and pinned host memory."""

    def __init__(self, pools, max_blocks: int, staging_ptr: int, staging_bytes: int, num_stages: int = 2):
        self.pools = list(pools)
        self.cfg = SwapperCfg(len(self.pools), int(max_blocks), int(num_stages), 0)
        arr = (C.c_void_p * len(self.pools))(*[p._h for p in self.pools])
        h = C.c_void_p()
        rc = lib().ic_swapper_create(C.byref(self.cfg), arr, C.c_void_p(staging_ptr), int(staging_bytes), C.byref(h))
        if rc != IC_OK:
            raise InferceptError(rc, "ic_swapper_create")
        self._h = h

    @staticmethod
    def staging_bytes(pool, num_layers: int, max_blocks: int, num_stages: int = 2) -> int:
        cfg = SwapperCfg(int(num_layers), int(max_blocks), int(num_stages), 0)
        return int(lib().ic_swapper_staging_bytes(C.byref(cfg), pool._h))

    def close(self):
        if self._h:
            lib().ic_swapper_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _call(self, fn, name, ids, host_ptr, layer_stride, after_stream, check):
        ids = _i32(ids)
        rc = fn(self._h, _ptr(ids), int(ids.shape[0]), C.c_void_p(host_ptr), int(layer_stride),
                C.c_void_p(after_stream))
        if check and rc != IC_OK:
            raise InferceptError(rc, name)
        return int(rc)

    def swap_out(self, ids, host_ptr: int, layer_stride: int, after_stream: int = 0, check: bool = True) -> int:
        return self._call(lib().kv_swap_out_layers, "kv_swap_out_layers", ids, host_ptr, layer_stride,
                          after_stream, check)

    def swap_in(self, ids, host_ptr: int, layer_stride: int, after_stream: int = 0, check: bool = True) -> int:
        return self._call(lib().kv_swap_in_layers, "kv_swap_in_layers", ids, host_ptr, layer_stride,
                          after_stream, check)

    def wait_layer(self, direction: int, layer: int, stream: int = 0) -> int:
        rc = lib().ic_swapper_wait_layer(self._h, int(direction), int(layer), C.c_void_p(stream))
        if rc != IC_OK:
            raise InferceptError(rc, "ic_swapper_wait_layer")
        return rc

    def sync_layer(self, direction: int, layer: int) -> int:
        rc = lib().ic_swapper_sync_layer(self._h, int(direction), int(layer))
        if rc != IC_OK:
            raise InferceptError(rc, "ic_swapper_sync_layer")
        return rc

    def sync(self):
        rc = lib().ic_swapper_sync(self._h)
        if rc != IC_OK:
            raise InferceptError(rc, "ic_swapper_sync")


class TfwdTable:
    """Profiled T_fwd as (tokens, seconds) points, kept alive next to the C struct."""

    def __init__(self, tokens, seconds):
        self.tokens = np.ascontiguousarray(tokens, dtype=np.float64)
        self.seconds = np.ascontiguousarray(seconds, dtype=np.float64)
        if self.tokens.shape != self.seconds.shape or self.tokens.ndim != 1:
            raise ValueError("tokens and seconds must be 1-D and of one length")
        f64p = C.POINTER(C.c_double)
        self.struct = TfwdTableC(int(self.tokens.shape[0]), self.tokens.ctypes.data_as(f64p),
                                 self.seconds.ctypes.data_as(f64p))

    def __call__(self, tokens: float) -> float:
        return float(lib().ic_tfwd_eval(C.byref(self.struct), float(tokens)))


def waste_discard(table: TfwdTable, ctx_tokens, other_tokens, token_bytes) -> float:
    return float(lib().ic_waste_discard(C.byref(table.struct), float(ctx_tokens), float(other_tokens), float(token_bytes)))


def waste_preserve(t_int_s, ctx_tokens, token_bytes) -> float:
    return float(lib().ic_waste_preserve(float(t_int_s), float(ctx_tokens), float(token_bytes)))


def waste_swap(t_swap_s, batch_tokens, token_bytes) -> float:
    return float(lib().ic_waste_swap(float(t_swap_s), float(batch_tokens), float(token_bytes)))


def waste_chunked_discard(table: TfwdTable, ctx_tokens, other_tokens, token_bytes, n_chunks: int) -> float:
    return float(lib().ic_waste_chunked_discard(C.byref(table.struct), float(ctx_tokens), float(other_tokens),
                                                float(token_bytes), int(n_chunks)))


def chunk_tokens(saturation_point: int, running_tokens: int) -> int:
    return int(lib().ic_chunk_tokens(int(saturation_point), int(running_tokens)))


def chunk_count(ctx_tokens: int, chunk: int) -> int:
    return int(lib().ic_chunk_count(int(ctx_tokens), int(chunk)))


def saturation_point(query_tokens, seconds, frac: float = 0.95) -> int:
    q = np.ascontiguousarray(query_tokens, dtype=np.float64)
    t = np.ascontiguousarray(seconds, dtype=np.float64)
    f64p = C.POINTER(C.c_double)
    return int(lib().ic_saturation_point(q.ctypes.data_as(f64p), t.ctypes.data_as(f64p), int(q.shape[0]), float(frac)))


def schedule_intercepted(waste_preserve_, waste_chunkd, ctx_tokens, budget: int):
    """-> (rc, swap_tokens int64 [n], action int32 [n])."""
    wp = np.ascontiguousarray(waste_preserve_, dtype=np.float64)
    wc = np.ascontiguousarray(waste_chunkd, dtype=np.float64)
    ct = np.ascontiguousarray(ctx_tokens, dtype=np.int64)
    n = int(ct.shape[0])
    sw, act = np.zeros(n, dtype=np.int64), np.zeros(n, dtype=np.int32)
    f64p, i64p = C.POINTER(C.c_double), C.POINTER(C.c_int64)
    rc = int(lib().ic_schedule_intercepted(n, wp.ctypes.data_as(f64p), wc.ctypes.data_as(f64p), ct.ctypes.data_as(i64p),
                                           int(budget), sw.ctypes.data_as(i64p), act.ctypes.data_as(C.POINTER(C.c_int32))))
    return rc, sw, act


def mfma_ceiling(dev_operands: int, operand_bytes: int, dev_sink: int, sink_bytes: int, iters: int, stream: int = 0):
    """ic_mfma_ceiling: returns (rc, tflops, shader_ghz)."""
    tf, ghz = C.c_double(0.0), C.c_double(0.0)
    rc = lib().ic_mfma_ceiling(C.c_void_p(dev_operands), C.c_size_t(operand_bytes), C.c_void_p(dev_sink),
                               C.c_size_t(sink_bytes), C.c_int32(iters), C.c_void_p(stream), C.byref(tf), C.byref(ghz))
    return rc, tf.value, ghz.value


def hbm_ceiling(dev_src: int, dev_dst: int, nbytes: int, mode: int, reps: int, stream: int = 0):
    """ic_hbm_ceiling: returns (rc, GB/s); mode 0 = streaming read, 1 = copy."""
    g = C.c_double(0.0)
    rc = lib().ic_hbm_ceiling(C.c_void_p(dev_src), C.c_void_p(dev_dst), C.c_size_t(nbytes), C.c_int32(mode),
                              C.c_int32(reps), C.c_void_p(stream), C.byref(g))
    return rc, g.value
