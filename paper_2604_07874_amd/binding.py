"""ctypes binding: same names as the C ABI, argument marshalling only.

Device arguments are torch tensors (their data_ptr is passed) or raw integer
addresses; host arguments are numpy arrays.  Streams are torch.cuda.Stream
objects, raw hipStream_t integers, or None for torch's current stream.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np

__all__ = [
    "VKV_OK", "VKV_YIELDED", "VKV_E_INVAL", "VKV_E_NOSPACE", "VKV_E_BUSY", "VKV_E_HIP", "VKV_E_STATE",
    "VKV_RECLAIM_ASYNC", "VKV_RECLAIM_NO_GRACE", "VkvError", "EvictInfo", "kv_handles_cost", "kv_evict_handles",
    "kv_reclaim_or_evict", "PoolConfig", "AttnPlanInfo", "ReclaimStats", "lib", "library_path",
    "last_error", "kv_pool_init", "kv_pool_destroy", "kv_pool_alloc", "kv_pool_adopt", "kv_pool_free",
    "kv_pool_return_range", "kv_pool_state", "kv_pool_check_tables", "kv_attn_plan", "kv_attn_plan_read",
    "kv_attn_bind", "paged_decode_attn_slice", "kv_attn_check", "kv_attn_run_layer",
    "paged_decode_attn_layer_static",
    "kv_yield_request", "kv_yield_clear", "kv_yield_pending", "kv_reclaim_plan", "kv_reclaim_range",
    "block_table_rewrite", "kv_profile_enable", "kv_profile_read", "kv_profile_sample", "ProfileRecord",
    "VKV_PROF_SLICE", "VKV_PROF_RELOCATE", "VKV_PROF_REWRITE",
    "PrefillPlanInfo", "kv_prefill_plan", "kv_prefill_plan_read", "kv_prefill_bind", "paged_prefill_attn_slice",
    "kv_prefill_merge", "kv_prefill_run_layer", "kv_prefill_check", "VKV_PROF_PREFILL", "VKV_PROF_PREFILL_MERGE",
    "kv_select_handles", "kv_invalidate_handles", "MiadConfig", "MiadStep", "kv_miad_init", "kv_miad_destroy",
    "kv_miad_observe", "kv_gate_init", "kv_gate_destroy", "kv_gate_online_busy", "kv_gate_online_idle",
    "kv_gate_poll", "kv_gate_stats", "kv_probe_read", "kv_probe_copy", "kv_probe_attn_reads", "kv_sched_set_overlap",
    "kv_arena_create", "kv_arena_destroy", "kv_pool_attach_arena", "kv_arena_release", "kv_arena_restore",
    "kv_arena_state", "DeviceSpan",
]

VKV_OK, VKV_YIELDED = 0, 1
VKV_E_INVAL, VKV_E_NOSPACE, VKV_E_BUSY, VKV_E_HIP, VKV_E_STATE = -1, -2, -3, -4, -5
VKV_RECLAIM_ASYNC = 1
VKV_RECLAIM_NO_GRACE = 2
VKV_PROF_SLICE, VKV_PROF_RELOCATE, VKV_PROF_REWRITE, VKV_PROF_PREFILL, VKV_PROF_PREFILL_MERGE = 0, 1, 2, 3, 4

_HERE = os.path.dirname(os.path.abspath(__file__))


def library_path() -> str:
    """The in-tree library; VALVEKV_LIBRARY names another build of the same sources (the host-sanitizer one)."""
    return os.environ.get("VALVEKV_LIBRARY") or os.path.join(_HERE, "libvalvekv.so")


class VkvError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"valvekv error {code}: {msg}")
        self.code = code


class PoolConfig(C.Structure):
    _fields_ = [("num_layers", C.c_int32), ("num_q_heads", C.c_int32), ("num_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("block_tokens", C.c_int32), ("num_blocks", C.c_int32),
                ("blocks_per_handle", C.c_int32), ("reserved", C.c_int32),
                ("base", C.c_void_p), ("bytes", C.c_uint64)]


class AttnPlanInfo(C.Structure):
    _fields_ = [("n_items", C.c_int32), ("n_slices", C.c_int32), ("workspace_bytes", C.c_uint64),
                ("kv_bytes_per_layer", C.c_uint64), ("max_slice_kv_bytes", C.c_uint64)]


class ReclaimStats(C.Structure):
    _fields_ = [("bytes_moved", C.c_uint64), ("blocks_moved", C.c_int32), ("blocks_in_range", C.c_int32),
                ("n_chunks", C.c_int32), ("reserved", C.c_int32), ("host_seconds", C.c_double)]


class ProfileRecord(C.Structure):
    _fields_ = [("kind", C.c_int32), ("index", C.c_int32), ("ms", C.c_float)]


class PrefillPlanInfo(C.Structure):
    _fields_ = [("n_items", C.c_int32), ("n_slices", C.c_int32), ("n_tiles", C.c_int32),
                ("tile_positions", C.c_int32), ("total_q", C.c_int32), ("n_merge_steps", C.c_int32),
                ("workspace_bytes", C.c_uint64), ("kv_bytes_per_layer", C.c_uint64),
                ("max_slice_kv_bytes", C.c_uint64), ("flops_per_layer", C.c_double)]


class EvictInfo(C.Structure):
    _fields_ = [("mode", C.c_int32), ("n_handles", C.c_int32), ("n_evicted", C.c_int32), ("n_invalidated", C.c_int32),
                ("total_cost", C.c_int64)]


class MiadConfig(C.Structure):
    _fields_ = [("h_init", C.c_int32), ("h_min", C.c_int32), ("h_max", C.c_int32), ("reserved", C.c_int32),
                ("alpha", C.c_double), ("pressure_frac", C.c_double), ("t_init", C.c_double), ("t_min", C.c_double),
                ("t_max", C.c_double), ("t_up", C.c_double), ("t_down", C.c_double), ("window_s", C.c_double),
                ("target_rate", C.c_double)]


class MiadStep(C.Structure):
    _fields_ = [("headroom", C.c_int32), ("grow_by", C.c_int32), ("release", C.c_int32),
                ("pressure_event", C.c_int32), ("interval_s", C.c_double)]


def _load():
    path = library_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: build it with `python -m paper_2604_07874_amd.build` "
                          "(there is no fallback path)")
    return C.CDLL(path)


lib = _load()

_P = C.c_void_p
_I32P = C.POINTER(C.c_int32)
_sigs = {
    "vkv_last_error": (C.c_char_p, []),
    "kv_pool_init": (C.c_int, [C.POINTER(PoolConfig), C.POINTER(_P)]),
    "kv_pool_destroy": (C.c_int, [_P]),
    "kv_pool_alloc": (C.c_int, [_P, C.c_int32, _P]),
    "kv_pool_adopt": (C.c_int, [_P, _P, C.c_int32]),
    "kv_pool_free": (C.c_int, [_P, _P, C.c_int32]),
    "kv_pool_return_range": (C.c_int, [_P, C.c_int32, C.c_int32]),
    "kv_pool_state": (C.c_int, [_P, _P, _P, C.c_int32, _I32P]),
    "kv_pool_check_tables": (C.c_int, [_P, _P, C.c_int64]),
    "kv_attn_plan": (C.c_int, [_P, _P, C.c_int32, C.c_uint64, C.c_int32, C.POINTER(AttnPlanInfo)]),
    "kv_attn_plan_read": (C.c_int, [_P, _P, _P]),
    "kv_attn_bind": (C.c_int, [_P, _P, C.c_uint64, _P]),
    "paged_decode_attn_slice": (C.c_int, [_P, C.c_int32, C.c_int32, _P, _P, C.c_int32, _P, _P, C.c_float, _P]),
    "kv_attn_check": (C.c_int, [_P, _P, _P]),
    "paged_decode_attn_layer_static": (C.c_int, [_P, C.c_int32, _P, _P, C.c_int32, _P, C.c_int32, C.c_int32, C.c_int32,
                                                 _P, _P, C.c_float, _P]),
    "kv_attn_run_layer": (C.c_int, [_P, C.c_int32, _I32P, _P, _P, C.c_int32, _P, _P, C.c_float, C.c_int32, _P]),
    "kv_yield_request": (C.c_int, [_P]),
    "kv_yield_clear": (C.c_int, [_P]),
    "kv_yield_pending": (C.c_int, [_P]),
    "kv_reclaim_plan": (C.c_int, [_P, C.c_int32, C.c_int32, _P, C.POINTER(ReclaimStats)]),
    "kv_reclaim_range": (C.c_int, [_P, C.c_int32, C.c_int32, _P, C.c_int64, C.c_uint64, C.c_uint64, _P, _P, _P,
                                   C.c_uint32, C.POINTER(ReclaimStats)]),
    "block_table_rewrite": (C.c_int, [_P, C.c_int64, _P, C.c_int32, _P]),
    "kv_prefill_plan": (C.c_int, [_P, _P, _P, C.c_int32, C.c_uint64, C.c_int32, C.POINTER(PrefillPlanInfo)]),
    "kv_prefill_plan_read": (C.c_int, [_P, _P, _P, _P, _P]),
    "kv_prefill_bind": (C.c_int, [_P, _P, C.c_uint64, _P]),
    "paged_prefill_attn_slice": (C.c_int, [_P, C.c_int32, C.c_int32, _P, _P, C.c_int32, _P, _P, C.c_float, _P]),
    "kv_prefill_merge": (C.c_int, [_P, C.c_int32, _P, _P, _P]),
    "kv_prefill_run_layer": (C.c_int, [_P, C.c_int32, _I32P, _P, _P, C.c_int32, _P, _P, C.c_float, C.c_int32, _P]),
    "kv_prefill_check": (C.c_int, [_P, _P, _P]),
    "kv_select_handles": (C.c_int, [_P, _P, C.c_int32, C.c_int32, _P, C.c_int32, _P, _P, _I32P, C.POINTER(C.c_int64)]),
    "kv_invalidate_handles": (C.c_int, [_P, _P, C.c_int32, _P, C.c_int32, C.c_int32, _P, _P, _P, C.c_int32, _I32P,
                                        _P, _P, _P, _P]),
    "kv_handles_cost": (C.c_int, [_P, _P, C.c_int32, C.c_int32, _P, _P, C.c_int32, _P, _I32P, C.POINTER(C.c_int64)]),
    "kv_evict_handles": (C.c_int, [_P, C.c_int32, _P, C.c_int32, C.c_int32, _P, _P, _P, _P, _P, _P, _P, _P, _P, _P,
                                   C.c_int32, C.POINTER(EvictInfo)]),
    "kv_reclaim_or_evict": (C.c_int, [_P, C.c_int32, C.c_int32, _P, _P, C.c_int32, C.c_int32, _P, C.c_uint64, C.c_uint64,
                                      _P, _P, _P, C.c_uint32, _P, _P, _P, _P, _P, C.c_int32, C.POINTER(EvictInfo),
                                      C.POINTER(ReclaimStats)]),
    "kv_miad_init": (C.c_int, [C.POINTER(MiadConfig), C.POINTER(_P)]),
    "kv_miad_destroy": (C.c_int, [_P]),
    "kv_miad_observe": (C.c_int, [_P, C.c_double, C.c_int32, C.POINTER(MiadStep)]),
    "kv_gate_init": (C.c_int, [C.c_double, C.POINTER(_P)]),
    "kv_gate_destroy": (C.c_int, [_P]),
    "kv_gate_online_busy": (C.c_int, [_P, C.c_double, C.c_int64]),
    "kv_gate_online_idle": (C.c_int, [_P, C.c_double]),
    "kv_gate_poll": (C.c_int, [_P, C.c_double]),
    "kv_gate_stats": (C.c_int, [_P, C.POINTER(C.c_double), C.POINTER(C.c_int64)]),
    "kv_profile_enable": (C.c_int, [_P, C.c_int32]),
    "kv_profile_read": (C.c_int, [_P, _P, C.c_int32, _I32P]),
    "kv_profile_sample": (C.c_int, [_P, C.c_int32]),
    "kv_sched_set_overlap": (C.c_int, [_P, C.c_int32]),
    "kv_arena_create": (C.c_int, [C.c_int32, C.c_uint64, C.c_int32, C.POINTER(_P), C.POINTER(_P)]),
    "kv_arena_destroy": (C.c_int, [_P]),
    "kv_pool_attach_arena": (C.c_int, [_P, _P]),
    "kv_arena_release": (C.c_int, [_P, _P, C.c_int32, C.c_int32]),
    "kv_arena_restore": (C.c_int, [_P, _P, C.c_int32, C.c_int32]),
    "kv_arena_state": (C.c_int, [_P, _P, C.POINTER(C.c_uint64)]),
    "kv_probe_read": (C.c_int, [_P, C.c_uint64, _P, _P]),
    "kv_probe_attn_reads": (C.c_int, [_P, C.c_int32, C.c_int32, _P, C.c_int32, _P, _P, _P]),
    "kv_probe_copy": (C.c_int, [_P, _P, C.c_uint64, _P]),
}
for _name, (_res, _args) in _sigs.items():
    _fn = getattr(lib, _name)
    _fn.restype = _res
    _fn.argtypes = _args


def last_error() -> str:
    return lib.vkv_last_error().decode()


def _check(code: int, ok=(VKV_OK,)):
    if code not in ok:
        raise VkvError(code, last_error())
    return code


def _dev(x) -> Optional[int]:
    """Device address of a torch tensor, or an int address, or None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    assert x.is_cuda and x.is_contiguous(), "device arguments must be contiguous device tensors"
    return x.data_ptr()


def _host(a: np.ndarray, dtype) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def _stream(s) -> Optional[int]:
    if s is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(s, int):
        return s or None
    return s.cuda_stream or None


# ---- pool -------------------------------------------------------------------------
def kv_pool_init(num_layers, num_q_heads, num_kv_heads, head_dim, num_blocks, blocks_per_handle,
                 base=None, nbytes=0, block_tokens=16):
    """base: torch tensor holding the pool (or None for a host-only pool).  Returns the pool handle."""
    cfg = PoolConfig(num_layers, num_q_heads, num_kv_heads, head_dim, block_tokens, num_blocks,
                     blocks_per_handle, 0, _dev(base),
                     nbytes if isinstance(base, int) or base is None else base.numel() * base.element_size())
    out = _P()
    _check(lib.kv_pool_init(C.byref(cfg), C.byref(out)))
    return out


def kv_pool_destroy(pool):
    _check(lib.kv_pool_destroy(pool))


def kv_pool_alloc(pool, n: int) -> np.ndarray:
    ids = np.empty(n, dtype=np.int32)
    _check(lib.kv_pool_alloc(pool, n, ids.ctypes.data))
    return ids


def kv_pool_adopt(pool, ids):
    ids = _host(ids, np.int32)
    _check(lib.kv_pool_adopt(pool, ids.ctypes.data, len(ids)))


def kv_pool_free(pool, ids):
    ids = _host(ids, np.int32)
    _check(lib.kv_pool_free(pool, ids.ctypes.data, len(ids)))


def kv_pool_return_range(pool, lo: int, hi: int):
    _check(lib.kv_pool_return_range(pool, lo, hi))


def kv_pool_state(pool, num_blocks: int, max_ranges: int = 64):
    """Returns (live uint8[NB], list of handed-over (lo, hi))."""
    live = np.empty(num_blocks, dtype=np.uint8)
    ranges = np.empty(2 * max_ranges, dtype=np.int32)
    n = C.c_int32(0)
    _check(lib.kv_pool_state(pool, live.ctypes.data, ranges.ctypes.data, max_ranges, C.byref(n)))
    k = min(n.value, max_ranges)
    return live, [(int(ranges[2 * i]), int(ranges[2 * i + 1])) for i in range(k)]


def kv_pool_check_tables(pool, tables_host):
    t = _host(tables_host, np.int32)
    _check(lib.kv_pool_check_tables(pool, t.ctypes.data, t.size))


# ---- attention --------------------------------------------------------------------
def kv_attn_plan(pool, ctx_len_host, slice_bytes: int, chunk_tokens: int) -> AttnPlanInfo:
    ctx = _host(ctx_len_host, np.int32)
    info = AttnPlanInfo()
    _check(lib.kv_attn_plan(pool, ctx.ctypes.data, len(ctx), slice_bytes, chunk_tokens, C.byref(info)))
    return info


def kv_attn_plan_read(pool, info: AttnPlanInfo):
    work = np.empty((info.n_items, 4), dtype=np.int32)
    starts = np.empty(info.n_slices + 1, dtype=np.int32)
    _check(lib.kv_attn_plan_read(pool, work.ctypes.data, starts.ctypes.data))
    return work, starts


def kv_attn_bind(pool, workspace, stream=None):
    _check(lib.kv_attn_bind(pool, _dev(workspace), workspace.numel() * workspace.element_size(), _stream(stream)))


def paged_decode_attn_slice(pool, layer: int, slice_idx: int, q, block_table, workspace, out,
                            softmax_scale: float = 0.0, stream=None):
    _check(lib.paged_decode_attn_slice(pool, layer, slice_idx, _dev(q), _dev(block_table), block_table.shape[-1],
                                       _dev(workspace), _dev(out), softmax_scale, _stream(stream)))


def paged_decode_attn_layer_static(pool, layer: int, q, block_table, ctx_len_dev, max_ctx_tokens: int,
                                   chunk_tokens: int, out, err_flag_dev=None, softmax_scale: float = 0.0, stream=None):
    _check(lib.paged_decode_attn_layer_static(pool, layer, _dev(q), _dev(block_table), block_table.shape[-1],
                                              _dev(ctx_len_dev), ctx_len_dev.numel(), max_ctx_tokens, chunk_tokens,
                                              _dev(out), _dev(err_flag_dev), softmax_scale, _stream(stream)))


def kv_attn_check(pool, workspace, stream=None):
    _check(lib.kv_attn_check(pool, _dev(workspace), _stream(stream)))


def kv_attn_run_layer(pool, layer: int, cursor: int, q, block_table, workspace, out,
                      softmax_scale: float = 0.0, max_inflight: int = 2, stream=None):
    """Returns (status, cursor): status VKV_OK or VKV_YIELDED."""
    cur = C.c_int32(cursor)
    st = lib.kv_attn_run_layer(pool, layer, C.byref(cur), _dev(q), _dev(block_table), block_table.shape[-1],
                               _dev(workspace), _dev(out), softmax_scale, max_inflight, _stream(stream))
    _check(st, ok=(VKV_OK, VKV_YIELDED))
    return st, cur.value


def kv_yield_request(pool):
    _check(lib.kv_yield_request(pool))


def kv_yield_clear(pool):
    _check(lib.kv_yield_clear(pool))


def kv_yield_pending(pool) -> bool:
    return bool(lib.kv_yield_pending(pool))


# ---- reclamation ------------------------------------------------------------------
def kv_reclaim_plan(pool, lo: int, hi: int, num_blocks: int):
    """Dry run.  Returns (remap int32[NB], stats)."""
    remap = np.empty(num_blocks, dtype=np.int32)
    stats = ReclaimStats()
    _check(lib.kv_reclaim_plan(pool, lo, hi, remap.ctypes.data, C.byref(stats)))
    return remap, stats


def kv_reclaim_range(pool, lo: int, hi: int, block_tables, remap_dev, chunk_bytes: int = 0,
                     rate_cap_bytes_per_s: int = 0, copy_stream=None, decode_stream=None,
                     flags: int = 0) -> ReclaimStats:
    stats = ReclaimStats()
    ds = None if decode_stream is None else _stream(decode_stream)
    _check(lib.kv_reclaim_range(pool, lo, hi, _dev(block_tables), block_tables.numel(), chunk_bytes,
                                int(rate_cap_bytes_per_s), _stream(copy_stream), ds, _dev(remap_dev), flags,
                                C.byref(stats)))
    return stats


def block_table_rewrite(block_tables, remap_dev, num_blocks: int, stream=None):
    _check(lib.block_table_rewrite(_dev(block_tables), block_tables.numel(), _dev(remap_dev), num_blocks,
                                   _stream(stream)))


# ---- per-launch timing ------------------------------------------------------------
def kv_profile_enable(pool, max_records: int):
    _check(lib.kv_profile_enable(pool, max_records))


def kv_profile_sample(pool, stride: int):
    _check(lib.kv_profile_sample(pool, stride))


def kv_profile_read(pool, cap: int) -> np.ndarray:
    """Structured array (kind, index, ms) of the launches recorded since the last read."""
    dt = np.dtype([("kind", np.int32), ("index", np.int32), ("ms", np.float32)])
    buf = np.zeros(cap, dtype=dt)
    n = C.c_int32(0)
    _check(lib.kv_profile_read(pool, buf.ctypes.data, cap, C.byref(n)))
    return buf[:n.value]


def kv_sched_set_overlap(pool, enable: bool):
    _check(lib.kv_sched_set_overlap(pool, 1 if enable else 0))


# ---- handle-backed pool memory ----------------------------------------------------
class DeviceSpan:
    """A raw device address range as an object torch can alias without copying
    (`torch.as_tensor(span, device="cuda")` gives an int16 tensor over it)."""

    def __init__(self, address: int, nbytes: int):
        self.address, self.nbytes = address, nbytes
        self.__cuda_array_interface__ = {"shape": (nbytes // 2,), "typestr": "<i2", "data": (address, False),
                                         "version": 2, "strides": None}


def kv_arena_create(device: int, handle_bytes: int, num_handles: int):
    """Returns (arena handle, DeviceSpan of the whole address range)."""
    arena, base = _P(), _P()
    _check(lib.kv_arena_create(device, handle_bytes, num_handles, C.byref(arena), C.byref(base)))
    return arena, DeviceSpan(base.value, handle_bytes * num_handles)


def kv_arena_destroy(arena):
    _check(lib.kv_arena_destroy(arena))


def kv_pool_attach_arena(pool, arena):
    _check(lib.kv_pool_attach_arena(pool, arena))


def kv_arena_release(arena, pool, lo: int, hi: int):
    _check(lib.kv_arena_release(arena, pool, lo, hi))


def kv_arena_restore(arena, pool, lo: int, hi: int):
    _check(lib.kv_arena_restore(arena, pool, lo, hi))


def kv_arena_state(arena, num_handles: int):
    """Returns (mapped uint8[num_handles], bytes currently backed)."""
    m = np.zeros(num_handles, dtype=np.uint8)
    n = C.c_uint64(0)
    _check(lib.kv_arena_state(arena, m.ctypes.data, C.byref(n)))
    return m, n.value


# ---- bandwidth yardsticks ---------------------------------------------------------
def kv_probe_read(src_dev, nbytes: int, sink_dev, stream=None):
    _check(lib.kv_probe_read(_dev(src_dev), nbytes, _dev(sink_dev), _stream(stream)))


def kv_probe_attn_reads(pool, layer: int, slice_idx: int, block_table, workspace, sink_dev, stream=None):
    _check(lib.kv_probe_attn_reads(pool, layer, slice_idx, _dev(block_table), block_table.shape[-1], _dev(workspace),
                                   _dev(sink_dev), _stream(stream)))


def kv_probe_copy(dst_dev, src_dev, nbytes: int, stream=None):
    _check(lib.kv_probe_copy(_dev(dst_dev), _dev(src_dev), nbytes, _stream(stream)))


# ---- prefill ----------------------------------------------------------------------
def kv_prefill_plan(pool, ctx_len_host, q_len_host, slice_bytes: int, chunk_tokens: int) -> PrefillPlanInfo:
    ctx = _host(ctx_len_host, np.int32)
    ql = _host(q_len_host, np.int32)
    assert len(ctx) == len(ql)
    info = PrefillPlanInfo()
    _check(lib.kv_prefill_plan(pool, ctx.ctypes.data, ql.ctypes.data, len(ctx), slice_bytes, chunk_tokens, C.byref(info)))
    return info


def kv_prefill_plan_read(pool, info: PrefillPlanInfo):
    """Returns (work [n_items,4], slice_start [n_slices+1], tiles [n_tiles,4], tile_base [n_tiles+1])."""
    work = np.empty((info.n_items, 4), dtype=np.int32)
    starts = np.empty(info.n_slices + 1, dtype=np.int32)
    tiles = np.empty((info.n_tiles, 4), dtype=np.int32)
    tile_base = np.empty(info.n_tiles + 1, dtype=np.int32)
    _check(lib.kv_prefill_plan_read(pool, work.ctypes.data, starts.ctypes.data, tiles.ctypes.data, tile_base.ctypes.data))
    return work, starts, tiles, tile_base


def kv_prefill_bind(pool, workspace, stream=None):
    _check(lib.kv_prefill_bind(pool, _dev(workspace), workspace.numel() * workspace.element_size(), _stream(stream)))


def paged_prefill_attn_slice(pool, layer: int, slice_idx: int, q, block_table, workspace, out,
                             softmax_scale: float = 0.0, stream=None):
    _check(lib.paged_prefill_attn_slice(pool, layer, slice_idx, _dev(q), _dev(block_table), block_table.shape[-1],
                                        _dev(workspace), _dev(out), softmax_scale, _stream(stream)))


def kv_prefill_merge(pool, step: int, workspace, out, stream=None):
    _check(lib.kv_prefill_merge(pool, step, _dev(workspace), _dev(out), _stream(stream)))


def kv_prefill_run_layer(pool, layer: int, cursor: int, q, block_table, workspace, out,
                         softmax_scale: float = 0.0, max_inflight: int = 2, stream=None):
    cur = C.c_int32(cursor)
    st = lib.kv_prefill_run_layer(pool, layer, C.byref(cur), _dev(q), _dev(block_table), block_table.shape[-1],
                                  _dev(workspace), _dev(out), softmax_scale, max_inflight, _stream(stream))
    _check(st, ok=(VKV_OK, VKV_YIELDED))
    return st, cur.value


def kv_prefill_check(pool, workspace, stream=None):
    _check(lib.kv_prefill_check(pool, _dev(workspace), _stream(stream)))


# ---- policies (host only) ---------------------------------------------------------
def kv_select_handles(pool, tables_host, cost_host, k: int):
    """Algorithm 1.  Returns (handles int32[k] in pick order, evicted rows int32[], total cost)."""
    t = _host(tables_host, np.int32)
    n_rows, max_blk = t.shape
    cost = _host(cost_host, np.int64)
    assert len(cost) == n_rows
    handles = np.empty(k, dtype=np.int32)
    ev = np.empty(n_rows, dtype=np.int32)
    n_ev = C.c_int32(0)
    total = C.c_int64(0)
    _check(lib.kv_select_handles(pool, t.ctypes.data, n_rows, max_blk, cost.ctypes.data, k, handles.ctypes.data,
                                 ev.ctypes.data, C.byref(n_ev), C.byref(total)))
    return handles, ev[:n_ev.value].copy(), total.value


def kv_invalidate_handles(pool, handles, tables_host, cap=None, tables_dev=None, remap_dev=None, stream=None,
                          decode_stream=None):
    """Returns (rows, columns, block ids) of the invalidated table entries, row-major order."""
    t = _host(tables_host, np.int32)
    n_rows, max_blk = t.shape
    h = _host(handles, np.int32)
    cap = t.size if cap is None else cap
    rows, cols, blks = (np.empty(cap, dtype=np.int32) for _ in range(3))
    n = C.c_int32(0)
    _check(lib.kv_invalidate_handles(pool, h.ctypes.data, len(h), t.ctypes.data, n_rows, max_blk, rows.ctypes.data,
                                     cols.ctypes.data, blks.ctypes.data, cap, C.byref(n), _dev(tables_dev),
                                     _dev(remap_dev), _stream(stream) if tables_dev is not None else None,
                                     _stream(decode_stream) if decode_stream is not None else None))
    return rows[:n.value].copy(), cols[:n.value].copy(), blks[:n.value].copy()


def kv_handles_cost(pool, tables_host, cost_host, handles):
    """Returns (rows with an entry in one of the handles, sum of their cost)."""
    t = _host(tables_host, np.int32)
    n_rows, max_blk = t.shape
    cost = _host(cost_host, np.int64)
    h = _host(handles, np.int32)
    ev = np.empty(n_rows, dtype=np.int32)
    n_ev, total = C.c_int32(0), C.c_int64(0)
    _check(lib.kv_handles_cost(pool, t.ctypes.data, n_rows, max_blk, cost.ctypes.data, h.ctypes.data, len(h),
                               ev.ctypes.data, C.byref(n_ev), C.byref(total)))
    return ev[:n_ev.value].copy(), total.value


def kv_evict_handles(pool, k: int, tables_host, cost_host, tables_dev=None, scratch_dev=None, stream=None,
                     decode_stream=None, cap=None):
    """tables_host (int32 [n_rows, max_blk], C-contiguous) is updated in place.
    Returns (info, handles, evicted rows, (rows, columns, block ids) of the invalidated entries)."""
    t = tables_host
    assert t.dtype == np.int32 and t.flags.c_contiguous and t.ndim == 2
    n_rows, max_blk = t.shape
    cost = _host(cost_host, np.int64)
    cap = t.size if cap is None else cap
    handles = np.empty(max(k, 1), dtype=np.int32)
    ev = np.empty(max(n_rows, 1), dtype=np.int32)
    rows, cols, blks = (np.empty(max(cap, 1), dtype=np.int32) for _ in range(3))
    info = EvictInfo()
    _check(lib.kv_evict_handles(pool, k, t.ctypes.data, n_rows, max_blk, cost.ctypes.data, _dev(tables_dev),
                                _dev(scratch_dev), _stream(stream) if tables_dev is not None else None,
                                _stream(decode_stream) if decode_stream is not None else None,
                                handles.ctypes.data, ev.ctypes.data, rows.ctypes.data, cols.ctypes.data, blks.ctypes.data,
                                cap, C.byref(info)))
    n = info.n_invalidated
    return info, handles[:k].copy(), ev[:info.n_evicted].copy(), (rows[:n].copy(), cols[:n].copy(), blks[:n].copy())


def kv_reclaim_or_evict(pool, lo: int, hi: int, tables_dev, tables_host, cost_host, remap_dev, chunk_bytes: int = 0,
                        rate_cap_bytes_per_s: int = 0, copy_stream=None, decode_stream=None, flags: int = 0, cap=None):
    """Returns (info, stats, handles, evicted rows, invalidated entries); tables_host is updated in place."""
    t = tables_host
    assert t.dtype == np.int32 and t.flags.c_contiguous and t.ndim == 2
    n_rows, max_blk = t.shape
    cost = _host(cost_host, np.int64)
    cap = t.size if cap is None else cap
    k = max(1, hi - lo)
    handles = np.empty(k, dtype=np.int32)
    ev = np.empty(max(n_rows, 1), dtype=np.int32)
    rows, cols, blks = (np.empty(max(cap, 1), dtype=np.int32) for _ in range(3))
    info, stats = EvictInfo(), ReclaimStats()
    ds = None if decode_stream is None else _stream(decode_stream)
    _check(lib.kv_reclaim_or_evict(pool, lo, hi, _dev(tables_dev), t.ctypes.data, n_rows, max_blk, cost.ctypes.data,
                                   chunk_bytes, int(rate_cap_bytes_per_s), _stream(copy_stream), ds, _dev(remap_dev), flags,
                                   handles.ctypes.data, ev.ctypes.data, rows.ctypes.data, cols.ctypes.data,
                                   blks.ctypes.data, cap, C.byref(info), C.byref(stats)))
    n = info.n_invalidated
    return (info, stats, handles[:info.n_handles].copy(), ev[:info.n_evicted].copy(),
            (rows[:n].copy(), cols[:n].copy(), blks[:n].copy()))


def kv_miad_init(**kw):
    cfg = MiadConfig(reserved=0, **kw)
    out = _P()
    _check(lib.kv_miad_init(C.byref(cfg), C.byref(out)))
    return out


def kv_miad_destroy(m):
    _check(lib.kv_miad_destroy(m))


def kv_miad_observe(m, now_s: float, used_handles: int):
    """Returns (headroom, grow_by, release, pressure_event, interval_s)."""
    st = MiadStep()
    _check(lib.kv_miad_observe(m, now_s, used_handles, C.byref(st)))
    return st.headroom, st.grow_by, st.release, st.pressure_event, st.interval_s


def kv_gate_init(initial_gap_s: float):
    out = _P()
    _check(lib.kv_gate_init(initial_gap_s, C.byref(out)))
    return out


def kv_gate_destroy(g):
    _check(lib.kv_gate_destroy(g))


def kv_gate_online_busy(g, now_s: float, request_id: int) -> int:
    return _check(lib.kv_gate_online_busy(g, now_s, request_id), ok=(0, 1))


def kv_gate_online_idle(g, now_s: float):
    _check(lib.kv_gate_online_idle(g, now_s))


def kv_gate_poll(g, now_s: float) -> int:
    return _check(lib.kv_gate_poll(g, now_s), ok=(0, 1))


def kv_gate_stats(g):
    gap, n = C.c_double(0), C.c_int64(0)
    _check(lib.kv_gate_stats(g, C.byref(gap), C.byref(n)))
    return gap.value, n.value
