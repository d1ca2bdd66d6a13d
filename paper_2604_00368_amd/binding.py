"""Thin ctypes binding over the engine's C ABI (include/tent.h).

Argument marshalling only: every function forwards to the entry point of the same
name in ``csrc/libtent.so``.  There is no fallback: if the library has not been built
(``python -m paper_2604_00368_amd.build``) loading raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from .workloads import DISPATCH_PARAMS_DTYPE, EXTENT_DTYPE, MONITOR_PARAMS_DTYPE, PROBE_DTYPE, RAIL_DTYPE

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "csrc", "libtent.so")

TENT_OK, TENT_DEFER = 0, 1
TENT_ERR_INVALID, TENT_ERR_RANGE, TENT_ERR_STATE, TENT_ERR_NOMEM, TENT_ERR_HIP = -1, -2, -3, -4, -5
TENT_MAX_RAILS = 64
TENT_STATIC_WORKSPACE_BYTES = 64 << 20
TENT_FLAG_SKIP_OVERLAP_CHECK, TENT_FLAG_PROFILE, TENT_FLAG_SERIAL_BINDING, TENT_FLAG_BOUNDED_STAGING = 1, 2, 4, 8
TENT_SLICE_PENDING, TENT_SLICE_BOUND, TENT_SLICE_DONE = 0, 1, 2
TENT_T_NAMES = ["extent_scan", "slice_scan", "expand", "compact", "bind", "gather", "scatter", "feedback"]

EXPORTS = ["tent_create", "tent_destroy", "tent_register_segment", "tent_declare", "tent_plan",
           "tent_sim_advance", "tent_sim_latency", "tent_update_bandwidth", "tent_get_latencies", "tent_execute", "tent_poll", "tent_reset", "tent_slice_count",
           "tent_get_plan", "tent_get_timings", "tent_release", "tent_strerror",
           "tent_sim_fail", "tent_get_retries", "tent_monitor_init", "tent_monitor_update",
           "tent_plan_dispatch", "tent_get_modes", "tent_execute_bounded", "tent_probe_copy", "tent_declare_static"]


class tent_config(C.Structure):
    _fields_ = [("slice_bytes", C.c_uint64), ("staging_arena", C.c_void_p), ("staging_bytes", C.c_uint64),
                ("flags", C.c_uint32), ("max_rails", C.c_uint32)]


class tent_plan_info(C.Structure):
    _fields_ = [("n_slices", C.c_uint64), ("n_pending_before", C.c_uint64),
                ("rail_bytes", C.c_uint64 * TENT_MAX_RAILS), ("rail_slices", C.c_uint64 * TENT_MAX_RAILS),
                ("queued_after", C.c_uint64 * TENT_MAX_RAILS), ("stage_base", C.c_uint64 * TENT_MAX_RAILS)]


class tent_dispatch_info(C.Structure):
    _fields_ = [("plan", tent_plan_info), ("n_mice", C.c_uint64), ("n_elephant", C.c_uint64),
                ("n_deferred", C.c_uint64), ("rr_next", C.c_uint64)]


MONITOR_DTYPE = np.dtype([("state", "<u4"), ("score", "<u4"), ("clean", "<u4"),
                          ("cooldown_left", "<u4"), ("cooldown_next", "<u4")])

SLICE_DTYPE = np.dtype(
    {"names": ["desc", "len", "off", "stage_off", "rail", "state"],
     "formats": ["<u4", "<u4", "<u8", "<u8", "<u4", "<u4"],
     "offsets": [0, 4, 8, 16, 24, 28], "itemsize": 32})


class TentError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: {tent_strerror(status)} ({status})")


_lib = None


def lib():
    """Load libtent.so; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2604_00368_amd.build`")
        L = C.CDLL(LIB_PATH)
        L.tent_strerror.restype = C.c_char_p
        L.tent_strerror.argtypes = [C.c_int]
        for name in EXPORTS:
            if name != "tent_strerror":
                getattr(L, name).restype = C.c_int
        L.tent_create.argtypes = [C.POINTER(C.c_void_p), C.POINTER(tent_config)]
        L.tent_destroy.argtypes = [C.c_void_p]
        L.tent_register_segment.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64, C.POINTER(C.c_uint32)]
        L.tent_declare.argtypes = [C.c_void_p, C.c_uint32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                   C.POINTER(C.c_uint64)]
        L.tent_declare_static.argtypes = L.tent_declare.argtypes
        L.tent_plan.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p, C.c_uint32, C.POINTER(tent_plan_info),
                                C.c_void_p]
        L.tent_sim_advance.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p, C.POINTER(C.c_uint64), C.c_void_p]
        L.tent_sim_latency.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p, C.c_void_p]
        L.tent_update_bandwidth.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p, C.c_void_p, C.c_uint32, C.c_void_p,
                                            C.c_void_p]
        L.tent_get_latencies.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p, C.c_uint64]
        L.tent_execute.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p]
        L.tent_execute_bounded.argtypes = [C.c_void_p, C.c_uint64, C.c_uint64, C.c_uint32, C.c_void_p]
        L.tent_poll.argtypes = [C.c_void_p, C.c_uint64, C.POINTER(C.c_uint64), C.c_void_p]
        L.tent_reset.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p]
        L.tent_slice_count.argtypes = [C.c_void_p, C.c_uint64, C.POINTER(C.c_uint64)]
        L.tent_get_plan.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p, C.c_uint64]
        L.tent_get_timings.argtypes = [C.c_void_p, C.POINTER(C.c_float), C.POINTER(C.c_uint32)]
        L.tent_release.argtypes = [C.c_void_p, C.c_uint64]
        L.tent_probe_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64, C.c_uint32, C.c_uint32, C.c_void_p,
                                      C.POINTER(C.c_float)]
        L.tent_plan_dispatch.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p, C.c_uint32, C.c_void_p, C.c_void_p,
                                         C.POINTER(tent_dispatch_info), C.c_void_p]
        L.tent_get_modes.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p, C.c_uint64]
        L.tent_sim_fail.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p]
        L.tent_get_retries.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p, C.c_uint64]
        L.tent_monitor_init.argtypes = [C.c_void_p, C.c_void_p, C.c_uint32]
        L.tent_monitor_update.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32, C.c_void_p, C.c_void_p,
                                          C.c_void_p, C.c_void_p]
        _lib = L
    return _lib


def _check(status, where, allow=(TENT_OK,)):
    if status not in allow:
        raise TentError(status, where)
    return status


def _host(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a, a.ctypes.data_as(C.c_void_p)


def _stream(stream):
    if stream is None:
        return None
    return C.c_void_p(int(getattr(stream, "cuda_stream", stream)))


def tent_strerror(status: int) -> str:
    return lib().tent_strerror(int(status)).decode()


def tent_create(slice_bytes: int, staging_arena_ptr: int, staging_bytes: int, flags: int = 0, max_rails: int = 0):
    cfg = tent_config(slice_bytes, staging_arena_ptr, staging_bytes, flags, max_rails)
    ctx = C.c_void_p()
    _check(lib().tent_create(C.byref(ctx), C.byref(cfg)), "tent_create")
    return ctx


def tent_destroy(ctx):
    _check(lib().tent_destroy(ctx), "tent_destroy")


def tent_register_segment(ctx, dev_ptr: int, nbytes: int) -> int:
    seg = C.c_uint32()
    _check(lib().tent_register_segment(ctx, C.c_void_p(dev_ptr), nbytes, C.byref(seg)), "tent_register_segment")
    return seg.value


def tent_declare(ctx, src_ptr, src_ext, dst_ptr, dst_ext) -> int:
    sp, spp = _host(src_ptr, np.uint32)
    dp, dpp = _host(dst_ptr, np.uint32)
    se, sep = _host(src_ext, EXTENT_DTYPE)
    de, dep = _host(dst_ext, EXTENT_DTYPE)
    h = C.c_uint64()
    _check(lib().tent_declare(ctx, sp.shape[0] - 1, spp, sep, dpp, dep, C.byref(h)), "tent_declare")
    return h.value


def tent_declare_static(ctx, src_ptr, src_ext, dst_ptr, dst_ext) -> int:
    sp, spp = _host(src_ptr, np.uint32)
    dp, dpp = _host(dst_ptr, np.uint32)
    se, sep = _host(src_ext, EXTENT_DTYPE)
    de, dep = _host(dst_ext, EXTENT_DTYPE)
    h = C.c_uint64()
    _check(lib().tent_declare_static(ctx, sp.shape[0] - 1, spp, sep, dpp, dep, C.byref(h)), "tent_declare_static")
    return h.value


def tent_plan(ctx, batch: int, rails, want_info: bool = True, stream=None):
    """Returns (status, info) with status TENT_OK or TENT_DEFER; info is None when not requested."""
    r, rp = _host(rails, RAIL_DTYPE)
    info = tent_plan_info() if want_info else None
    st = lib().tent_plan(ctx, batch, rp, r.shape[0], C.byref(info) if want_info else None, _stream(stream))
    _check(st, "tent_plan", allow=(TENT_OK, TENT_DEFER))
    return st, info


def tent_sim_advance(ctx, batch: int, budget_bytes, stream=None, want_done: bool = True):
    """Returns the number of slices that stayed BOUND, or None (and only enqueues) when it is not asked for."""
    b, bp = _host(budget_bytes, np.uint64)
    if not want_done:
        _check(lib().tent_sim_advance(ctx, batch, bp, None, _stream(stream)), "tent_sim_advance")
        return None
    n = C.c_uint64()
    _check(lib().tent_sim_advance(ctx, batch, bp, C.byref(n), _stream(stream)), "tent_sim_advance")
    return n.value


def tent_plan_dispatch(ctx, batch: int, rails, params, priority=None, want_info: bool = True, stream=None):
    """Returns (status, info) with status TENT_OK or TENT_DEFER; info is None when not requested."""
    r, rp = _host(rails, RAIL_DTYPE)
    p, pp = _host(params, DISPATCH_PARAMS_DTYPE)
    pr = None if priority is None else np.ascontiguousarray(priority, dtype=np.uint8)
    info = tent_dispatch_info() if want_info else None
    st = lib().tent_plan_dispatch(ctx, batch, rp, r.shape[0], pp, None if pr is None else pr.ctypes.data_as(C.c_void_p),
                                  C.byref(info) if want_info else None, _stream(stream))
    _check(st, "tent_plan_dispatch", allow=(TENT_OK, TENT_DEFER))
    return st, info


def tent_get_modes(ctx, batch: int, n_desc: int) -> np.ndarray:
    out = np.zeros(max(n_desc, 1), dtype=np.uint8)
    _check(lib().tent_get_modes(ctx, batch, out.ctypes.data_as(C.c_void_p), n_desc), "tent_get_modes")
    return out[:n_desc]


def tent_sim_fail(ctx, batch: int, rail_failed, want_counts: bool = True, stream=None):
    """Returns the number of slices that failed per rail (None when not requested)."""
    f, fp = _host(rail_failed, np.uint8)
    out = np.zeros(f.shape[0], dtype=np.uint64) if want_counts else None
    _check(lib().tent_sim_fail(ctx, batch, fp, out.ctypes.data_as(C.c_void_p) if want_counts else None,
                               _stream(stream)), "tent_sim_fail")
    return out


def tent_get_retries(ctx, batch: int) -> np.ndarray:
    n = tent_slice_count(ctx, batch)
    out = np.zeros(max(n, 1), dtype=np.uint8)
    _check(lib().tent_get_retries(ctx, batch, out.ctypes.data_as(C.c_void_p), n), "tent_get_retries")
    return out[:n]


def tent_monitor_init(params, n_rails: int) -> np.ndarray:
    p, pp = _host(params, MONITOR_PARAMS_DTYPE)
    mon = np.zeros(n_rails, dtype=MONITOR_DTYPE)
    _check(lib().tent_monitor_init(pp, mon.ctypes.data_as(C.c_void_p), n_rails), "tent_monitor_init")
    return mon


def tent_monitor_update(params, mon, rails, hard_errors, congestion_errors, probe_MBps, bw_before_MBps):
    """Advances `mon` in place by one window; returns the rails with their health fields updated."""
    p, pp = _host(params, MONITOR_PARAMS_DTYPE)
    r = np.ascontiguousarray(rails, dtype=RAIL_DTYPE).copy()
    h, hp = _host(hard_errors, np.uint32)
    c, cp = _host(congestion_errors, np.uint32)
    pr, prp = _host(probe_MBps, np.uint32)
    bw, bwp = _host(bw_before_MBps, np.uint32)
    assert mon.dtype == MONITOR_DTYPE and mon.flags["C_CONTIGUOUS"]
    _check(lib().tent_monitor_update(pp, mon.ctypes.data_as(C.c_void_p), r.ctypes.data_as(C.c_void_p), r.shape[0],
                                     hp, cp, prp, bwp), "tent_monitor_update")
    return r


def tent_sim_latency(ctx, batch: int, true_bw_MBps, stream=None):
    b, bp = _host(true_bw_MBps, np.uint32)
    _check(lib().tent_sim_latency(ctx, batch, bp, _stream(stream)), "tent_sim_latency")


def tent_update_bandwidth(ctx, batch: int, params, rails, stream=None):
    """Returns (rails with updated bw_MBps, probe_MBps); the input arrays are not modified."""
    p, pp = _host(params, PROBE_DTYPE)
    r = np.ascontiguousarray(rails, dtype=RAIL_DTYPE).copy()
    probe = np.zeros(r.shape[0], dtype=np.uint32)
    _check(lib().tent_update_bandwidth(ctx, batch, pp, r.ctypes.data_as(C.c_void_p), r.shape[0],
                                       probe.ctypes.data_as(C.c_void_p), _stream(stream)), "tent_update_bandwidth")
    return r, probe


def tent_get_latencies(ctx, batch: int) -> np.ndarray:
    n = tent_slice_count(ctx, batch)
    out = np.zeros(n, dtype=np.uint64)
    _check(lib().tent_get_latencies(ctx, batch, out.ctypes.data_as(C.c_void_p), n), "tent_get_latencies")
    return out


def tent_execute(ctx, batch: int, stream=None):
    _check(lib().tent_execute(ctx, batch, _stream(stream)), "tent_execute")


def tent_execute_bounded(ctx, batch: int, chunk_bytes: int, stream=None, slots: int = 1):
    _check(lib().tent_execute_bounded(ctx, batch, chunk_bytes, slots, _stream(stream)), "tent_execute_bounded")


def tent_poll(ctx, batch: int, stream=None) -> int:
    n = C.c_uint64()
    _check(lib().tent_poll(ctx, batch, C.byref(n), _stream(stream)), "tent_poll")
    return n.value


def tent_reset(ctx, batch: int, stream=None):
    _check(lib().tent_reset(ctx, batch, _stream(stream)), "tent_reset")


def tent_slice_count(ctx, batch: int) -> int:
    n = C.c_uint64()
    _check(lib().tent_slice_count(ctx, batch, C.byref(n)), "tent_slice_count")
    return n.value


def tent_get_plan(ctx, batch: int) -> np.ndarray:
    n = tent_slice_count(ctx, batch)
    out = np.zeros(n, dtype=SLICE_DTYPE)
    _check(lib().tent_get_plan(ctx, batch, out.ctypes.data_as(C.c_void_p), n), "tent_get_plan")
    return out


def tent_get_timings(ctx) -> dict:
    """{stage: (total_ms, intervals)} since the previous call."""
    ms = (C.c_float * len(TENT_T_NAMES))()
    cnt = (C.c_uint32 * len(TENT_T_NAMES))()
    _check(lib().tent_get_timings(ctx, ms, cnt), "tent_get_timings")
    return {k: (float(ms[i]), int(cnt[i])) for i, k in enumerate(TENT_T_NAMES)}


def tent_probe_copy(read_window: int, write_window: int, nbytes: int, page_bytes: int = 32768, repeats: int = 2,
                    stream=None) -> float:
    """Shortest of `repeats` timed probe copies (ms) from one device window to another."""
    ms = C.c_float(0)
    _check(lib().tent_probe_copy(C.c_void_p(read_window), C.c_void_p(write_window), nbytes, page_bytes, repeats,
                                 _stream(stream), C.byref(ms)), "tent_probe_copy")
    return float(ms.value)


def tent_release(ctx, batch: int):
    _check(lib().tent_release(ctx, batch), "tent_release")
