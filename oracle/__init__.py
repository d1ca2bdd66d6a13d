"""TEST INFRASTRUCTURE: ctypes front end of the sequential CPU oracle (tent_oracle.c).

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this package.  It shares nothing with the HIP engine; inputs are the plain
numpy arrays produced by the workload generator.

Every function is a thin call into the C file; the comments there cite the
passages of the paper each step follows.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liboracle.so")
_SRC_PATH = os.path.join(_HERE, "tent_oracle.c")

OK, DEFER = 0, 1


def build(force: bool = False) -> str:
    """Compile tent_oracle.c with gcc (plain -O2, no vectorisation flags beyond the default)."""
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(_SRC_PATH):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-fPIC", "-shared",
                               "-o", _LIB_PATH, _SRC_PATH])
    return _LIB_PATH


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB_PATH)
        L.ora_count_slices.restype = C.c_uint64
        L.ora_cost.restype = C.c_uint64
        L.ora_cost.argtypes = [C.c_uint64] * 4
        L.ora_bind.restype = C.c_int
        L.ora_retire.restype = C.c_uint64
        L.ora_split.restype = None
        L.ora_coeffs.restype = None
        L.ora_stage_bases.restype = None
        L.ora_execute.restype = None
        L.ora_sim_latency.restype = None
        L.ora_probe.restype = None
        L.ora_fail.restype = C.c_uint64
        L.ora_rotation_candidates.restype = C.c_uint32
        L.ora_plan.restype = C.c_int
        L.ora_monitor_init.restype = None
        L.ora_monitor_step.restype = None
        L.ora_dispatch.restype = C.c_int
        L.ora_execute_bounded.restype = C.c_int
        _lib = L
    return _lib


def _p(a: Optional[np.ndarray]):
    if a is None:
        return None
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(C.c_void_p)


@dataclass
class Slices:
    first: np.ndarray      # uint64[D+1]
    desc: np.ndarray       # uint32[N]
    off: np.ndarray        # uint64[N]
    len: np.ndarray        # uint32[N]

    @property
    def n(self) -> int:
        return int(self.desc.shape[0])


@dataclass
class Binding:
    status: int
    rail: np.ndarray       # uint32[N]   (only entries of bound ids are meaningful)
    stage_off: np.ndarray  # uint64[N]
    T: np.ndarray          # uint64[R]   bytes bound per rail in this call
    n_slices: np.ndarray   # uint64[R]
    A_after: np.ndarray    # uint64[R]   queued bytes after this call
    base: np.ndarray       # uint64[R]   staging region bases


def split(src_ptr, src_ext, slice_bytes: int) -> Slices:
    L = lib()
    D = src_ptr.shape[0] - 1
    first = np.zeros(D + 1, dtype=np.uint64)
    n = L.ora_count_slices(C.c_uint32(D), _p(src_ptr), _p(src_ext), C.c_uint64(slice_bytes), _p(first))
    desc = np.zeros(n, dtype=np.uint32)
    off = np.zeros(n, dtype=np.uint64)
    ln = np.zeros(n, dtype=np.uint32)
    L.ora_split(C.c_uint32(D), _p(src_ptr), _p(src_ext), C.c_uint64(slice_bytes), _p(desc), _p(off), _p(ln))
    return Slices(first, desc, off, ln)


def coeffs(rails):
    L = lib()
    R = rails.shape[0]
    c0 = np.zeros(R, dtype=np.uint64)
    c1 = np.zeros(R, dtype=np.uint64)
    ex = np.zeros(R, dtype=np.uint8)
    A = np.zeros(R, dtype=np.uint64)
    L.ora_coeffs(_p(np.ascontiguousarray(rails)), C.c_uint32(R), _p(c0), _p(c1), _p(ex), _p(A))
    return c0, c1, ex, A


def cost(c0: int, c1: int, A: int, Lbytes: int) -> int:
    return int(lib().ora_cost(c0, c1, A, Lbytes))


def bind(slice_len, rails, ids=None, rail=None, stage_off=None) -> Binding:
    """Bind slices (all, or those listed in ids) under the given telemetry."""
    L = lib()
    R = rails.shape[0]
    N = slice_len.shape[0]
    c0, c1, ex, A = coeffs(rails)
    T = np.zeros(R, dtype=np.uint64)
    cnt = np.zeros(R, dtype=np.uint64)
    if rail is None:
        rail = np.full(N, 0xFFFFFFFF, dtype=np.uint32)
    if stage_off is None:
        stage_off = np.zeros(N, dtype=np.uint64)
    n = N if ids is None else ids.shape[0]
    st = L.ora_bind(C.c_uint64(n), _p(ids), _p(slice_len), C.c_uint32(R), _p(c0), _p(c1), _p(ex),
                    _p(A), _p(T), _p(cnt), _p(rail), _p(stage_off))
    base = np.zeros(R, dtype=np.uint64)
    L.ora_stage_bases(_p(T), C.c_uint32(R), _p(base))
    return Binding(int(st), rail, stage_off, T, cnt, A, base)


def fail(b: Binding, rail_failed, retry, ids=None):
    """Hard errors on the rails flagged in rail_failed: the listed slices bound to them get one
    more retry (retry is updated in place).  Returns (failed flags per listed slice, count per rail)."""
    L = lib()
    R = len(rail_failed)
    n = b.rail.shape[0] if ids is None else ids.shape[0]
    failed = np.zeros(n, dtype=np.uint8)
    per_rail = np.zeros(R, dtype=np.uint64)
    L.ora_fail(C.c_uint64(n), _p(ids), _p(b.rail), C.c_uint32(R),
               _p(np.ascontiguousarray(rail_failed, dtype=np.uint8)), _p(retry), _p(failed), _p(per_rail))
    return failed, per_rail


def rotation_candidates(rails) -> np.ndarray:
    cand = np.zeros(64, dtype=np.uint32)
    n = lib().ora_rotation_candidates(_p(np.ascontiguousarray(rails)), C.c_uint32(rails.shape[0]), _p(cand))
    return cand[:n].copy()


def plan(slice_len, retry, rails, ids=None, rail=None, stage_off=None) -> Binding:
    """Plan with retried slices: rotation for retry counts > 0, predicted cost for the rest."""
    L = lib()
    R = rails.shape[0]
    N = slice_len.shape[0]
    c0, c1, ex, A = coeffs(rails)
    T = np.zeros(R, dtype=np.uint64)
    cnt = np.zeros(R, dtype=np.uint64)
    if rail is None:
        rail = np.full(N, 0xFFFFFFFF, dtype=np.uint32)
    if stage_off is None:
        stage_off = np.zeros(N, dtype=np.uint64)
    n = N if ids is None else ids.shape[0]
    st = L.ora_plan(C.c_uint64(n), _p(ids), _p(slice_len), _p(retry), _p(np.ascontiguousarray(rails)),
                    C.c_uint32(R), _p(c0), _p(c1), _p(ex), _p(A), _p(T), _p(cnt), _p(rail), _p(stage_off))
    base = np.zeros(R, dtype=np.uint64)
    L.ora_stage_bases(_p(T), C.c_uint32(R), _p(base))
    return Binding(int(st), rail, stage_off, T, cnt, A, base)


DISPATCH_PARAMS_DTYPE = np.dtype([("theta_bytes", "<u8"), ("gamma_q8", "<u4"), ("window", "<u4"), ("rr_start", "<u8")])


@dataclass
class Dispatch:
    binding: Binding
    bound: np.ndarray      # uint8[N]  slices dealt by this call
    mode: np.ndarray       # uint8[D]  0 nothing pending, 1 mice, 2 elephant, 3 deferred
    rr_end: int            # round-robin counter after the call


def dispatch(s: Slices, rails, dp, priority=None, done=None, rail=None, stage_off=None) -> Dispatch:
    """Algorithm 1 per request: QoS admission, mice / elephant dispatch (see tent_oracle.c)."""
    L = lib()
    R = rails.shape[0]
    D = s.first.shape[0] - 1
    c0, c1, ex, A = coeffs(rails)
    T = np.zeros(R, dtype=np.uint64)
    cnt = np.zeros(R, dtype=np.uint64)
    if rail is None:
        rail = np.full(s.n, 0xFFFFFFFF, dtype=np.uint32)
    if stage_off is None:
        stage_off = np.zeros(s.n, dtype=np.uint64)
    if done is None:
        done = np.zeros(s.n, dtype=np.uint8)
    req_len = np.zeros(D, dtype=np.uint64)
    np.add.at(req_len, s.desc, s.len.astype(np.uint64))
    bound = np.zeros(s.n, dtype=np.uint8)
    mode = np.zeros(D, dtype=np.uint8)
    rr_end = C.c_uint64()
    st = L.ora_dispatch(C.c_uint32(D), _p(s.first), _p(s.len), _p(np.ascontiguousarray(done, dtype=np.uint8)),
                        _p(req_len), _p(None if priority is None else np.ascontiguousarray(priority, dtype=np.uint8)),
                        C.c_uint32(R), _p(c0), _p(c1), _p(ex), _p(np.ascontiguousarray(dp)),
                        _p(A), _p(T), _p(cnt), _p(rail), _p(stage_off), _p(bound), _p(mode), C.byref(rr_end))
    base = np.zeros(R, dtype=np.uint64)
    L.ora_stage_bases(_p(T), C.c_uint32(R), _p(base))
    return Dispatch(Binding(int(st), rail, stage_off, T, cnt, A, base), bound, mode, int(rr_end.value))


MONITOR_PARAMS_DTYPE = np.dtype([("err_threshold", "<u4"), ("recover_windows", "<u4"),
                                 ("cooldown_windows", "<u4"), ("degrade_q8", "<u4")])
MONITOR_DTYPE = np.dtype([("state", "<u4"), ("score", "<u4"), ("clean", "<u4"),
                          ("cooldown_left", "<u4"), ("cooldown_next", "<u4")])


def monitor_init(R: int, mp) -> np.ndarray:
    mon = np.zeros(R, dtype=MONITOR_DTYPE)
    lib().ora_monitor_init(C.c_uint32(R), _p(np.ascontiguousarray(mp)), _p(mon))
    return mon


def monitor_step(mp, mon, hard, congestion, probe_MBps, bw_MBps) -> None:
    """One measurement window of the rail health monitor; mon is updated in place."""
    R = mon.shape[0]
    lib().ora_monitor_step(C.c_uint32(R), _p(np.ascontiguousarray(mp)), _p(mon),
                           _p(np.ascontiguousarray(hard, dtype=np.uint32)),
                           _p(np.ascontiguousarray(congestion, dtype=np.uint32)),
                           _p(np.ascontiguousarray(probe_MBps, dtype=np.uint32)),
                           _p(np.ascontiguousarray(bw_MBps, dtype=np.uint32)))


def execute(w, s: Slices, b: Binding, pools, staging: np.ndarray, ids=None) -> None:
    """Move the listed slices: paged source -> per-rail staging -> destination."""
    L = lib()
    n = s.n if ids is None else ids.shape[0]
    seg = (C.c_void_p * len(pools))(*[p.ctypes.data for p in pools])
    L.ora_execute(C.c_uint64(n), _p(ids), _p(s.desc), _p(s.off), _p(s.len), _p(b.rail), _p(b.stage_off),
                  _p(b.base), _p(w.src_ptr), _p(w.src_ext), _p(w.dst_ptr), _p(w.dst_ext), seg, _p(staging))


def execute_bounded(w, s: Slices, b: Binding, pools, staging: np.ndarray, chunk_bytes: int, ids=None,
                    slots: int = 1, slot_bytes: Optional[int] = None) -> int:
    """Move the listed slices chunk by chunk through a staging buffer of fixed size (see tent_oracle.c).
    Returns 0, or -1 if some chunk does not fit the buffer (then nothing has moved)."""
    L = lib()
    n = s.n if ids is None else ids.shape[0]
    seg = (C.c_void_p * len(pools))(*[p.ctypes.data for p in pools])
    P = np.concatenate([[0], np.cumsum(s.len.astype(np.uint64))]).astype(np.uint64)
    return int(L.ora_execute_bounded(C.c_uint64(s.n), C.c_uint64(n), _p(ids), _p(s.desc), _p(s.off),
                                     _p(b.rail), _p(b.stage_off), C.c_uint32(b.T.shape[0]),
                                     _p(w.src_ptr), _p(w.src_ext), _p(w.dst_ptr), _p(w.dst_ext), seg, _p(staging),
                                     C.c_uint64(staging.shape[0]), C.c_uint64(chunk_bytes), C.c_uint32(slots),
                                     C.c_uint64(staging.shape[0] if slot_bytes is None else slot_bytes), _p(P)))


def retire(s: Slices, b: Binding, queued, budget, ids=None) -> np.ndarray:
    L = lib()
    n = s.n if ids is None else ids.shape[0]
    done = np.zeros(n, dtype=np.uint8)
    L.ora_retire(C.c_uint64(n), _p(ids), _p(s.len), _p(b.rail), _p(b.stage_off),
                 _p(np.ascontiguousarray(queued, dtype=np.uint64)),
                 _p(np.ascontiguousarray(budget, dtype=np.uint64)), _p(done))
    return done


def sim_latency(s: Slices, b: Binding, rails, true_bw_MBps, ids=None, tau=None) -> np.ndarray:
    """Simulated end-to-end latency (ns) of the listed slices; entries of other slices are left alone."""
    L = lib()
    n = s.n if ids is None else ids.shape[0]
    if tau is None:
        tau = np.zeros(s.n, dtype=np.uint64)
    L.ora_sim_latency(C.c_uint64(n), _p(ids), _p(s.len), _p(b.rail), _p(b.stage_off),
                      _p(np.ascontiguousarray(rails["queued_bytes"], dtype=np.uint64)),
                      _p(np.ascontiguousarray(rails["lat_ns"], dtype=np.uint32)),
                      _p(np.ascontiguousarray(true_bw_MBps, dtype=np.uint32)), _p(tau))
    return tau


def probe(s: Slices, b: Binding, tau, params, bw_MBps, ids=None):
    """Eq. 2 peak picking over the listed slices and the smoothed update; returns (new estimates, probes)."""
    L = lib()
    n = s.n if ids is None else ids.shape[0]
    bw = np.ascontiguousarray(bw_MBps, dtype=np.uint32).copy()
    out = np.zeros(bw.shape[0], dtype=np.uint32)
    L.ora_probe(C.c_uint64(n), _p(ids), _p(s.len), _p(b.rail), _p(tau), C.c_uint32(bw.shape[0]),
                _p(np.ascontiguousarray(params)), _p(bw), _p(out))
    return bw, out


def run_epochs_closed_loop(w, s: Slices, params, pools=None, staging=None):
    """Re-planning with the telemetry loop closed: the planner's bandwidth estimates start at the
    nominal values and follow the probes of the slices that completed in each epoch; the epochs'
    own bandwidths act as the rails' true bandwidths (budgets and simulated latencies)."""
    pending = np.arange(s.n, dtype=np.uint32)
    est = w.rails["bw_MBps"].astype(np.uint32).copy()
    records = []
    for ep in list(w.epochs) + [w.drain]:
        rails = ep.rails.copy()
        rails["bw_MBps"] = est
        rec = dict(pending=pending, est=est.copy(), rails=rails, status=OK, rail=None, stage_off=None,
                   done_ids=pending[:0], probe=None, est_after=est.copy(), tau=None)
        if pending.shape[0]:
            b = bind(s.len, rails, ids=pending)
            rec["status"] = b.status
            if b.status == OK:
                done = retire(s, b, rails["queued_bytes"], ep.budget, ids=pending).astype(bool)
                done_ids = np.ascontiguousarray(pending[done])
                tau = sim_latency(s, b, rails, ep.rails["bw_MBps"], ids=done_ids)
                est, pr = probe(s, b, tau, params, est, ids=done_ids)
                if pools is not None and done_ids.shape[0]:
                    execute(w, s, b, pools, staging, ids=done_ids)
                rec.update(rail=b.rail[pending].copy(), stage_off=b.stage_off[pending].copy(), done_ids=done_ids,
                           probe=pr, est_after=est.copy(), tau=tau[done_ids].copy(), T=b.T, base=b.base)
                pending = np.ascontiguousarray(pending[~done])
        records.append(rec)
    return records, pending


def run_epochs_resilient(w, s: Slices, params, mp, rail_fails, congestion, pools=None, staging=None, max_passes=64):
    """Re-planning with the telemetry loop closed and hard errors injected (Section 4.3).  Per window:
    plan (rotation for retried slices, predicted cost for the rest) under the monitor's health states,
    fail the slices on the rails that report a hard error, retire what the budgets allow, probe, move
    the completed slices, step the health monitor.  rail_fails[e] / congestion[e] give the failing
    rails and congestion-error counts of window e (none after the listed windows); after the
    workload's epochs the drain telemetry repeats until nothing is pending."""
    R = w.rails.shape[0]
    pending = np.arange(s.n, dtype=np.uint32)
    retry = np.zeros(s.n, dtype=np.uint8)
    est = w.rails["bw_MBps"].astype(np.uint32).copy()
    mon = monitor_init(R, mp)
    records = []
    e = 0
    while e < len(w.epochs) or pending.shape[0]:
        assert e < len(w.epochs) + max_passes, "the workload does not drain"
        ep = w.epochs[e] if e < len(w.epochs) else w.drain
        fails = rail_fails[e] if e < len(rail_fails) else np.zeros(R, dtype=np.uint8)
        cong = congestion[e] if e < len(congestion) else np.zeros(R, dtype=np.uint32)
        rails = ep.rails.copy()
        rails["bw_MBps"] = est
        rails["health"] = np.where(ep.rails["health"] == 2, 2, mon["state"]).astype(np.uint8)
        rec = dict(pending=pending, rails=rails, retry=retry.copy(), status=OK, rail=None, stage_off=None,
                   failed_per_rail=np.zeros(R, dtype=np.uint64), done_ids=pending[:0], probe=np.zeros(R, dtype=np.uint32),
                   T=None, base=None, tau=None)
        est_before = est.copy()
        hard = np.zeros(R, dtype=np.uint32)
        b = plan(s.len, retry, rails, ids=pending) if pending.shape[0] else None
        if b is not None:
            rec["status"] = b.status
        if b is not None and b.status == OK:
            failed, per_rail = fail(b, fails, retry, ids=pending)
            hard = np.minimum(per_rail, 0xFFFFFFFF).astype(np.uint32)
            live = np.ascontiguousarray(pending[failed == 0])
            done = retire(s, b, rails["queued_bytes"], ep.budget, ids=live).astype(bool)
            done_ids = np.ascontiguousarray(live[done])
            tau = sim_latency(s, b, rails, ep.rails["bw_MBps"], ids=done_ids)
            est, pr = probe(s, b, tau, params, est, ids=done_ids)
            if pools is not None and done_ids.shape[0]:
                execute(w, s, b, pools, staging, ids=done_ids)
            rec.update(rail=b.rail[pending].copy(), stage_off=b.stage_off[pending].copy(), failed_per_rail=per_rail,
                       done_ids=done_ids, probe=pr, tau=tau[done_ids].copy(), T=b.T, base=b.base,
                       n_slices=b.n_slices, A_after=b.A_after)
            pending = np.ascontiguousarray(np.setdiff1d(pending, done_ids).astype(np.uint32))
        monitor_step(mp, mon, hard, cong, rec["probe"], est_before)
        rec.update(retry_after=retry.copy(), est_after=est.copy(), mon_after=mon.copy(), hard=hard, cong=cong,
                   est_before=est_before, epoch=ep)
        records.append(rec)
        e += 1
    return records


def run_epochs(w, s: Slices, pools=None, staging=None):
    """Re-planning workload: per epoch bind the pending slices under that epoch's
    telemetry, retire what the rails' byte budgets allow, move the retired slices,
    and carry the rest over; a final drain pass with unlimited budget finishes.
    Returns one record per pass."""
    pending = np.arange(s.n, dtype=np.uint32)
    records = []
    for ep in list(w.epochs) + [w.drain]:
        if pending.shape[0] == 0:
            records.append(dict(pending=pending, status=OK, rail=None, stage_off=None, done_ids=pending,
                                T=None, base=None))
            continue
        b = bind(s.len, ep.rails, ids=pending)
        if b.status != OK:
            records.append(dict(pending=pending, status=b.status, rail=None, stage_off=None,
                                done_ids=pending[:0], T=b.T, base=b.base))
            continue
        done = retire(s, b, ep.rails["queued_bytes"], ep.budget, ids=pending).astype(bool)
        done_ids = np.ascontiguousarray(pending[done])
        if pools is not None and done_ids.shape[0]:
            execute(w, s, b, pools, staging, ids=done_ids)
        records.append(dict(pending=pending, status=OK, rail=b.rail[pending].copy(),
                            stage_off=b.stage_off[pending].copy(), done_ids=done_ids, T=b.T, base=b.base))
        pending = np.ascontiguousarray(pending[~done])
    return records, pending
