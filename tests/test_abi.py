"""CPU-side checks of the C ABI: the library loads, exports every declared symbol, and the
Python-side structure layouts agree with the header (compiled with gcc)."""
import ctypes as C
import os
import re
import subprocess
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "tent.h")


@pytest.fixture(scope="module")
def T():
    from paper_2604_00368_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2604_00368_amd import build
        build.build()
    return binding


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tent_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(T):
    L = T.lib()
    names = declared_functions()
    assert "tent_declare" in names and "tent_plan" in names and "tent_execute" in names
    for n in names:
        assert hasattr(L, n), n
    assert sorted(T.EXPORTS) == names                       # the binding covers the whole header


def test_binding_has_the_same_names(T):
    for n in declared_functions():
        assert callable(getattr(T, n)), n


def test_struct_layouts_match_header(T, tmp_path):
    from paper_2604_00368_amd import workloads as W
    src = tmp_path / "layout.c"
    src.write_text(r'''
#include <stdio.h>
#include <stddef.h>
#include "tent.h"
int main(void) {
  printf("config %zu %zu %zu %zu %zu %zu\n", sizeof(tent_config), offsetof(tent_config, slice_bytes),
         offsetof(tent_config, staging_arena), offsetof(tent_config, staging_bytes), offsetof(tent_config, flags),
         offsetof(tent_config, max_rails));
  printf("extent %zu %zu %zu %zu\n", sizeof(tent_extent), offsetof(tent_extent, seg), offsetof(tent_extent, len),
         offsetof(tent_extent, off));
  printf("rail %zu %zu %zu %zu %zu %zu %zu\n", sizeof(tent_rail_state), offsetof(tent_rail_state, bw_MBps),
         offsetof(tent_rail_state, lat_ns), offsetof(tent_rail_state, queued_bytes), offsetof(tent_rail_state, beta1_q8),
         offsetof(tent_rail_state, penalty_q8), offsetof(tent_rail_state, health));
  printf("info %zu %zu %zu %zu %zu %zu %zu\n", sizeof(tent_plan_info), offsetof(tent_plan_info, n_slices),
         offsetof(tent_plan_info, n_pending_before), offsetof(tent_plan_info, rail_bytes),
         offsetof(tent_plan_info, rail_slices), offsetof(tent_plan_info, queued_after), offsetof(tent_plan_info, stage_base));
  printf("slice %zu %zu %zu %zu %zu %zu %zu\n", sizeof(tent_slice), offsetof(tent_slice, desc), offsetof(tent_slice, len),
         offsetof(tent_slice, off), offsetof(tent_slice, stage_off), offsetof(tent_slice, rail), offsetof(tent_slice, state));
  printf("dparams %zu %zu %zu %zu %zu\n", sizeof(tent_dispatch_params), offsetof(tent_dispatch_params, theta_bytes),
         offsetof(tent_dispatch_params, gamma_q8), offsetof(tent_dispatch_params, window), offsetof(tent_dispatch_params, rr_start));
  printf("dinfo %zu %zu %zu %zu %zu %zu\n", sizeof(tent_dispatch_info), offsetof(tent_dispatch_info, plan),
         offsetof(tent_dispatch_info, n_mice), offsetof(tent_dispatch_info, n_elephant),
         offsetof(tent_dispatch_info, n_deferred), offsetof(tent_dispatch_info, rr_next));
  printf("mparams %zu %zu %zu %zu %zu\n", sizeof(tent_monitor_params), offsetof(tent_monitor_params, err_threshold),
         offsetof(tent_monitor_params, recover_windows), offsetof(tent_monitor_params, cooldown_windows),
         offsetof(tent_monitor_params, degrade_q8));
  printf("monitor %zu %zu %zu %zu %zu %zu\n", sizeof(tent_rail_monitor), offsetof(tent_rail_monitor, state),
         offsetof(tent_rail_monitor, score), offsetof(tent_rail_monitor, clean), offsetof(tent_rail_monitor, cooldown_left),
         offsetof(tent_rail_monitor, cooldown_next));
  printf("probe %zu %zu %zu %zu %zu\n", sizeof(tent_probe_params), offsetof(tent_probe_params, hw_MBps),
         offsetof(tent_probe_params, alpha_q8), offsetof(tent_probe_params, delta_ns), offsetof(tent_probe_params, ewma_q8));
  printf("flags %d %d %d %d\n", TENT_FLAG_SKIP_OVERLAP_CHECK, TENT_FLAG_PROFILE, TENT_FLAG_SERIAL_BINDING,
         TENT_FLAG_BOUNDED_STAGING);
  printf("consts %d %d %d %d %d %d %d\n", TENT_MAX_RAILS, TENT_T_COUNT, TENT_DEFER, TENT_ERR_INVALID, TENT_ERR_RANGE,
         TENT_ERR_STATE, TENT_FLAG_SERIAL_BINDING);
  return 0;
}''')
    exe = tmp_path / "layout"
    subprocess.check_call(["gcc", "-std=c11", "-I", os.path.join(ROOT, "include"), "-o", str(exe), str(src)])
    out = {l.split()[0]: [int(x) for x in l.split()[1:]] for l in subprocess.check_output([str(exe)]).decode().splitlines()}

    def ct(struct, *fields):
        return [C.sizeof(struct)] + [getattr(struct, f).offset for f in fields]

    def nd(dtype, *fields):
        return [dtype.itemsize] + [dtype.fields[f][1] for f in fields]

    assert out["config"] == ct(T.tent_config, "slice_bytes", "staging_arena", "staging_bytes", "flags", "max_rails")
    assert out["extent"] == nd(W.EXTENT_DTYPE, "seg", "len", "off")
    assert out["rail"] == nd(W.RAIL_DTYPE, "bw_MBps", "lat_ns", "queued_bytes", "beta1_q8", "penalty_q8", "health")
    assert out["info"] == ct(T.tent_plan_info, "n_slices", "n_pending_before", "rail_bytes", "rail_slices",
                             "queued_after", "stage_base")
    assert out["slice"] == nd(T.SLICE_DTYPE, "desc", "len", "off", "stage_off", "rail", "state")
    assert out["dparams"] == nd(W.DISPATCH_PARAMS_DTYPE, "theta_bytes", "gamma_q8", "window", "rr_start")
    assert out["dinfo"] == ct(T.tent_dispatch_info, "plan", "n_mice", "n_elephant", "n_deferred", "rr_next")
    assert out["mparams"] == nd(W.MONITOR_PARAMS_DTYPE, "err_threshold", "recover_windows", "cooldown_windows", "degrade_q8")
    assert out["monitor"] == nd(T.MONITOR_DTYPE, "state", "score", "clean", "cooldown_left", "cooldown_next")
    assert out["probe"] == nd(W.PROBE_DTYPE, "hw_MBps", "alpha_q8", "delta_ns", "ewma_q8")
    assert out["flags"] == [T.TENT_FLAG_SKIP_OVERLAP_CHECK, T.TENT_FLAG_PROFILE, T.TENT_FLAG_SERIAL_BINDING,
                            T.TENT_FLAG_BOUNDED_STAGING]
    assert out["consts"] == [T.TENT_MAX_RAILS, len(T.TENT_T_NAMES), T.TENT_DEFER, T.TENT_ERR_INVALID,
                             T.TENT_ERR_RANGE, T.TENT_ERR_STATE, T.TENT_FLAG_SERIAL_BINDING]


def test_argument_errors_need_no_device(T):
    # null / malformed arguments are rejected before any HIP call
    L = T.lib()
    assert L.tent_create(None, None) == T.TENT_ERR_INVALID
    ctx = C.c_void_p()
    cfg = T.tent_config(0, 0x1000, 4096, 0, 0)              # slice size 0
    assert L.tent_create(C.byref(ctx), C.byref(cfg)) == T.TENT_ERR_INVALID
    cfg = T.tent_config(65536, None, 4096, 0, 0)             # no arena
    assert L.tent_create(C.byref(ctx), C.byref(cfg)) == T.TENT_ERR_INVALID
    cfg = T.tent_config(65536, 0x1000, 4096, 0, 65)          # too many rails
    assert L.tent_create(C.byref(ctx), C.byref(cfg)) == T.TENT_ERR_RANGE
    assert L.tent_destroy(None) == T.TENT_ERR_INVALID
    assert L.tent_execute(None, 1, None) == T.TENT_ERR_INVALID
    assert L.tent_execute_bounded(None, 1, 1 << 20, 1, None) == T.TENT_ERR_INVALID
    assert L.tent_plan_dispatch(None, 1, None, 0, None, None, None, None) == T.TENT_ERR_INVALID
    assert L.tent_sim_fail(None, 1, None, None, None) == T.TENT_ERR_INVALID
    assert L.tent_get_retries(None, 1, None, 0) == T.TENT_ERR_INVALID
    assert L.tent_get_modes(None, 1, None, 0) == T.TENT_ERR_INVALID
    assert L.tent_monitor_init(None, None, 3) == T.TENT_ERR_INVALID
    for st, word in [(0, "ok"), (1, "defer"), (-1, "invalid"), (-2, "range"), (-3, "order"), (-4, "memory"), (-5, "HIP")]:
        assert word.lower() in T.tent_strerror(st).lower()


def test_rail_monitor_matches_the_oracle(T):
    # the health monitor is host arithmetic: the library's state machine against the oracle's, window by window
    import oracle
    from paper_2604_00368_amd import workloads as W
    for seed in range(6):
        rng = np.random.Generator(np.random.PCG64(600 + seed))
        R = int(rng.integers(1, 65))
        mp = W.make_monitor_params(err_threshold=int(rng.integers(0, 6)), recover_windows=int(rng.integers(0, 4)),
                                   cooldown_windows=int(rng.integers(0, 4)), degrade_q8=int(rng.choice([0, 128, 200, 256])))
        rails = W.make_rails(rng.integers(1000, 100000, R))
        mon = T.tent_monitor_init(mp, R)
        ref = oracle.monitor_init(R, mp)
        for f in mon.dtype.names:
            assert np.array_equal(mon[f], ref[f])
        for window in range(60):
            hard = (rng.integers(0, 8, R) * (rng.random(R) < 0.2)).astype(np.uint32)
            cong = (rng.integers(0, 12, R) * (rng.random(R) < 0.3)).astype(np.uint32)
            bw = rng.integers(1000, 100000, R).astype(np.uint32)
            probe = (bw * rng.choice([0.0, 0.3, 0.49, 0.5, 0.9, 1.0], R)).astype(np.uint32)
            out = T.tent_monitor_update(mp, mon, rails, hard, cong, probe, bw)
            oracle.monitor_step(mp, ref, hard, cong, probe, bw)
            for f in mon.dtype.names:
                assert np.array_equal(mon[f], ref[f]), (seed, window, f)
            assert np.array_equal(out["health"], ref["state"].astype(np.uint8))
            assert np.array_equal(out["bw_MBps"], rails["bw_MBps"])      # only the health field changes
    # argument errors
    mp = W.make_monitor_params()
    mon = T.tent_monitor_init(mp, 2)
    with pytest.raises(T.TentError) as ei:
        T.tent_monitor_init(mp, 65)
    assert ei.value.status == T.TENT_ERR_RANGE
    mon["state"][1] = 7
    with pytest.raises(T.TentError) as ei:
        T.tent_monitor_update(mp, mon, W.make_rails([1, 1]), [0, 0], [0, 0], [0, 0], [1, 1])
    assert ei.value.status == T.TENT_ERR_INVALID


def test_product_path_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2604_00368_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), os.path.join(dirpath, f)


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr
