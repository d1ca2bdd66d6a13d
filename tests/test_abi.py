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
    for st, word in [(0, "ok"), (1, "defer"), (-1, "invalid"), (-2, "range"), (-3, "order"), (-4, "memory"), (-5, "HIP")]:
        assert word.lower() in T.tent_strerror(st).lower()


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
