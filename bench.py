#!/usr/bin/env python3
"""Benchmark of the slice-spraying hot path on one MI355X.

One step = tent_plan (extent scans, slice scan, slice-table expansion, rail binding) followed by
tent_execute (gather into per-rail staging, scatter to destination) over one freshly declared
batch of the KVCache-migration workload; descriptor tables and byte pools are resident in HBM
before the timed region starts.  The K timed steps run twice: on a single stream, and with the
plans on a second stream so that step k+1's binding (a one-wavefront dependency chain) runs under
step k's copies; the second figure is the headline unless --single-stream is given, both are
printed.  Prints ONE JSON line.

  value        read+write GB/s of the whole step: 4 * payload * steps / elapsed
  roofline     the slower of the two copy kernels (gather: source pages -> staging, scatter: staging ->
               destination): 2 * payload bytes per launch against HBM peak, duration from HIP events
               recorded on the launch stream around every launch inside the timed region
  configs      the same two timed passes, shorter, for the other workloads (tiny, rl_params, many_small,
               many_small_x6; the re-planning workload is the `replanning` entry)
  verified     after the timed passes the destination of the last batch is compared on the device with its
               definition (DST_j[x] == SRC_j[x] for every transfer j and byte x)
  cpu_baseline the sequential CPU oracle on the same workload (a reduced instance when host memory is short)

Other legs (--ceilings, --sweep) print a line of their own and nothing else.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

HBM_PEAK_GBPS = 8000.0
ALL_LEGS = ("configs", "declare", "concurrent", "feedback", "recovery", "replanning", "dispatch", "bounded", "graph")

# HBM bytes per copy launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (scaled by the
# plain-copy calibration dispatch of the same run; summaries under profiles/).  The figures belong
# to one version of the copy kernels and of the kernels that build their tables: when one of those
# sources changes they are reported as null until the counters are taken again.
PMC_SOURCES = ("copy.hip", "copy_generic.h", "split.hip", "tile_tables.h")
PMC_TRAFFIC = {
    "copy_sources_sha256": "40cb27ddb00ff4ebb63f4a50cccb998e176129192c040f14719fefbf480c15aa",
    # bytes read + bytes written per launch (profiles/copy_kernels_hbm_traffic.txt)
    "kv_migration": {"gather": 43019356871, "scatter": 43019353287},
    "rl_params": {"gather": 30488282590, "scatter": 30488290142},
    "many_small_x6": {"gather": 33592918724, "scatter": 33592915140},
}


def measured_traffic(workload, kernel):
    import hashlib
    csrc = os.path.join(os.path.dirname(os.path.abspath(__file__)), "paper_2604_00368_amd", "csrc")
    try:
        digest = hashlib.sha256(b"".join(open(os.path.join(csrc, f), "rb").read() for f in PMC_SOURCES)).hexdigest()
    except OSError:
        return None
    if digest != PMC_TRAFFIC["copy_sources_sha256"]:
        return None
    return PMC_TRAFFIC.get(workload, {}).get(kernel)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="kv_migration",
                    choices=["tiny", "kv_migration", "rl_params", "many_small", "many_small_x6", "kv_skewed"])
    ap.add_argument("--placement", default="regions", choices=["regions", "plain"],
                    help="regions: the pools are carved from one reservation so that the read side and the write side of "
                         "either copy lie in different regions of the device memory, found by measurement (default); "
                         "plain: three ordinary allocations")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--serial-binding", action="store_true")
    ap.add_argument("--headline-only", action="store_true",
                    help="run only the headline pass (and the plain-copy calibration): no second timed pass and "
                         "none of the other legs; used for the profiler summaries under profiles/")
    ap.add_argument("--legs", default="all",
                    help="comma-separated subset of the legs beside the timed passes: " + ", ".join(ALL_LEGS)
                         + " (default: all; 'none' for the timed passes only)")
    ap.add_argument("--single-stream", action="store_true",
                    help="report the single-stream step time as the headline (default: plan of step k+1 "
                         "overlaps execute of step k on a second stream)")
    ap.add_argument("--ceilings", action="store_true",
                    help="measure the copy ceilings of the box instead (plain, read-only, write-only, contiguous and "
                         "paged copies through the engine) and print them as one JSON line")
    ap.add_argument("--sweep", action="store_true",
                    help="slice-size sweep (4 KiB - 64 MiB, contiguous and 32 KiB-paged layouts) instead; one JSON line")
    return ap.parse_args()


_T0 = time.perf_counter()


def log(msg):
    """Progress line on stderr (stdout carries the one JSON line)."""
    print(f"[bench {time.perf_counter() - _T0:6.1f}s] {msg}", file=sys.stderr, flush=True)


def make_workload(name):
    from paper_2604_00368_amd import workloads as W
    if name == "many_small_x6":
        return W.many_small(layers=6)
    if name == "kv_skewed":          # a quarter of config 2 with every page at an odd address (unaligned 16-byte accesses)
        return W.kv_migration(n_req=8, skew=(3, 5))
    return W.CONFIGS[name]()


def host_memory_available():
    try:
        import psutil
        return int(psutil.virtual_memory().available)
    except Exception:
        return 0


def cpu_baseline(name):
    """Time the oracle as it stands on the benchmarked workload (host memory only): a bounded number of
    repetitions of plan + execute.  When the host cannot hold source pool, destination pool and arena, a
    reduced instance of the same generator is used, and the sample says so."""
    import oracle
    from paper_2604_00368_amd import workloads as W
    oracle.build()
    w = make_workload(name)
    need = w.seg_bytes[0] + w.seg_bytes[1] + w.staging_bytes
    avail = host_memory_available()
    if need + (8 << 30) <= avail:
        sample = f"the benchmarked {name} batch in full"
    else:
        why = f"host memory short ({avail >> 30} GiB available, {need >> 30} GiB needed)"
        if name == "kv_migration":
            w = W.kv_migration(n_req=3)
            sample = f"kv_migration generator with 3 of 32 requests (all 32 layers, 32 KiB pages, 256 KiB slices, 9 rails): {why}"
        elif name == "rl_params":
            w = W.rl_params(layers=4)
            sample = f"rl_params generator with 4 of 32 layers plus the embedding (1 MiB slices, 8 rails): {why}"
        elif name.startswith("many_small"):
            w = W.many_small()
            sample = f"many_small generator, 4096 requests, one layer (18 KiB pages, 16 KiB slices, 16 rails): {why}"
        else:
            w = W.kv_migration(n_req=2, skew=(3, 5))
            sample = f"kv_skewed generator with 2 requests: {why}"
    # source bytes: one random block repeated (the oracle's time does not depend on the values); the pages of
    # all three buffers are committed before anything is timed, by one thread per host core
    import threading
    n_thr = max(1, min(len(os.sched_getaffinity(0)), int(os.environ.get("OMP_NUM_THREADS", "1024"))))
    rng = np.random.Generator(np.random.PCG64(99))
    block = np.frombuffer(rng.bytes(64 << 20), dtype=np.uint8)
    src = np.empty(w.seg_bytes[0], dtype=np.uint8)
    dst = np.empty(w.seg_bytes[1], dtype=np.uint8)
    staging = np.empty(w.staging_bytes, dtype=np.uint8)

    def prepare(k):
        for buf, fill in ((src, True), (dst, False), (staging, False)):
            per = -(-buf.shape[0] // n_thr)
            lo, hi = k * per, min(buf.shape[0], (k + 1) * per)
            for at in range(lo, hi, block.shape[0]):
                n = min(block.shape[0], hi - at)
                if fill:
                    buf[at:at + n] = block[:n]
                else:
                    buf[at:at + n] = 0
    thr = [threading.Thread(target=prepare, args=(k,)) for k in range(n_thr)]
    for t in thr:
        t.start()
    for t in thr:
        t.join()
    log(f"cpu baseline: buffers ready ({(src.shape[0] + dst.shape[0] + staging.shape[0]) >> 30} GiB)")
    reps = 0
    t_plan = t_exec = 0.0
    n_slices = 0
    t_begin = time.perf_counter()
    while reps < 1 or (time.perf_counter() - t_begin < 10.0 and reps < 80):
        t0 = time.perf_counter()
        s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
        b = oracle.bind(s.len, w.rails)
        t1 = time.perf_counter()
        oracle.execute(w, s, b, [src, dst], staging)
        t2 = time.perf_counter()
        t_plan += t1 - t0
        t_exec += t2 - t1
        n_slices = s.n
        reps += 1
        if reps == 1:
            log(f"cpu baseline: first repetition {t2 - t0:.1f} s")
    step = (t_plan + t_exec) / reps

    # the same execute with the slices dealt to one thread per host core (each thread runs the
    # oracle's gather pass and scatter pass over its own slices; ctypes releases the GIL)
    parts = [np.ascontiguousarray(np.arange(k, n_slices, n_thr, dtype=np.uint32)) for k in range(n_thr)]
    t0 = time.perf_counter()
    thr = [threading.Thread(target=oracle.execute, args=(w, s, b, [src, dst], staging, ids)) for ids in parts]
    for t in thr:
        t.start()
    for t in thr:
        t.join()
    t_all = time.perf_counter() - t0
    return {
        "value": round(4 * w.payload / step / 1e9, 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
        "sample": f"{sample}; payload {w.payload / 2**30:.2f} GiB, {n_slices} slices, {reps} repetitions",
        "plan_slices_per_s": round(n_slices / (t_plan / reps), 1),
        "execute_GBps": round(4 * w.payload / (t_exec / reps) / 1e9, 3),
        "execute_GBps_threads": round(4 * w.payload / t_all / 1e9, 3), "threads": n_thr,
    }


def destination_matches_definition(torch, w, src, dst, chunk_extents=1 << 15):
    """DST_j[x] == SRC_j[x] for every transfer j and byte x, on the device, for workloads whose source and
    destination extents pair up one to one (all of the benchmark's workloads)."""
    if not (np.array_equal(w.src_ptr, w.dst_ptr) and np.array_equal(w.src_ext["len"], w.dst_ext["len"])):
        return None
    lens = np.unique(w.src_ext["len"])
    if lens.shape[0] == 1 and (w.src_ext["off"] % lens[0] == 0).all() and (w.dst_ext["off"] % lens[0] == 0).all():
        page = int(lens[0])
        n_src, n_dst = src.numel() // page * page, dst.numel() // page * page
        sv, dv = src[:n_src].view(-1, page), dst[:n_dst].view(-1, page)
        for lo in range(0, w.src_ext.shape[0], chunk_extents):
            si = torch.from_numpy((w.src_ext["off"][lo:lo + chunk_extents] // page).astype(np.int64)).to(src.device)
            di = torch.from_numpy((w.dst_ext["off"][lo:lo + chunk_extents] // page).astype(np.int64)).to(src.device)
            if not torch.equal(sv[si], dv[di]):
                return False
        return True
    if w.src_ext.shape[0] > 4096:                # many extents of mixed or unaligned sizes: a sample of them
        rng = np.random.Generator(np.random.PCG64(7))
        pick = rng.choice(w.src_ext.shape[0], size=4096, replace=False)
    else:
        pick = range(w.src_ext.shape[0])
    for e in pick:
        se, de = w.src_ext[e], w.dst_ext[e]
        a = src[int(se["off"]):int(se["off"]) + int(se["len"])]
        b = dst[int(de["off"]):int(de["off"]) + int(de["len"])]
        if not torch.equal(a, b):
            return False
    return True


class Run:
    """One workload in given pools: context, declared batches and the two timed passes."""

    def __init__(self, T, W, torch, dev, w, pools, steps, warmup, flags):
        self.T, self.W, self.torch, self.dev, self.w = T, W, torch, dev, w
        self.steps, self.warmup = steps, warmup
        self.src = pools[0][:w.seg_bytes[0]]
        self.arena = pools[1][:w.staging_bytes]
        self.dst = pools[2][:w.seg_bytes[1]]
        W.fill_torch(w, 0, dev, out=self.src)
        self.dst.zero_()
        self.stream = torch.cuda.current_stream(dev)
        self.ctx = T.tent_create(w.slice_bytes, self.arena.data_ptr(), self.arena.numel(), flags)
        T.tent_register_segment(self.ctx, self.src.data_ptr(), self.src.numel())
        T.tent_register_segment(self.ctx, self.dst.data_ptr(), self.dst.numel())
        total = warmup + steps
        torch.cuda.synchronize(dev)
        t0 = time.perf_counter()
        self.batches = [T.tent_declare(self.ctx, w.src_ptr, w.src_ext, w.dst_ptr, w.dst_ext) for _ in range(total)]
        self.declare_host_ms = (time.perf_counter() - t0) * 1e3 / total     # host time per call; device work still queued
        torch.cuda.synchronize(dev)
        self.n_slices = T.tent_slice_count(self.ctx, self.batches[0])

    def declare(self):
        w = self.w
        return self.T.tent_declare(self.ctx, w.src_ptr, w.src_ext, w.dst_ptr, w.dst_ext)

    def step_single(self, h):
        self.T.tent_plan(self.ctx, h, self.w.rails, want_info=False, stream=self.stream)
        self.T.tent_execute(self.ctx, h, self.stream)

    def step_pipelined(self, h, plan_stream):
        # every step still plans and executes its own batch; the plan is enqueued on a second stream
        # so that the next step's (mostly one-wavefront) binding runs under this step's copies
        self.T.tent_plan(self.ctx, h, self.w.rails, want_info=False, stream=plan_stream)
        ev = self.torch.cuda.Event()
        ev.record(plan_stream)
        self.stream.wait_event(ev)
        self.T.tent_execute(self.ctx, h, self.stream)

    def timed_pass(self, step):
        T, torch = self.T, self.torch
        for h in self.batches[:self.warmup]:
            step(h)
        torch.cuda.synchronize(self.dev)
        T.tent_get_timings(self.ctx)                   # drop warm-up intervals
        torch.cuda.synchronize(self.dev)
        t0 = time.perf_counter()
        for h in self.batches[self.warmup:]:
            step(h)
        torch.cuda.synchronize(self.dev)
        dt = time.perf_counter() - t0
        tm_ = T.tent_get_timings(self.ctx)
        assert T.tent_poll(self.ctx, self.batches[-1], self.stream) == 0
        return dt, tm_

    def reset_all(self):
        for h in self.batches:
            self.T.tent_reset(self.ctx, h, self.stream)
        self.torch.cuda.synchronize(self.dev)

    def verify(self):
        return destination_matches_definition(self.torch, self.w, self.src, self.dst)

    def close(self):
        self.T.tent_destroy(self.ctx)


def summarize(w, n_slices, steps, elapsed_single, tm_single, elapsed_piped, tm_piped):
    """Compact record of one workload's two timed passes."""
    plan_ms = sum(tm_single[n][0] for n in ("extent_scan", "slice_scan", "expand", "compact", "bind")) / max(1, steps)
    g_ms, g_n = tm_piped["gather"]
    s_ms, s_n = tm_piped["scatter"]
    g_avg, s_avg = g_ms / max(1, g_n), s_ms / max(1, s_n)
    ms1, ms2 = elapsed_single * 1e3 / steps, elapsed_piped * 1e3 / steps
    value = 4 * w.payload / (ms2 * 1e-3) / 1e9
    return {"payload_bytes": w.payload, "n_slices": n_slices, "slice_bytes": w.slice_bytes,
            "n_rails": int(w.rails.shape[0]), "steps": steps,
            "ms_per_step_single_stream": round(ms1, 4), "ms_per_step_two_streams": round(ms2, 4),
            "GBps": round(value, 1), "pct_of_hbm_peak": round(100 * value / HBM_PEAK_GBPS, 2),
            "plan_ms": round(plan_ms, 4), "slices_planned_per_s": round(n_slices / (plan_ms * 1e-3), 1) if plan_ms > 0 else None,
            "gather_GBps": round(2 * w.payload / (g_avg * 1e-3) / 1e9, 1),
            "scatter_GBps": round(2 * w.payload / (s_avg * 1e-3) / 1e9, 1)}


def ceilings(args):
    """Copy ceilings of the box: what plain kernels reach, beside the engine's copies of contiguous and paged bytes."""
    import torch
    from paper_2604_00368_amd import binding as T
    from paper_2604_00368_amd import placement
    from paper_2604_00368_amd import workloads as W
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    T.lib()
    n = 4 << 30
    ws = {"contiguous": W.sweep(1 << 20, False, payload=n), "paged_32KiB": W.sweep(1 << 20, True, payload=n)}
    src, arena, dst, layout = placement.place_pools(dev, max(w.seg_bytes[0] for w in ws.values()),
                                                    max(w.staging_bytes for w in ws.values()),
                                                    max(w.seg_bytes[1] for w in ws.values()), mode=args.placement)

    def timed(fn, reps=5):
        fn()
        torch.cuda.synchronize(dev)
        best = None
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            torch.cuda.synchronize(dev)
            ms = e0.elapsed_time(e1)
            best = ms if best is None else min(best, ms)
        return best

    a, b = src[:n], arena[:n]
    a.random_(0, 256)
    out = {"bytes": n, "unit": "GB/s, bytes read plus bytes written", "placement": layout.mode,
           "plain_copy_torch_bitwise_not": round(2 * n / (timed(lambda: torch.bitwise_not(a, out=b)) * 1e-3) / 1e9, 1),
           "write_only_torch_fill": round(n / (timed(lambda: b.fill_(7)) * 1e-3) / 1e9, 1),
           "read_only_torch_sum_int64": round(n / (timed(lambda: a.view(torch.int64).sum()) * 1e-3) / 1e9, 1)}
    stream = torch.cuda.current_stream(dev)
    for name, w in ws.items():
        r = Run(T, W, torch, dev, w, (src, arena, dst), 4, 1, T.TENT_FLAG_PROFILE)
        dt, tm = r.timed_pass(r.step_single)
        out[f"engine_{name}_gather"] = round(2 * w.payload / (tm["gather"][0] / tm["gather"][1] * 1e-3) / 1e9, 1)
        out[f"engine_{name}_scatter"] = round(2 * w.payload / (tm["scatter"][0] / tm["scatter"][1] * 1e-3) / 1e9, 1)
        out[f"engine_{name}_verified"] = r.verify()
        r.close()
    print(json.dumps({"ceilings": out}))


def sweep(args):
    """Slice-size sweep (the shape of the paper's block-size sweeps, Section 5.2): 4 GiB in 64 equal transfers,
    9 rails, slice size 4 KiB - 64 MiB, contiguous extents or 32 KiB pages shuffled on both sides."""
    import torch
    from paper_2604_00368_amd import binding as T
    from paper_2604_00368_amd import placement
    from paper_2604_00368_amd import workloads as W
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    T.lib()
    payload = 4 << 30
    biggest = [W.sweep(kib * 1024, paged, payload=payload) for paged in (False, True) for kib in (4, 65536)]
    src, arena, dst, layout = placement.place_pools(dev, max(w.seg_bytes[0] for w in biggest),
                                                    max(w.staging_bytes for w in biggest),
                                                    max(w.seg_bytes[1] for w in biggest), mode=args.placement)
    rows = []
    for paged in (False, True):
        for kib in (4, 16, 64, 256, 1024, 4096, 16384, 65536):
            w = W.sweep(kib * 1024, paged, payload=payload)
            r = Run(T, W, torch, dev, w, (src, arena, dst), 4, 1, T.TENT_FLAG_PROFILE)
            dt, tm = r.timed_pass(r.step_single)
            plan = sum(tm[k][0] for k in ("extent_scan", "slice_scan", "expand", "compact", "bind")) / 4
            g, s = tm["gather"][0] / tm["gather"][1], tm["scatter"][0] / tm["scatter"][1]
            rows.append({"layout": "paged_32KiB" if paged else "contiguous", "slice_KiB": kib, "slices": r.n_slices,
                         "plan_ms": round(plan, 4), "gather_GBps": round(2 * w.payload / g / 1e6, 0),
                         "scatter_GBps": round(2 * w.payload / s / 1e6, 0),
                         "execute_GBps": round(4 * w.payload / (g + s) / 1e6, 0)})
            r.close()
    print(json.dumps({"sweep": {"payload_bytes": payload, "placement": layout.mode, "rows": rows}}))


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU only: the rails are simulated staging regions in one device's HBM; "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2604_00368_amd import binding as T
    from paper_2604_00368_amd import workloads as W

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    T.lib()                                            # fails loudly when the HIP library is missing
    if args.ceilings:
        return ceilings(args)
    if args.sweep:
        return sweep(args)
    legs = set() if args.headline_only or args.legs == "none" else \
        set(ALL_LEGS) if args.legs == "all" else set(x for x in args.legs.split(",") if x)
    unknown = legs - set(ALL_LEGS)
    if unknown:
        print(f"unknown legs: {sorted(unknown)}", file=sys.stderr)
        sys.exit(2)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    w = make_workload(args.workload)
    others = []
    if "configs" in legs:
        others = [make_workload(n) for n in ("tiny", "kv_migration", "rl_params", "many_small", "many_small_x6")
                  if n != args.workload]
    # The pools: by default carved from one reservation so that the read side and the write side of either copy
    # lie in different regions of the device memory (placement.py: what the regions are, how they are found).
    # They are sized for the largest workload of the run; every workload uses the front of each pool.
    from paper_2604_00368_amd import placement
    every = [w] + others
    pools3 = placement.place_pools(dev, max(x.seg_bytes[0] for x in every), max(x.staging_bytes for x in every),
                                   max(x.seg_bytes[1] for x in every), mode=args.placement)
    pools, layout = pools3[:3], pools3[3]
    flags = T.TENT_FLAG_PROFILE | (T.TENT_FLAG_SERIAL_BINDING if args.serial_binding else 0)
    log(f"pools placed ({layout.mode})")
    run = Run(T, W, torch, dev, w, pools, args.steps, args.warmup, flags)
    log(f"{args.workload}: {len(run.batches)} batches declared")
    ctx, batches, stream, src, arena, dst = run.ctx, run.batches, run.stream, run.src, run.arena, run.dst
    n_slices, declare_ms = run.n_slices, run.declare_host_ms

    # default priority; created one after the other so that, with the process's four hardware queues dealt to
    # streams in turn, the two plan streams and the first stream sit on three different queues
    plan_stream = torch.cuda.Stream(dev)
    plan_stream2 = torch.cuda.Stream(dev)

    def step_pipelined(h):
        run.step_pipelined(h, plan_stream)

    lean = args.headline_only
    elapsed_deep = concurrent_plan_s = None
    many = []
    if lean:
        elapsed, tm = run.timed_pass(run.step_single if args.single_stream else step_pipelined)
        elapsed_single, tm_single = elapsed, tm
        elapsed_piped, tm_piped = elapsed, tm
    else:
        elapsed_single, tm_single = run.timed_pass(run.step_single)
        run.reset_all()                                # back to PENDING: the next pass re-plans from scratch
        elapsed_piped, tm_piped = run.timed_pass(step_pipelined)
        if args.single_stream:
            elapsed, tm = elapsed_single, tm_single
        else:
            elapsed, tm = elapsed_piped, tm_piped
    verified = run.verify()                            # the last timed batch's bytes against their definition
    log(f"timed passes done, verified={verified}")

    if "concurrent" in legs:
        # Third pass, reported beside the headline only: plans alternate between two plan streams, so the (mostly
        # one-wavefront) binding chains of two later steps run side by side under the copies of an earlier one.
        run.reset_all()
        plan_streams = [plan_stream, plan_stream2]
        turn = [0]

        def step_two_plan_streams(h):
            ps = plan_streams[turn[0] & 1]
            turn[0] += 1
            run.step_pipelined(h, ps)

        elapsed_deep, _ = run.timed_pass(step_two_plan_streams)
        # Planning throughput when independent batches are planned side by side (each chain is one wavefront, so
        # the chains of different batches run on different compute units): every batch on its own stream.
        run.reset_all()
        many = [torch.cuda.Stream(dev) for _ in range(min(8, len(batches)))]
        for k, h in enumerate(batches[:len(many)]):      # warm-up
            T.tent_plan(ctx, h, w.rails, want_info=False, stream=many[k])
        torch.cuda.synchronize(dev)
        run.reset_all()
        t0 = time.perf_counter()
        for k, h in enumerate(batches):
            T.tent_plan(ctx, h, w.rails, want_info=False, stream=many[k % len(many)])
        torch.cuda.synchronize(dev)
        concurrent_plan_s = time.perf_counter() - t0
        T.tent_get_timings(ctx)
        run.reset_all()

    # A step that also declares its batch (Section 4.1: submitting a transfer returns at once): declare, plan on
    # the second stream, execute; the batch of two steps ago, long complete, is released, so the tables of
    # released batches serve the new declarations.  The host arrays cross PCIe inside the timed region.
    with_declare = None
    if "declare" in legs:
        run.reset_all()
        live = []

        def step_with_declare(_h):
            t0 = time.perf_counter()
            h = run.declare()
            host[0] += time.perf_counter() - t0
            run.step_pipelined(h, plan_stream)
            live.append(h)
            if len(live) > 2:
                T.tent_release(ctx, live.pop(0))

        host = [0.0]
        for k in range(args.warmup):
            step_with_declare(None)
        torch.cuda.synchronize(dev)
        host = [0.0]
        t0 = time.perf_counter()
        for k in range(args.steps):
            step_with_declare(None)
        torch.cuda.synchronize(dev)
        dt = time.perf_counter() - t0
        ok_left = T.tent_poll(ctx, live[-1], stream) == 0
        for h in live:
            T.tent_release(ctx, h)
        T.tent_get_timings(ctx)
        with_declare = {"ms_per_step": round(dt * 1e3 / args.steps, 4),
                        "GBps": round(4 * w.payload * args.steps / dt / 1e9, 1),
                        "pct_of_hbm_peak": round(100 * 4 * w.payload * args.steps / dt / 1e9 / HBM_PEAK_GBPS, 2),
                        "declare_host_ms_per_call": round(host[0] * 1e3 / args.steps, 4), "complete": bool(ok_left),
                        "verified": run.verify()}

    log("step-with-declare leg done")
    fb_ms, fb_n, rec_ms, n_retried, fastest = 0.0, 0, [], 0, 0
    R = int(w.rails.shape[0])
    disp_ms, dinfo, bounded, graph_ms, replanning = [], None, [], None, None
    h_fb = batches[-1]
    if "feedback" in legs:
        # Telemetry feedback (Eq. 2 probe + smoothed update) over one full window, outside the timed region:
        # every slice of one batch BOUND, latencies from the rail simulator at the nominal bandwidths.
        T.tent_reset(ctx, h_fb, stream)
        T.tent_plan(ctx, h_fb, w.rails, want_info=False, stream=stream)
        T.tent_sim_latency(ctx, h_fb, w.rails["bw_MBps"], stream)
        torch.cuda.synchronize(dev)
        T.tent_get_timings(ctx)
        fb_params = W.make_probe_params(2 * w.rails["bw_MBps"].astype(np.uint64))
        for _ in range(5):
            T.tent_update_bandwidth(ctx, h_fb, fb_params, w.rails, stream)
        fb_ms, fb_n = T.tent_get_timings(ctx)["feedback"]

    if "recovery" in legs:
        # Recovery after a hard error (Section 4.3), outside the timed region: the fastest rail fails with the
        # whole batch bound, its slices come back with a retry count, and the next plan (compaction into
        # retried and fresh slices, rotation pass, cost-model pass) is timed.
        fastest = int(np.argmax(w.rails["bw_MBps"]))
        failed_mask = np.zeros(R, dtype=np.uint8)
        failed_mask[fastest] = 1
        after = w.rails.copy()
        after["health"][fastest] = 2
        if R > 1:
            for _ in range(3):
                T.tent_reset(ctx, h_fb, stream)
                T.tent_plan(ctx, h_fb, w.rails, want_info=False, stream=stream)
                n_retried = int(T.tent_sim_fail(ctx, h_fb, failed_mask, True, stream)[fastest])
                torch.cuda.synchronize(dev)
                T.tent_get_timings(ctx)
                T.tent_plan(ctx, h_fb, after, want_info=False, stream=stream)
                torch.cuda.synchronize(dev)
                tm_rec = T.tent_get_timings(ctx)
                rec_ms.append(tm_rec["compact"][0] + tm_rec["bind"][0])
        T.tent_reset(ctx, h_fb, stream)

    if "replanning" in legs and args.workload == "kv_migration":
        # Re-planning over telemetry epochs (config 4: the same batch, bandwidths resampled and queues redrawn per
        # epoch, two rails lost on the way; what an epoch's byte budgets do not cover is re-planned), outside the
        # timed region.  One sequence = 16 epochs and a drain pass: plan, rail simulator, execute.
        wr = W.replanning()
        assert np.array_equal(wr.src_ext, w.src_ext) and np.array_equal(wr.dst_ext, w.dst_ext)
        seqs = []
        replan_stream = plan_stream                       # streams share 4 hardware queues: no further stream here
        for _ in range(2):
            T.tent_reset(ctx, h_fb, stream)
            dst.zero_()
            torch.cuda.synchronize(dev)
            T.tent_get_timings(ctx)
            t0 = time.perf_counter()
            passes = 0
            for ep in list(wr.epochs) + [wr.drain]:
                # plan and rail simulator on the second stream: the library orders the re-plan after
                # the previous execute's bookkeeping, beside its copies; the simulator's read-back
                # waits for the second stream only and gives the execute the exact count of slices to
                # move (enqueue-only, with launches sized by the budgets alone, measured slower: 23.6
                # against 20.7 ms, because the looser bound sends some passes through the full-batch copy)
                st_r, _ = T.tent_plan(ctx, h_fb, ep.rails, want_info=False, stream=replan_stream)
                T.tent_sim_advance(ctx, h_fb, ep.budget, replan_stream)
                T.tent_execute(ctx, h_fb, stream)
                passes += 1
            left = T.tent_poll(ctx, h_fb, stream)
            dt = time.perf_counter() - t0
            tm_r = T.tent_get_timings(ctx)
            assert left == 0
            seqs.append((dt, tm_r, passes))
        dt, tm_r, passes = min(seqs, key=lambda x: x[0])
        copy_ms = tm_r["gather"][0] + tm_r["scatter"][0]
        replanning = {"passes": passes, "total_ms": round(dt * 1e3, 3),
                      "GBps": round(4 * w.payload / dt / 1e9, 2),
                      "pct_of_hbm_peak": round(100 * 4 * w.payload / dt / 1e9 / HBM_PEAK_GBPS, 2),
                      "plan_ms_total": round(sum(tm_r[k][0] for k in ("extent_scan", "slice_scan", "expand",
                                                                        "compact", "bind")), 3),
                      "plan_stage_ms": {k: round(tm_r[k][0], 3) for k in ("extent_scan", "slice_scan", "expand",
                                                                               "compact", "bind")},
                      "copy_ms_total": round(copy_ms, 3),
                      "copy_GBps": round(4 * w.payload / (copy_ms * 1e-3) / 1e9, 1),
                      "verified": run.verify()}
        T.tent_reset(ctx, h_fb, stream)

    log("feedback / recovery / re-planning legs done")
    if "dispatch" in legs:
        # Request-level dispatch (Algorithm 1: mice round robin / weighted spraying of elephants), outside the
        # timed region: the whole batch, every transfer HIGH priority, theta = 4 slices.
        dparams = W.make_dispatch_params(4 * w.slice_bytes)
        for _ in range(3):
            T.tent_reset(ctx, h_fb, stream)
            torch.cuda.synchronize(dev)
            T.tent_get_timings(ctx)
            st_d, dinfo = T.tent_plan_dispatch(ctx, h_fb, w.rails, dparams, None, True, stream)
            tm_d = T.tent_get_timings(ctx)
            disp_ms.append(sum(tm_d[k][0] for k in ("extent_scan", "slice_scan", "expand", "bind")))
        T.tent_reset(ctx, h_fb, stream)

    if "bounded" in legs and w.payload >= (64 << 20):
        # Bounded, pipelined staging (Section 4.1), outside the timed region: the same batch through an arena of
        # one eighth of the payload (rounded to MiB) and through a 256 MiB arena, chunk after chunk.
        ctx_b = T.tent_create(w.slice_bytes, arena.data_ptr(), arena.numel(),
                              T.TENT_FLAG_PROFILE | T.TENT_FLAG_BOUNDED_STAGING)
        T.tent_register_segment(ctx_b, src.data_ptr(), src.numel())
        T.tent_register_segment(ctx_b, dst.data_ptr(), dst.numel())
        h_b = T.tent_declare(ctx_b, w.src_ptr, w.src_ext, w.dst_ptr, w.dst_ext)
        for chunk in sorted({max(1, (w.payload // 8) >> 20) << 20, 256 << 20, 128 << 20}, reverse=True):
            for slots in (1, 2):
                if slots * (chunk + 256 * R) > arena.numel() or chunk >= w.payload:
                    continue
                best = None
                for _ in range(3):
                    T.tent_reset(ctx_b, h_b, stream)
                    T.tent_plan(ctx_b, h_b, w.rails, want_info=False, stream=stream)
                    torch.cuda.synchronize(dev)
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record()
                    T.tent_execute_bounded(ctx_b, h_b, chunk, stream, slots=slots)
                    e1.record()
                    torch.cuda.synchronize(dev)
                    ms = e0.elapsed_time(e1)
                    best = ms if best is None else min(best, ms)
                assert T.tent_poll(ctx_b, h_b, stream) == 0
                bounded.append({"slot_MiB": chunk >> 20, "slots": slots, "chunks": -(-w.payload // chunk),
                                "execute_ms": round(best, 4), "GBps": round(4 * w.payload / (best * 1e-3) / 1e9, 2)})
        T.tent_destroy(ctx_b)

    log("dispatch / bounded legs done")
    if "graph" in legs:
        # One whole cycle (reset, plan, execute) recorded into a HIP graph and replayed, outside the timed region:
        # what is left of the step when the host's launch work is taken out.
        ctx_g = T.tent_create(w.slice_bytes, arena.data_ptr(), arena.numel(), 0)        # no event timers inside a capture
        T.tent_register_segment(ctx_g, src.data_ptr(), src.numel())
        T.tent_register_segment(ctx_g, dst.data_ptr(), dst.numel())
        h_g = T.tent_declare(ctx_g, w.src_ptr, w.src_ext, w.dst_ptr, w.dst_ext)
        T.tent_plan(ctx_g, h_g, w.rails, want_info=False, stream=stream)
        T.tent_execute(ctx_g, h_g, stream)
        torch.cuda.synchronize(dev)
        try:
            side = torch.cuda.Stream(dev)
            side.wait_stream(stream)
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.stream(side):
                with torch.cuda.graph(graph, stream=side):
                    cap = torch.cuda.current_stream(dev)
                    T.tent_reset(ctx_g, h_g, cap)
                    T.tent_plan(ctx_g, h_g, w.rails, want_info=False, stream=cap)
                    T.tent_execute(ctx_g, h_g, cap)
            torch.cuda.synchronize(dev)
            graph.replay()
            torch.cuda.synchronize(dev)
            n_rep = 5
            g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            g0.record()
            for _ in range(n_rep):
                graph.replay()
            g1.record()
            torch.cuda.synchronize(dev)
            graph_ms = g0.elapsed_time(g1) / n_rep
            assert T.tent_poll(ctx_g, h_g, stream) == 0
            del graph
        except RuntimeError:
            graph_ms = None
        T.tent_destroy(ctx_g)

    # Plain copy of known size (1 GiB read + 1 GiB written by one elementwise kernel), outside the
    # timed region: the practical copy ceiling of the box and the reference dispatch that scales
    # hardware byte counters when this script runs under a counter-collecting profiler.
    cal_n = min(1 << 30, src.numel(), dst.numel())
    cal_in, cal_out = src[:cal_n], arena[:cal_n]
    torch.bitwise_not(cal_in, out=cal_out)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    torch.bitwise_not(cal_in, out=cal_out)
    ev1.record()
    torch.cuda.synchronize(dev)
    plain_copy_GBps = 2 * cal_n / (ev0.elapsed_time(ev1) * 1e-3) / 1e9

    # plan stages are timed on the single-stream pass, where nothing runs beside them
    plan_ms = sum(tm_single[n][0] for n in ("extent_scan", "slice_scan", "expand", "compact", "bind")) / max(1, args.steps)
    gather_ms, gather_n = tm["gather"]
    scatter_ms, scatter_n = tm["scatter"]
    gather_avg = gather_ms / max(1, gather_n)
    scatter_avg = scatter_ms / max(1, scatter_n)
    ms_per_step = elapsed * 1e3 / args.steps
    value = 4 * w.payload / (ms_per_step * 1e-3) / 1e9
    # the roofline entry describes the slower of the two copy launches
    dom, dom_avg = ("scatter", scatter_avg) if scatter_avg >= gather_avg else ("gather", gather_avg)
    achieved = 2 * w.payload / (dom_avg * 1e-3) / 1e9
    run.close()

    # The other workloads, each through the same two timed passes (fewer steps), in the same pools.
    configs = []
    for wo in others:
        steps_o, warm_o = max(3, min(args.steps, 10)), 2
        ro = Run(T, W, torch, dev, wo, pools, steps_o, warm_o, T.TENT_FLAG_PROFILE)
        e1, t1 = ro.timed_pass(ro.step_single)
        ro.reset_all()
        e2, t2 = ro.timed_pass(lambda h: ro.step_pipelined(h, plan_stream))
        rec = {"workload": wo.name}
        rec.update(summarize(wo, ro.n_slices, steps_o, e1, t1, e2, t2))
        # plans alternating between two plan streams: the one-wavefront binding chains of two later steps side by side
        ro.reset_all()
        pair, turn_o = [plan_stream, plan_stream2], [0]

        def step_two_plan_streams_o(h):
            turn_o[0] += 1
            ro.step_pipelined(h, pair[turn_o[0] & 1])

        e3, _ = ro.timed_pass(step_two_plan_streams_o)
        ms3 = e3 * 1e3 / steps_o
        rec["ms_per_step_two_plan_streams"] = round(ms3, 4)
        rec["pct_of_hbm_peak_two_plan_streams"] = round(100 * 4 * wo.payload / (ms3 * 1e-3) / 1e9 / HBM_PEAK_GBPS, 2)
        rec["declare_host_ms"] = round(ro.declare_host_ms, 3)
        rec["verified"] = ro.verify()
        configs.append(rec)
        ro.close()
        log(f"config {wo.name} done")

    out = {
        "metric": "slice gather/scatter GB/s (% of HBM peak) + slices planned/sec, 1 MI355X",
        "value": round(value, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u8", "data": "synthetic",
        "config": {"workload": args.workload, "payload_bytes": w.payload, "n_desc": w.n_desc,
                   "n_extents": int(w.src_ext.shape[0]), "n_slices": n_slices, "slice_bytes": w.slice_bytes,
                   "n_rails": int(w.rails.shape[0]), "binding": "serial" if args.serial_binding else "default",
                   "streams": "single" if args.single_stream else
                              "two: plan of step k+1 overlaps execute of step k; every step plans and executes its own batch",
                   "placement": {"mode": layout.mode, "note": layout.note,
                                 "reserved_GiB": round(layout.reserved_bytes / 2**30, 1),
                                 "region_of_each_%d_GiB_chunk" % (placement.CHUNK >> 30): "".join(str(x) for x in layout.labels),
                                 "offsets_GiB": [round(o / 2**30, 2) for o in layout.offsets],
                                 "probes": layout.probes, "verified": layout.verified}},
        "verified": verified,
        "ms_per_step_single_stream": round(elapsed_single * 1e3 / args.steps, 4),
        "ms_per_step_two_streams": round(elapsed_piped * 1e3 / args.steps, 4),
        "ms_per_step_two_plan_streams": None if elapsed_deep is None else round(elapsed_deep * 1e3 / args.steps, 4),
        "ms_per_step_with_declare": None if with_declare is None else with_declare["ms_per_step"],
        "with_declare": with_declare,
        "pct_of_hbm_peak": round(100 * value / HBM_PEAK_GBPS, 2),
        "slices_planned_per_s": round(n_slices / (plan_ms * 1e-3), 1) if plan_ms > 0 else None,
        "slices_planned_per_s_concurrent": None if concurrent_plan_s is None else
                                           {"streams": len(many), "batches": len(batches),
                                            "value": round(n_slices * len(batches) / concurrent_plan_s, 1)},
        "stage_ms": {k: round(v[0] / max(1, args.steps), 4) for k, v in tm.items()},
        "stage_ms_single_stream": {k: round(v[0] / max(1, args.steps), 4) for k, v in tm_single.items()},
        "execute_GBps": round(4 * w.payload / ((gather_avg + scatter_avg) * 1e-3) / 1e9, 2),
        "declare_ms": round(declare_ms, 3),
        "configs": configs,
        "feedback": {"window_slices": n_slices, "ms_per_window": round(fb_ms / max(1, fb_n), 4),
                     "bytes_per_slice": 17},
        "recovery": {"failed_rail": fastest, "retried_slices": n_retried, "replanned_slices": n_slices,
                     "replan_ms": round(min(rec_ms), 4) if rec_ms else None},
        "replanning": replanning,
        "dispatch": None if dinfo is None else
                    {"theta_slices": 4, "mice": int(dinfo.n_mice), "elephants": int(dinfo.n_elephant),
                     "plan_ms": round(min(disp_ms), 4), "slices_per_s": round(n_slices / (min(disp_ms) * 1e-3), 1)},
        "bounded_staging": bounded,
        "graph_replay_ms_per_step": None if graph_ms is None else round(graph_ms, 4),
        "plain_copy_GBps": round(plain_copy_GBps, 2),
        "roofline": {"bound": "hbm", "kernel": "ordered_copy_kernel<%s>" % ("true" if dom == "gather" else "false"), "achieved": round(achieved, 2),
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
                     "traffic": measured_traffic(args.workload, dom),
                     "algorithmic_bytes_per_launch": 2 * w.payload,
                     "avg_launch_ms": round(dom_avg, 4),
                     "gather_GBps": round(2 * w.payload / (gather_avg * 1e-3) / 1e9, 2),
                     "scatter_GBps": round(2 * w.payload / (scatter_avg * 1e-3) / 1e9, 2)},
    }
    del src, dst, arena, pools, pools3, run
    if not args.no_cpu_baseline:
        torch.cuda.empty_cache()
        log("GPU part done; CPU baseline")
        out["cpu_baseline"] = cpu_baseline(args.workload)
    print(json.dumps(out))


if __name__ == "__main__":
    sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
    main()
