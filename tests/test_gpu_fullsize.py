"""Full-size GPU parity on the benchmark's launch configuration.

The plan (slice table, rails, staging offsets, per-rail totals) is compared with the CPU oracle in
full.  Bytes are compared two ways: (1) for a sample of transfers the oracle moves the bytes on the
host (source extents fetched from the device pool) and every destination and staging byte of those
transfers must match; (2) for every transfer, DST_j[x] == SRC_j[x] is checked on the device with
plain torch indexing (the definition of the result, independent of slices and rails).
"""
import gc

import numpy as np
import pytest

from paper_2604_00368_amd import workloads as W

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def H():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import gpu_harness
    return gpu_harness


def device_definition_check(w, src, dst, chunk_extents=1 << 15):
    """DST_j[x] == SRC_j[x] for all j, x, when source and destination extents pair up one to one."""
    assert np.array_equal(w.src_ptr, w.dst_ptr) and np.array_equal(w.src_ext["len"], w.dst_ext["len"])
    lens = np.unique(w.src_ext["len"])
    if lens.shape[0] == 1:                       # uniform pages: gather both sides as rows
        page = int(lens[0])
        assert (w.src_ext["off"] % page == 0).all() and (w.dst_ext["off"] % page == 0).all()
        sv, dv = src.view(-1, page), dst.view(-1, page)
        for lo in range(0, w.src_ext.shape[0], chunk_extents):
            si = torch.from_numpy((w.src_ext["off"][lo:lo + chunk_extents] // page).astype(np.int64)).to(src.device)
            di = torch.from_numpy((w.dst_ext["off"][lo:lo + chunk_extents] // page).astype(np.int64)).to(src.device)
            assert torch.equal(sv[si], dv[di]), f"extent chunk at {lo}"
    else:                                        # few large extents: compare slice by slice
        for se, de in zip(w.src_ext, w.dst_ext):
            a = src[int(se["off"]):int(se["off"]) + int(se["len"])]
            b = dst[int(de["off"]):int(de["off"]) + int(de["len"])]
            assert torch.equal(a, b)


def sampled_bytes_check(oracle, w, s, b, eng, sample, ids_filter=None):
    """Oracle moves the sampled transfers on the host; device bytes of those transfers must match."""
    src_h = np.zeros(w.seg_bytes[0], dtype=np.uint8)          # untouched pages are never committed
    dst_h = np.zeros(w.seg_bytes[1], dtype=np.uint8)
    stg_h = np.zeros(w.staging_bytes, dtype=np.uint8)
    for j in sample:
        for e in w.src_ext[w.src_ptr[j]:w.src_ptr[j + 1]]:
            o, n = int(e["off"]), int(e["len"])
            src_h[o:o + n] = eng.src[o:o + n].cpu().numpy()
    ids = np.concatenate([np.arange(s.first[j], s.first[j + 1], dtype=np.uint32) for j in sample])
    oracle.execute(w, s, b, [src_h, dst_h], stg_h, ids=np.ascontiguousarray(ids))
    for j in sample:
        for e in w.dst_ext[w.dst_ptr[j]:w.dst_ptr[j + 1]]:
            o, n = int(e["off"]), int(e["len"])
            assert np.array_equal(eng.dst[o:o + n].cpu().numpy(), dst_h[o:o + n]), (j, o)
    for i in ids:
        o, n = int(b.base[b.rail[i]] + b.stage_off[i]), int(s.len[i])
        assert np.array_equal(eng.arena[o:o + n].cpu().numpy(), stg_h[o:o + n]), ("staging", int(i))


def pick_sample(w, k, seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    D = w.n_desc
    ext_count = np.diff(w.src_ptr.astype(np.int64))
    small = np.nonzero(ext_count <= 600)[0]
    picks = set(rng.choice(small, size=min(k, small.shape[0]), replace=False).tolist())
    picks.update([0, D - 1])
    return sorted(picks)


def full_config(name):
    if name == "many_small_x6":
        return W.many_small(layers=6)
    return W.CONFIGS[name]()


@pytest.mark.parametrize("name", ["kv_migration", "rl_params", "many_small", "many_small_x6"])
def test_full_size_config(H, oracle, name):
    from paper_2604_00368_amd import binding as T
    print("full-size", name, flush=True)
    w = full_config(name)
    s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
    b = oracle.bind(s.len, w.rails)
    eng = H.Engine(w, flags=T.TENT_FLAG_PROFILE)             # pools filled on the device, as in bench.py
    try:
        eng.declare()
        st, _ = eng.plan(want_info=False)
        assert st == 0
        eng.execute()
        print("  executed", s.n, "slices", flush=True)
        H.assert_plan_equal(eng.table(), s, b)
        assert T.tent_poll(eng.ctx, eng.batch, eng.stream) == 0
        device_definition_check(w, eng.src, eng.dst)
        print("  definition check done", flush=True)
        if name == "rl_params":
            sample = [1, 6, 2, 3, w.n_desc - 1]               # norms (8 KiB) and 8-32 MiB projections
        else:
            sample = pick_sample(w, 12, seed=len(name))
        sampled_bytes_check(oracle, w, s, b, eng, sample)
    finally:
        eng.close()
        del eng
        gc.collect()
        torch.cuda.empty_cache()


def test_full_size_config_in_the_benchmarks_pool_layout(H, oracle):
    """Config 2 with the pools where bench.py puts them: carved from one reservation by measured region."""
    from paper_2604_00368_amd import binding as T
    from paper_2604_00368_amd import placement
    print("full-size kv_migration, pools carved by region", flush=True)
    w = full_config("kv_migration")
    gc.collect()
    torch.cuda.empty_cache()
    dev = torch.device("cuda:0")
    src, arena, dst, lay = placement.place_pools(dev, w.seg_bytes[0], w.staging_bytes, w.seg_bytes[1])
    print("  layout:", lay.mode, lay.note, "".join(str(x) for x in lay.labels), [o >> 30 for o in lay.offsets], flush=True)
    if lay.mode != "regions":
        # bench.py would run in these very pools (ordinary allocations): the parity check is the same and is
        # not skipped; the reason is kept in the test's output
        import warnings
        warnings.warn("no region layout in this process, parity checked in ordinary allocations: " + lay.note)
    s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
    b = oracle.bind(s.len, w.rails)
    eng = H.Engine(w, flags=T.TENT_FLAG_PROFILE, pools=(src, arena, dst))
    try:
        eng.declare()
        st, _ = eng.plan(want_info=False)
        assert st == 0
        eng.execute()
        H.assert_plan_equal(eng.table(), s, b)
        assert T.tent_poll(eng.ctx, eng.batch, eng.stream) == 0
        device_definition_check(w, eng.src, eng.dst)
        sampled_bytes_check(oracle, w, s, b, eng, pick_sample(w, 8, seed=5))
    finally:
        eng.close()
        del eng, src, arena, dst
        gc.collect()
        torch.cuda.empty_cache()


def test_full_size_replanning(H, oracle):
    from paper_2604_00368_amd import binding as T
    print("full-size replanning", flush=True)
    w = W.replanning()
    s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
    records, left = oracle.run_epochs(w, s)                   # plan and retire only: no host byte pools
    assert left.shape[0] == 0
    eng = H.Engine(w, flags=T.TENT_FLAG_PROFILE)
    try:
        eng.declare()
        for e, (rec, ep) in enumerate(zip(records, list(w.epochs) + [w.drain])):
            st, info = eng.plan(rails=ep.rails)
            assert st == 0 and info.n_slices == rec["pending"].shape[0]
            tab = eng.table()
            pend = rec["pending"]
            assert np.array_equal(np.nonzero(tab["state"] != 2)[0], pend)
            if rec["rail"] is not None:
                assert np.array_equal(tab["rail"][pend], rec["rail"])
                assert np.array_equal(tab["stage_off"][pend], rec["stage_off"])
                R = ep.rails.shape[0]
                assert list(info.rail_bytes)[:R] == rec["T"].tolist()
            n_done = T.tent_sim_advance(eng.ctx, eng.batch, ep.budget, eng.stream)
            assert n_done == rec["done_ids"].shape[0]
            eng.execute()
            print("  epoch", e, "pending", pend.shape[0], "done", n_done, flush=True)
        assert T.tent_poll(eng.ctx, eng.batch, eng.stream) == 0
        device_definition_check(w, eng.src, eng.dst)
    finally:
        eng.close()
        del eng
        gc.collect()
        torch.cuda.empty_cache()


def test_full_size_replanning_plan_beside_copies(H, oracle):
    """Config 4 the way the benchmark runs it: plans and the rail simulator on a second stream, executes on
    the first, no host wait between an execute and the next plan."""
    from paper_2604_00368_amd import binding as T
    print("full-size replanning, plans beside copies", flush=True)
    w = W.replanning()
    s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
    records, left = oracle.run_epochs(w, s)
    assert left.shape[0] == 0
    eng = H.Engine(w)
    try:
        eng.declare()
        side = torch.cuda.Stream(eng.dev)
        side.wait_stream(eng.stream)
        for e, (rec, ep) in enumerate(zip(records, list(w.epochs) + [w.drain])):
            st, info = T.tent_plan(eng.ctx, eng.batch, ep.rails, True, side)
            assert st == 0 and info.n_slices == rec["pending"].shape[0]
            if rec["T"] is not None:
                R = ep.rails.shape[0]
                assert list(info.rail_bytes)[:R] == rec["T"].tolist()
            n_done = T.tent_sim_advance(eng.ctx, eng.batch, ep.budget, side)
            assert n_done == rec["done_ids"].shape[0]
            T.tent_execute(eng.ctx, eng.batch, eng.stream)
            print("  epoch", e, "done", n_done, flush=True)
        assert T.tent_poll(eng.ctx, eng.batch, eng.stream) == 0
        torch.cuda.synchronize(eng.dev)
        device_definition_check(w, eng.src, eng.dst)
    finally:
        eng.close()
        del eng
        gc.collect()
        torch.cuda.empty_cache()


def test_full_size_closed_loop(H, oracle):
    # config 4 with the telemetry loop closed (plan, rails, latencies, probes and estimates per epoch)
    import test_gpu_parity as P
    print("full-size closed loop", flush=True)
    w = W.replanning()
    params = W.make_probe_params(2 * w.rails["bw_MBps"].astype(np.uint64), ewma_q8=64)
    P.run_closed_loop_and_compare(H, oracle, w, params, bytes_too=False)
    gc.collect()
    torch.cuda.empty_cache()


def test_full_size_faulty_rails(H, oracle):
    # config 4 with hard errors injected, the telemetry loop closed and the health monitor in charge of the
    # rails' states: every window's plan (rotation pass included), failures, probes and monitor records
    # against the oracle; at the end every destination byte by the plain definition
    import test_gpu_resilience as Rz
    print("full-size faulty rails", flush=True)
    w = W.replanning()
    R = w.rails.shape[0]
    params = W.make_probe_params(2 * w.rails["bw_MBps"].astype(np.uint64), ewma_q8=64)
    fails, cong = W.failure_schedule(12, len(w.epochs), R)
    recs = Rz.run_resilient_and_compare(H, oracle, w, params, W.make_monitor_params(), fails, cong, bytes_too=False,
                                        final_check=lambda eng: device_definition_check(w, eng.src, eng.dst))
    assert max(int((r["retry"][r["pending"]] > 0).sum()) for r in recs) > 4 * 1024
    gc.collect()
    torch.cuda.empty_cache()


@pytest.mark.parametrize("name", ["kv_migration", "many_small_x6"])
def test_full_size_dispatch(H, oracle, name):
    # Algorithm 1 request by request at full size: three priority windows, plan compared in full each window,
    # at the end every destination byte by the plain definition
    import test_gpu_dispatch as Dz
    print("full-size dispatch", name, flush=True)
    w = full_config(name)
    prio = W.make_priorities(21, w.n_desc)
    done, modes = Dz.dispatch_windows_and_compare(
        H, oracle, w, theta=16 * w.slice_bytes, gamma_q8=26, prio=prio, windows=[0, 1, 2], bytes_too=False,
        final_check=lambda eng, done: device_definition_check(w, eng.src, eng.dst))
    assert done.all() and 2 in modes
    gc.collect()
    torch.cuda.empty_cache()


def test_full_size_bounded_staging(H, oracle):
    # config 2 through an arena of one sixteenth of the payload: plan in full against the oracle, every
    # destination byte by the plain definition, sampled transfers against the oracle's bounded execute
    from paper_2604_00368_amd import binding as T
    print("full-size bounded staging", flush=True)
    w = full_config("kv_migration")
    R = w.rails.shape[0]
    chunk = 1280 << 20
    cap = chunk + 256 * R
    s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
    b = oracle.bind(s.len, w.rails)
    eng = H.Engine(w, flags=T.TENT_FLAG_PROFILE | T.TENT_FLAG_BOUNDED_STAGING, arena_bytes=cap)
    try:
        eng.declare()
        st, _ = eng.plan(want_info=False)
        assert st == 0
        T.tent_execute_bounded(eng.ctx, eng.batch, chunk, eng.stream)
        torch.cuda.synchronize()
        H.assert_plan_equal(eng.table(), s, b)
        assert T.tent_poll(eng.ctx, eng.batch, eng.stream) == 0
        device_definition_check(w, eng.src, eng.dst)
        # destination bytes of a few transfers, moved by the oracle on the host
        sample = pick_sample(w, 6, seed=5)
        src_h = np.zeros(w.seg_bytes[0], dtype=np.uint8)
        dst_h = np.zeros(w.seg_bytes[1], dtype=np.uint8)
        for j in sample:
            for e in w.src_ext[w.src_ptr[j]:w.src_ptr[j + 1]]:
                o, n = int(e["off"]), int(e["len"])
                src_h[o:o + n] = eng.src[o:o + n].cpu().numpy()
        ids = np.concatenate([np.arange(s.first[j], s.first[j + 1], dtype=np.uint32) for j in sample])
        stg_h = np.zeros(cap, dtype=np.uint8)
        assert oracle.execute_bounded(w, s, b, [src_h, dst_h], stg_h, chunk, ids=np.ascontiguousarray(ids)) == 0
        for j in sample:
            for e in w.dst_ext[w.dst_ptr[j]:w.dst_ptr[j + 1]]:
                o, n = int(e["off"]), int(e["len"])
                assert np.array_equal(eng.dst[o:o + n].cpu().numpy(), dst_h[o:o + n]), (j, o)
    finally:
        eng.close()
        del eng
        gc.collect()
        torch.cuda.empty_cache()


def test_maximum_slice_and_extent_sizes(H, oracle):
    # the largest slice size the library accepts (2^31 bytes) and extents close to the 32-bit length limit:
    # one transfer of 3 GiB + 12 KiB (two slices: 2 GiB and the rest) next to a 4 KiB one; plan and every byte
    print("maximum sizes", flush=True)
    GiB = 1 << 30
    S = 1 << 31
    big = 3 * GiB + 12288
    ptr_s = np.array([0, 2, 3], dtype=np.uint32)
    ptr_d = np.array([0, 3, 4], dtype=np.uint32)
    se = W._extents(W.SRC_SEG, [4096, 8192 + big - 1 * GiB - 8192, 0], [big - 1 * GiB - 8192, 1 * GiB + 8192, 4096])
    # destination: three extents (4 GiB - 4 KiB would not fit a u32 length, so 1.5 GiB + 1.5 GiB + 12 KiB), then 4 KiB
    de = W._extents(W.DST_SEG, [8192, 8192 + 3 * GiB // 2, 8192 + 3 * GiB, 0], [3 * GiB // 2, 3 * GiB // 2, 12288, 4096])
    pool = 8192 + big + 4096
    rails = W.make_rails([50000, 400000, 25000])
    w = W.Workload("max_sizes", 0, S, [pool, pool], ptr_s, se, ptr_d, de, rails, "u8")
    assert w.payload == big + 4096
    g = torch.Generator(device="cuda")
    g.manual_seed(77)
    src_t = torch.randint(0, 256, (pool,), dtype=torch.uint8, device="cuda", generator=g)
    src = src_t.cpu().numpy()
    dst0 = np.zeros(pool, dtype=np.uint8)
    s = oracle.split(w.src_ptr, w.src_ext, S)
    assert s.n == 3 and s.len.tolist() == [S, big - S, 4096]
    b = oracle.bind(s.len, w.rails)
    dst_want = dst0.copy()
    staging_want = np.zeros(w.staging_bytes, dtype=np.uint8)
    oracle.execute(w, s, b, [src, dst_want], staging_want)
    eng = H.Engine(w, src, dst0)
    try:
        del src_t
        eng.declare()
        st, info = eng.plan()
        assert st == 0
        H.assert_plan_equal(eng.table(), s, b, info)
        eng.execute()
        assert np.array_equal(eng.dst.cpu().numpy(), dst_want)
        assert np.array_equal(eng.arena.cpu().numpy(), staging_want)
    finally:
        eng.close()
        del eng
        gc.collect()
        torch.cuda.empty_cache()
