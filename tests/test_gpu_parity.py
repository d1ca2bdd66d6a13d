"""GPU parity: the HIP engine (through its C ABI) against the CPU oracle, bit for bit."""
import numpy as np
import pytest

from helpers import expected_destination
from paper_2604_00368_amd import workloads as W

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def H():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import gpu_harness
    return gpu_harness


def run_and_compare(H, oracle, w, flags=0, arena_skew=0):
    src = W.fill_numpy(w, 0)
    dst0 = W.fill_numpy(w, 1)
    s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
    b = oracle.bind(s.len, w.rails)
    dst_want = dst0.copy()
    staging_want = np.zeros(w.staging_bytes, dtype=np.uint8)
    oracle.execute(w, s, b, [src, dst_want], staging_want)
    with H.Engine(w, src, dst0, flags=flags, arena_skew=arena_skew) as eng:
        eng.declare()
        st, info = eng.plan()
        assert st == 0
        H.assert_plan_equal(eng.table(), s, b, info)
        eng.execute()
        assert np.array_equal(eng.dst.cpu().numpy(), dst_want)
        assert np.array_equal(eng.arena.cpu().numpy(), staging_want)
        assert np.array_equal(eng.src.cpu().numpy(), src)
        tab = eng.table()
        assert (tab["state"] == 2).all()


@pytest.mark.parametrize("name", ["tiny", "kv_migration", "rl_params", "many_small"])
def test_small_configs_bit_exact(H, oracle, name):
    print("case", name, flush=True)
    run_and_compare(H, oracle, W.small_variant(name))


@pytest.mark.parametrize("seed", range(8))
def test_ragged_bit_exact(H, oracle, seed):
    print("ragged seed", seed, flush=True)
    S = [1, 17, 4096, 5000, 65536, 4099, 333, 16][seed]
    align = [1, 1, 1, 1, 1, 4, 1, 16][seed]
    run_and_compare(H, oracle, W.ragged(seed, slice_bytes=S, n_desc=12, max_len=40_000, max_ext=900, align=align))


@pytest.mark.parametrize("S", [1024, 3072, 4096, 6144, 8192 + 2048, 65536 + 1024])
def test_tile_sizes_and_partial_blocks(H, oracle, S):
    # slice sizes that give 1 KiB / 2 KiB / 4 KiB tiles, partial last blocks and extent boundaries inside blocks
    print("tile case S", S, flush=True)
    w = W.ragged(7, slice_bytes=S, n_desc=10, max_len=300_000, max_ext=20_000, align=1024)
    run_and_compare(H, oracle, w)
    w = W.many_small(n_req=24, layers=2, slice_bytes=S)
    run_and_compare(H, oracle, w)


def test_serial_binding_flag_matches_oracle(H, oracle):
    from paper_2604_00368_amd import binding as T
    print("serial binding", flush=True)
    for name in ["tiny", "many_small", "kv_migration"]:
        run_and_compare(H, oracle, W.small_variant(name), flags=T.TENT_FLAG_SERIAL_BINDING)


def _runs_workload(rng, kind):
    """Transfers that produce runs of equal-length slices of arbitrary length and count, with tails."""
    S = int(rng.integers(1, 1 << int(rng.integers(4, 17))))
    lens = []
    for _ in range(int(rng.integers(1, 12))):
        m = int(rng.integers(1, 200 if kind != 5 else 1500))
        if rng.random() < 0.6:
            lens.append(m * S + (int(rng.integers(1, S)) if (S > 1 and rng.random() < 0.7) else 0))
        else:
            lens += [int(rng.integers(1, S + 1))] * m          # m short transfers: a run of equal tails
    lens = np.array(lens, dtype=np.uint64)
    off = np.concatenate([[0], np.cumsum(lens)[:-1]]).astype(np.uint64)
    ptr = np.arange(len(lens) + 1, dtype=np.uint32)
    total = int(lens.sum())
    R = int(rng.integers(1, 20))
    bw = rng.integers(1000, 400000, size=R)
    lat = rng.integers(0, 20000, size=R)
    queued = rng.integers(0, 1 << 24, size=R)
    b1 = rng.integers(128, 1024, size=R)
    pen = rng.integers(26, 1280, size=R)
    if kind == 1:                                              # identical rails: every cost ties
        bw[:], lat[:], queued[:], b1[:], pen[:] = 50000, 5000, 0, 256, 256
    if kind == 2:                                              # cost grows by less than 1 ps per slot
        bw, lat = rng.integers(3_000_000_000, 4_000_000_000, size=R), np.zeros(R, dtype=np.int64)
    if kind == 3:                                              # latencies spread over the whole range
        lat = rng.integers(0, 2**32 - 1, size=R)
    if kind == 4:                                              # long queues
        queued = rng.integers(0, 1 << 31, size=R)                # (max A + payload) * max c1 stays below 2^63
    if kind in (6, 7, 8):
        # many transfers on rails that start level with each other (the chain's short path and its near keys);
        # kind 7: some rails behind queues so long that they join late or never; kind 8: up to 64 rails
        S = int(rng.choice([4096, 16384, 65536])) + (int(rng.integers(0, 64)) if rng.random() < 0.3 else 0)
        pages = rng.integers(2, 80, size=int(rng.integers(60, 260)))
        page = int(rng.choice([2048, 18432, 32768]))
        lens = (pages * page).astype(np.uint64)
        off = np.concatenate([[0], np.cumsum(lens)[:-1]]).astype(np.uint64)
        ptr = np.arange(len(lens) + 1, dtype=np.uint32)
        total = int(lens.sum())
        R = int(rng.integers(2, 17)) if kind != 8 else int(rng.integers(17, 65))
        bw = rng.choice([25000, 50000, 100000, 400000], size=R)
        lat = np.full(R, 5000)
        queued = rng.integers(0, 1 << 12, size=R)
        b1, pen = np.full(R, 256), np.full(R, 256)
        if kind == 7:
            far = rng.random(R) < 0.4
            queued = np.where(far, rng.integers(1 << 20, 1 << 30, size=R), queued)
    u = rng.random(R)
    health = np.where(u < 0.2, 2, np.where(u < 0.4, 1, 0)).astype(np.uint8)       # excluded / degraded / healthy
    if (health == 2).all():
        health[0] = 0
    if kind == 3:
        pen = np.minimum(pen, 500)               # doubled coefficients of degraded rails must stay in range
    rails = W.make_rails(bw, lat_ns=lat, queued=queued, health=health, beta1_q8=b1, penalty_q8=pen)
    return W.Workload("runs", 0, S, [total, total], ptr, W._extents(0, off, lens), ptr.copy(),
                      W._extents(1, off, lens), rails, "u8")


@pytest.mark.parametrize("kind", range(9))
def test_run_parallel_binding_matches_oracle(H, oracle, kind):
    # plan-only: degenerate telemetry (ties, sub-picosecond steps, huge latencies and queues)
    rng = np.random.Generator(np.random.PCG64(1000 + kind))
    for trial in range(25 if kind < 6 else 12):
        w = _runs_workload(rng, kind)
        print("runs kind", kind, "trial", trial, "S", w.slice_bytes, "D", w.n_desc, "R", w.rails.shape[0], flush=True)
        s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
        b = oracle.bind(s.len, w.rails)
        with H.Engine(w, np.zeros(w.seg_bytes[0], np.uint8), np.zeros(w.seg_bytes[1], np.uint8)) as eng:
            eng.declare()
            st, info = eng.plan()
            assert st == 0
            H.assert_plan_equal(eng.table(), s, b, info)


def run_epochs_and_compare(H, oracle, w, flags=0):
    from paper_2604_00368_amd import binding as T
    src = W.fill_numpy(w, 0)
    dst0 = W.fill_numpy(w, 1)
    s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
    dst_want = dst0.copy()
    staging_want = np.zeros(w.staging_bytes, dtype=np.uint8)
    records, left = oracle.run_epochs(w, s, [src, dst_want], staging_want)
    assert left.shape[0] == 0
    with H.Engine(w, src, dst0, flags=flags) as eng:
        eng.declare()
        done_so_far = np.zeros(s.n, dtype=bool)
        for e, (rec, ep) in enumerate(zip(records, list(w.epochs) + [w.drain])):
            print("epoch", e, "pending", rec["pending"].shape[0], flush=True)
            st, info = eng.plan(rails=ep.rails)
            assert st == rec["status"] == 0
            assert info.n_slices == rec["pending"].shape[0] == info.n_pending_before
            tab = eng.table()
            pend = rec["pending"]
            assert np.array_equal(np.nonzero(tab["state"] != 2)[0], pend)           # pending set
            if rec["rail"] is not None:
                assert np.array_equal(tab["rail"][pend], rec["rail"])
                assert np.array_equal(tab["stage_off"][pend], rec["stage_off"])
            if rec["T"] is not None:
                R = ep.rails.shape[0]
                assert list(info.rail_bytes)[:R] == rec["T"].tolist()
                assert list(info.stage_base)[:R] == rec["base"].tolist()
            n_done = T.tent_sim_advance(eng.ctx, eng.batch, ep.budget, eng.stream)
            assert n_done == rec["done_ids"].shape[0]
            tab = eng.table()
            assert np.array_equal(np.nonzero(tab["state"] == 1)[0], rec["done_ids"])  # done set of the epoch
            eng.execute()
            done_so_far[rec["done_ids"]] = True
            assert T.tent_poll(eng.ctx, eng.batch, eng.stream) == int((~done_so_far).sum())
        assert done_so_far.all()
        assert np.array_equal(eng.dst.cpu().numpy(), dst_want)
        assert np.array_equal(eng.arena.cpu().numpy(), staging_want)


def test_replanning_epochs_bit_exact(H, oracle):
    from paper_2604_00368_amd import binding as T
    run_epochs_and_compare(H, oracle, W.small_variant("replanning"))
    run_epochs_and_compare(H, oracle, W.small_variant("replanning"), flags=T.TENT_FLAG_SERIAL_BINDING)


def run_epochs_plan_beside_copies(H, oracle, w, flags=0):
    """The same epochs with plans and the rail simulator on a second stream and executes on the first, and no
    wait of the host's between an execute and the next plan: the library itself orders a re-plan after the
    execute's bookkeeping, beside its copies."""
    import torch
    from paper_2604_00368_amd import binding as T
    src = W.fill_numpy(w, 0)
    dst0 = W.fill_numpy(w, 1)
    s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
    dst_want = dst0.copy()
    staging_want = np.zeros(w.staging_bytes, dtype=np.uint8)
    records, left = oracle.run_epochs(w, s, [src, dst_want], staging_want)
    assert left.shape[0] == 0
    with H.Engine(w, src, dst0, flags=flags) as eng:
        eng.declare()
        side = torch.cuda.Stream(eng.dev)
        side.wait_stream(eng.stream)                      # the pools were filled on the first stream
        for e, (rec, ep) in enumerate(zip(records, list(w.epochs) + [w.drain])):
            st, info = T.tent_plan(eng.ctx, eng.batch, ep.rails, True, side)
            assert st == rec["status"] == 0
            assert info.n_slices == rec["pending"].shape[0] == info.n_pending_before
            if rec["T"] is not None:
                R = ep.rails.shape[0]
                assert list(info.rail_bytes)[:R] == rec["T"].tolist()
                assert list(info.stage_base)[:R] == rec["base"].tolist()
            n_done = T.tent_sim_advance(eng.ctx, eng.batch, ep.budget, side)   # waits for the second stream only
            assert n_done == rec["done_ids"].shape[0]
            T.tent_execute(eng.ctx, eng.batch, eng.stream)
        assert T.tent_poll(eng.ctx, eng.batch, eng.stream) == 0
        torch.cuda.synchronize(eng.dev)
        tab = eng.table()
        assert (tab["state"] == 2).all()
        assert np.array_equal(eng.dst.cpu().numpy(), dst_want)
        assert np.array_equal(eng.arena.cpu().numpy(), staging_want)


def test_replanning_epochs_plan_beside_copies(H, oracle):
    from paper_2604_00368_amd import binding as T
    run_epochs_plan_beside_copies(H, oracle, W.small_variant("replanning"))
    run_epochs_plan_beside_copies(H, oracle, W.small_variant("replanning"), flags=T.TENT_FLAG_SERIAL_BINDING)


def test_replanning_epochs_enqueued_without_a_host_wait(H, oracle):
    # the whole sequence of epochs is enqueued at once: the rail simulator reads nothing back, an event orders
    # each execute after its plan, and the execute sizes its launches by the budgets alone
    import torch
    from paper_2604_00368_amd import binding as T
    w = W.small_variant("replanning")
    src = W.fill_numpy(w, 0)
    dst0 = W.fill_numpy(w, 1)
    s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
    dst_want = dst0.copy()
    staging_want = np.zeros(w.staging_bytes, dtype=np.uint8)
    records, left = oracle.run_epochs(w, s, [src, dst_want], staging_want)
    assert left.shape[0] == 0
    with H.Engine(w, src, dst0) as eng:
        eng.declare()
        side = torch.cuda.Stream(eng.dev)
        side.wait_stream(eng.stream)
        for ep in list(w.epochs) + [w.drain]:
            st, _ = T.tent_plan(eng.ctx, eng.batch, ep.rails, False, side)
            assert st == 0
            assert T.tent_sim_advance(eng.ctx, eng.batch, ep.budget, side, want_done=False) is None
            ev = torch.cuda.Event()
            ev.record(side)
            eng.stream.wait_event(ev)
            T.tent_execute(eng.ctx, eng.batch, eng.stream)
        assert T.tent_poll(eng.ctx, eng.batch, eng.stream) == 0
        torch.cuda.synchronize(eng.dev)
        assert (eng.table()["state"] == 2).all()
        assert np.array_equal(eng.dst.cpu().numpy(), dst_want)
        assert np.array_equal(eng.arena.cpu().numpy(), staging_want)


@pytest.mark.parametrize("seed", range(10))
def test_partial_executes_random_tiled_geometry(H, oracle, seed):
    # lengths in multiples of 1-4 KiB, source and destination cut differently, a few epochs with random budgets:
    # partial executes go over the list of the BOUND slices' tiles, on one stream and with plans on a second
    rng = np.random.Generator(np.random.PCG64(9000 + seed))
    align = int(rng.choice([1024, 2048, 4096]))
    w = W.ragged(7000 + seed, n_desc=int(rng.integers(3, 60)), max_len=int(rng.integers(20, 400)) * 1024,
                 max_ext=int(rng.integers(1, 24)) * 1024, slice_bytes=align * int(rng.integers(1, 40)),
                 n_rails=int(rng.integers(1, 12)), align=align)
    R = w.rails.shape[0]
    t_us = max(1, -(-w.payload // int(float(rng.choice([2, 4, 8])) * int(w.rails["bw_MBps"].astype(np.uint64).sum()))))
    epochs = []
    for e in range(int(rng.integers(2, 7))):
        bw = np.maximum(1, np.rint(w.rails["bw_MBps"] * np.exp(0.5 * rng.standard_normal(R)))).astype(np.uint64)
        rails = W.make_rails(bw, queued=rng.integers(0, 64 * 1024, size=R), health=w.rails["health"].copy())
        epochs.append(W.Epoch(rails, bw * np.uint64(t_us)))
    w.epochs = epochs
    w.drain = W.Epoch(epochs[-1].rails.copy(), np.full(R, np.iinfo(np.uint64).max, dtype=np.uint64))
    run_epochs_and_compare(H, oracle, w)
    run_epochs_plan_beside_copies(H, oracle, w)


def test_replanning_many_small_shape(H, oracle):
    # re-planning over a workload whose slices straddle pages and whose pending runs are short
    w = W.many_small(n_req=48, layers=2)
    kv = W.replanning(n_req=4, layers=2, ctx_lo=200, ctx_hi=900, queued_hi=64 * 1024)
    R = w.rails.shape[0]
    rng = np.random.Generator(np.random.PCG64(77))
    t_us = -(-w.payload // int(6 * int(w.rails["bw_MBps"].astype(np.uint64).sum())))
    epochs = []
    for e in range(8):
        bw = np.maximum(1, np.rint(w.rails["bw_MBps"] * np.exp(0.5 * rng.standard_normal(R)))).astype(np.uint64)
        health = np.zeros(R, dtype=np.uint8)
        if e >= 2:
            health[5] = 2
        if e >= 4:
            health[0] = 2
        rails = W.make_rails(bw, queued=rng.integers(0, 64 * 1024, size=R), health=health)
        epochs.append(W.Epoch(rails, bw * np.uint64(t_us)))
    w.epochs = epochs
    w.drain = W.Epoch(epochs[-1].rails.copy(), np.full(R, np.iinfo(np.uint64).max, dtype=np.uint64))
    run_epochs_and_compare(H, oracle, w)


def test_defer_errors_and_reuse(H, oracle):
    from paper_2604_00368_amd import binding as T
    w = W.tiny()
    src = W.fill_numpy(w, 0)
    dst0 = np.zeros(w.seg_bytes[1], dtype=np.uint8)
    with H.Engine(w, src, dst0) as eng:
        h = eng.declare()
        # execute before plan
        with pytest.raises(T.TentError) as ei:
            T.tent_execute(eng.ctx, h, eng.stream)
        assert ei.value.status == T.TENT_ERR_STATE
        # every rail excluded: deferred, nothing bound, batch still usable
        rails = w.rails.copy()
        rails["health"] = 2
        st, info = eng.plan(rails=rails)
        assert st == T.TENT_DEFER
        assert T.tent_poll(eng.ctx, h, eng.stream) == T.tent_slice_count(eng.ctx, h)
        # range errors
        bad = w.rails.copy(); bad["bw_MBps"][0] = 0
        with pytest.raises(T.TentError) as ei:
            eng.plan(rails=bad)
        assert ei.value.status == T.TENT_ERR_RANGE
        bad = w.rails.copy(); bad["queued_bytes"][0] = 1 << 62
        with pytest.raises(T.TentError) as ei:
            eng.plan(rails=bad)
        assert ei.value.status == T.TENT_ERR_RANGE
        with pytest.raises(T.TentError) as ei:
            T.tent_plan(eng.ctx, h, np.zeros(65, dtype=W.RAIL_DTYPE), True, eng.stream)
        assert ei.value.status == T.TENT_ERR_RANGE
        # malformed declarations
        def declare(sp, se, dp, de):
            return T.tent_declare(eng.ctx, sp, se, dp, de)
        se = w.src_ext.copy(); se["len"][3] = 0
        with pytest.raises(T.TentError) as ei:
            declare(w.src_ptr, se, w.dst_ptr, w.dst_ext)
        assert ei.value.status == T.TENT_ERR_INVALID
        se = w.src_ext.copy(); se["off"][3] = w.seg_bytes[0] - 10
        with pytest.raises(T.TentError):
            declare(w.src_ptr, se, w.dst_ptr, w.dst_ext)
        se = w.src_ext.copy(); se["len"][0] += 16                                   # source longer than destination
        with pytest.raises(T.TentError):
            declare(w.src_ptr, se, w.dst_ptr, w.dst_ext)
        # overlaps are found on the device while tent_declare has already returned: the first plan on
        # the batch delivers the verdict and releases the batch
        de = w.dst_ext.copy(); de["off"][1] = de["off"][0] + 100                    # overlapping destinations
        hb = declare(w.src_ptr, w.src_ext, w.dst_ptr, de)
        with pytest.raises(T.TentError) as ei:
            T.tent_plan(eng.ctx, hb, w.rails, True, eng.stream)
        assert ei.value.status == T.TENT_ERR_INVALID
        with pytest.raises(T.TentError):
            T.tent_slice_count(eng.ctx, hb)                                         # the handle is dead
        de = w.dst_ext.copy(); de["seg"][:] = 0                                     # destination on top of sources
        hb = declare(w.src_ptr, w.src_ext, w.dst_ptr, de)
        with pytest.raises(T.TentError) as ei:
            T.tent_plan_dispatch(eng.ctx, hb, w.rails, W.make_dispatch_params(1 << 20), None, True, eng.stream)
        assert ei.value.status == T.TENT_ERR_INVALID
        # a health value the header does not define
        bad = w.rails.copy(); bad["health"][2] = 3
        with pytest.raises(T.TentError) as ei:
            eng.plan(rails=bad)
        assert ei.value.status == T.TENT_ERR_INVALID
        with pytest.raises(T.TentError) as ei:
            T.tent_plan_dispatch(eng.ctx, h, bad, W.make_dispatch_params(1 << 20), None, True, eng.stream)
        assert ei.value.status == T.TENT_ERR_INVALID
        sp = w.src_ptr.copy(); sp[5] = sp[4]                                        # empty transfer
        with pytest.raises(T.TentError):
            declare(sp, w.src_ext, w.dst_ptr, w.dst_ext)
        with pytest.raises(T.TentError):
            T.tent_execute(eng.ctx, 12345, eng.stream)                             # unknown handle
        # the batch still plans and executes correctly after all of that; reset + second pass is idempotent
        s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
        b = oracle.bind(s.len, w.rails)
        want = dst0.copy()
        staging = np.zeros(w.staging_bytes, dtype=np.uint8)
        oracle.execute(w, s, b, [src, want], staging)
        for _ in range(2):
            st, info = eng.plan()
            assert st == 0
            H.assert_plan_equal(eng.table(), s, b, info)
            eng.execute()
            assert T.tent_poll(eng.ctx, h, eng.stream) == 0
            assert np.array_equal(eng.dst.cpu().numpy(), want)
            T.tent_reset(eng.ctx, h, eng.stream)
        # plan after completion without reset binds nothing
        st, info = eng.plan(); eng.execute()
        st, info = eng.plan()
        assert info.n_slices == 0 and info.n_pending_before == 0
        # release, then the handle is dead and its slot is reused with a new generation
        T.tent_release(eng.ctx, h)
        with pytest.raises(T.TentError):
            T.tent_slice_count(eng.ctx, h)
        h2 = eng.declare()
        assert h2 != h and T.tent_slice_count(eng.ctx, h2) == s.n


@pytest.mark.parametrize("R", [1, 16, 17, 33, 64])
def test_rail_counts_up_to_the_maximum(H, oracle, R):
    # 1, 16 | 17 | 33, 64 rails exercise the three reduction widths of the binder
    print("rails", R, flush=True)
    rng = np.random.Generator(np.random.PCG64(500 + R))
    w = W.many_small(n_req=40, layers=1)
    w.rails = W.make_rails(rng.integers(5000, 200000, size=R), lat_ns=rng.integers(1000, 9000, size=R),
                           queued=rng.integers(0, 1 << 20, size=R),
                           health=np.where(rng.random(R) < 0.15, 2, 0).astype(np.uint8) if R > 1 else 0)
    if (w.rails["health"] == 2).all():
        w.rails["health"][0] = 0
    run_and_compare(H, oracle, w)
    from paper_2604_00368_amd import binding as T
    run_and_compare(H, oracle, w, flags=T.TENT_FLAG_SERIAL_BINDING)


def test_degenerate_batches(H, oracle):
    from paper_2604_00368_amd import binding as T
    print("degenerate", flush=True)
    # one transfer of one byte
    ptr = np.array([0, 1], dtype=np.uint32)
    w = W.Workload("one_byte", 9, 65536, [64, 64], ptr, W._extents(0, [5], 1), ptr.copy(), W._extents(1, [17], 1),
                   W.make_rails([25000, 50000]), "u8")
    run_and_compare(H, oracle, w)
    # a transfer exactly one slice long, one exactly two slices long, slice size 1 byte over a ragged batch
    ptr = np.array([0, 1, 2], dtype=np.uint32)
    w = W.Workload("exact", 10, 4096, [16384, 16384], ptr, W._extents(0, [0, 4096], [4096, 8192]), ptr.copy(),
                   W._extents(1, [8192, 0], [4096, 8192]), W.make_rails([25000, 50000, 100000]), "u8")
    run_and_compare(H, oracle, w)
    # no transfers at all is rejected
    with H.Engine(w, np.zeros(16384, np.uint8), np.zeros(16384, np.uint8)) as eng:
        with pytest.raises(T.TentError) as ei:
            T.tent_declare(eng.ctx, np.zeros(1, np.uint32), np.zeros(0, W.EXTENT_DTYPE),
                           np.zeros(1, np.uint32), np.zeros(0, W.EXTENT_DTYPE))
        assert ei.value.status == T.TENT_ERR_INVALID
        # the arena must hold the payload plus one alignment gap per rail
    small_arena = W.Workload("exact", 10, 4096, [16384, 16384], ptr, W._extents(0, [0, 4096], [4096, 8192]),
                             ptr.copy(), W._extents(1, [8192, 0], [4096, 8192]), W.make_rails([25000] * 3), "u8")
    eng = H.Engine(small_arena, np.zeros(16384, np.uint8), np.zeros(16384, np.uint8))
    try:
        ctx2 = T.tent_create(4096, eng.arena.data_ptr(), 12288 + 256, 0)        # 3 rails need 12288 + 768
        T.tent_register_segment(ctx2, eng.src.data_ptr(), eng.src.numel())
        T.tent_register_segment(ctx2, eng.dst.data_ptr(), eng.dst.numel())
        h = T.tent_declare(ctx2, small_arena.src_ptr, small_arena.src_ext, small_arena.dst_ptr, small_arena.dst_ext)
        with pytest.raises(T.TentError) as ei:
            T.tent_plan(ctx2, h, small_arena.rails, True, eng.stream)
        assert ei.value.status == T.TENT_ERR_RANGE
        T.tent_destroy(ctx2)
    finally:
        eng.close()


def run_closed_loop_and_compare(H, oracle, w, params, bytes_too=True):
    from paper_2604_00368_amd import binding as T
    s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
    src = W.fill_numpy(w, 0) if bytes_too else None
    dst0 = W.fill_numpy(w, 1) if bytes_too else None
    dst_want = dst0.copy() if bytes_too else None
    staging_want = np.zeros(w.staging_bytes, dtype=np.uint8) if bytes_too else None
    records, left = oracle.run_epochs_closed_loop(w, s, params, [src, dst_want] if bytes_too else None, staging_want)
    assert left.shape[0] == 0
    eng = H.Engine(w, src, dst0) if bytes_too else H.Engine(w)
    try:
        eng.declare()
        est = w.rails["bw_MBps"].astype(np.uint32).copy()
        for e, (rec, ep) in enumerate(zip(records, list(w.epochs) + [w.drain])):
            print("closed-loop epoch", e, "pending", rec["pending"].shape[0], flush=True)
            assert np.array_equal(est, rec["est"])
            rails = ep.rails.copy()
            rails["bw_MBps"] = est
            st, info = eng.plan(rails=rails)
            assert st == 0 and info.n_slices == rec["pending"].shape[0]
            n_done = T.tent_sim_advance(eng.ctx, eng.batch, ep.budget, eng.stream)
            assert n_done == rec["done_ids"].shape[0]
            T.tent_sim_latency(eng.ctx, eng.batch, ep.rails["bw_MBps"], eng.stream)
            new_rails, probe = T.tent_update_bandwidth(eng.ctx, eng.batch, params, rails, eng.stream)
            if rec["tau"] is not None:
                tab = eng.table()
                assert np.array_equal(tab["rail"][rec["pending"]], rec["rail"])
                tau = T.tent_get_latencies(eng.ctx, eng.batch)
                assert np.array_equal(tau[rec["done_ids"]], rec["tau"])
                assert np.array_equal(probe, rec["probe"])
            else:
                assert not probe.any()
            assert np.array_equal(new_rails["bw_MBps"], rec["est_after"])
            assert np.array_equal(new_rails["queued_bytes"], rails["queued_bytes"])     # only bw_MBps changes
            est = new_rails["bw_MBps"].astype(np.uint32)
            eng.execute()
        assert T.tent_poll(eng.ctx, eng.batch, eng.stream) == 0
        if bytes_too:
            assert np.array_equal(eng.dst.cpu().numpy(), dst_want)
            assert np.array_equal(eng.arena.cpu().numpy(), staging_want)
        return eng
    finally:
        eng.close()


def test_telemetry_feedback_closed_loop(H, oracle):
    from paper_2604_00368_amd import binding as T
    w = W.small_variant("replanning")
    params = W.make_probe_params(2 * w.rails["bw_MBps"].astype(np.uint64), ewma_q8=128)
    run_closed_loop_and_compare(H, oracle, w, params)
    # other calibrations: alpha != 1, hardware cap below the true bandwidth, delta above some latencies
    rng = np.random.Generator(np.random.PCG64(8))
    R = w.rails.shape[0]
    params = W.make_probe_params(rng.integers(20000, 90000, size=R), alpha_q8=rng.integers(128, 700, size=R),
                                 delta_ns=rng.integers(0, 40000, size=R), ewma_q8=rng.integers(0, 257, size=R))
    run_closed_loop_and_compare(H, oracle, w, params)
    # argument errors
    with H.Engine(w, W.fill_numpy(w, 0), W.fill_numpy(w, 1)) as eng:
        h = eng.declare()
        with pytest.raises(T.TentError) as ei:
            T.tent_sim_latency(eng.ctx, h, w.rails["bw_MBps"], eng.stream)
        assert ei.value.status == T.TENT_ERR_STATE
        eng.plan()
        bad = w.rails["bw_MBps"].copy(); bad[2] = 0
        with pytest.raises(T.TentError) as ei:
            T.tent_sim_latency(eng.ctx, h, bad, eng.stream)
        assert ei.value.status == T.TENT_ERR_RANGE
        with pytest.raises(T.TentError) as ei:
            T.tent_update_bandwidth(eng.ctx, h, params[:3], w.rails[:3], eng.stream)
        assert ei.value.status == T.TENT_ERR_RANGE
        p2 = params.copy(); p2["ewma_q8"][0] = 300
        with pytest.raises(T.TentError) as ei:
            T.tent_update_bandwidth(eng.ctx, h, p2, w.rails, eng.stream)
        assert ei.value.status == T.TENT_ERR_RANGE


@pytest.mark.parametrize("skew,arena_skew", [((3, 5), 0), ((0, 0), 7), ((1, 0), 9), ((8, 4), 0)])
def test_unaligned_addresses_take_the_fast_paths(H, oracle, skew, arena_skew):
    # pages and staging arena at odd addresses: same bytes, table-driven kernels with unaligned accesses
    print("skew", skew, arena_skew, flush=True)
    w = W.kv_migration(n_req=4, layers=2, ctx_lo=200, ctx_hi=900, skew=skew if skew != (0, 0) else (0, 0))
    run_and_compare(H, oracle, w, arena_skew=arena_skew)
    w = W.many_small(n_req=24, layers=2)
    run_and_compare(H, oracle, w, arena_skew=arena_skew)


def test_poll_on_another_stream_sees_the_bytes(H, oracle):
    # Batch-level completion (Section 4.4) holds on every stream: a poll on a stream that never saw the
    # execute returns 0 only once the copies have ended, so the destination read on that stream is complete.
    from paper_2604_00368_amd import binding as T
    w = W.small_variant("kv_migration")
    src, dst0 = W.fill_numpy(w, 0), W.fill_numpy(w, 1)
    want = expected_destination(w, src, dst0)
    other = torch.cuda.Stream()
    with H.Engine(w, src, dst0) as eng:
        h = eng.declare()
        for rep in range(3):
            st, _ = eng.plan()
            assert st == 0
            T.tent_execute(eng.ctx, h, eng.stream)             # no synchronisation of the execute's stream
            assert T.tent_poll(eng.ctx, h, other) == 0
            with torch.cuda.stream(other):
                got = eng.dst.clone()
            other.synchronize()
            assert np.array_equal(got.cpu().numpy(), want), rep
            torch.cuda.synchronize()
            # release without any wait of the caller's: the library waits for the batch's own work
            eng.dst.copy_(torch.from_numpy(dst0))
            torch.cuda.synchronize()
            T.tent_reset(eng.ctx, h, other)
            other.synchronize()
        st, _ = eng.plan()
        T.tent_execute(eng.ctx, h, eng.stream)
        T.tent_release(eng.ctx, h)
        assert np.array_equal(eng.dst.cpu().numpy(), want)


def test_declare_of_a_large_batch_finds_a_bad_extent_anywhere(H, oracle):
    # large descriptor lists are walked by several host threads, each over a range of transfers: a malformed
    # extent must be found in whichever range it lies, and the sound batch must count its slices right
    import torch
    from paper_2604_00368_amd import binding as T
    n, piece = 300_000, 48
    off = (np.arange(n, dtype=np.uint64) * np.uint64(piece))
    ptr = np.arange(n + 1, dtype=np.uint32)
    seg_bytes = n * piece
    dev = torch.device("cuda:0")
    src = torch.zeros(seg_bytes, dtype=torch.uint8, device=dev)
    dst = torch.zeros(seg_bytes, dtype=torch.uint8, device=dev)
    arena = torch.zeros(seg_bytes + 256 * 4, dtype=torch.uint8, device=dev)
    ctx = T.tent_create(32, arena.data_ptr(), arena.numel(), T.TENT_FLAG_SKIP_OVERLAP_CHECK)
    try:
        T.tent_register_segment(ctx, src.data_ptr(), src.numel())
        T.tent_register_segment(ctx, dst.data_ptr(), dst.numel())
        se, de = W._extents(0, off, piece), W._extents(1, off, piece)
        h = T.tent_declare(ctx, ptr, se, ptr, de)
        assert T.tent_slice_count(ctx, h) == 2 * n                 # 48 bytes = a slice of 32 and a tail of 16
        T.tent_release(ctx, h)
        for where in (5, n // 4 + 7, n // 2 + 1, (3 * n) // 4 + 3, n - 1):
            for side, field, value in ((0, "len", 0), (1, "off", seg_bytes), (0, "seg", 9), (1, "len", piece - 1)):
                bad_s, bad_d = se.copy(), de.copy()
                (bad_s if side == 0 else bad_d)[field][where] = value
                with pytest.raises(T.TentError) as ei:
                    T.tent_declare(ctx, ptr, bad_s, ptr, bad_d)
                assert ei.value.status == T.TENT_ERR_INVALID, (where, side, field)
        h = T.tent_declare(ctx, ptr, se, ptr, de)                  # the context is still sound
        assert T.tent_slice_count(ctx, h) == 2 * n
    finally:
        T.tent_destroy(ctx)


def test_declare_release_cycles_reuse_tables(H, oracle):
    # a loop of declare ... release: later declarations take over the table allocations of released batches,
    # of equal and of different sizes, and every batch still plans and moves correctly
    from paper_2604_00368_amd import binding as T
    ws = [W.small_variant("kv_migration"), W.tiny(), W.small_variant("many_small"), W.tiny(), W.small_variant("kv_migration")]
    wbig = ws[0]
    src_big = W.fill_numpy(wbig, 0)
    with H.Engine(wbig, src_big, np.zeros(wbig.seg_bytes[1], dtype=np.uint8)) as eng:
        s = oracle.split(wbig.src_ptr, wbig.src_ext, wbig.slice_bytes)
        b = oracle.bind(s.len, wbig.rails)
        want = expected_destination(wbig, src_big, np.zeros(wbig.seg_bytes[1], dtype=np.uint8))
        handles = []
        for k in range(7):
            h = eng.declare()
            st, info = eng.plan()
            assert st == 0
            H.assert_plan_equal(eng.table(), s, b, info)
            eng.dst.zero_()
            T.tent_execute(eng.ctx, h, eng.stream)
            if k % 2:
                T.tent_release(eng.ctx, h)                     # straight after the execute was enqueued
                assert np.array_equal(eng.dst.cpu().numpy(), want)
            else:
                handles.append(h)
        for h in handles:
            assert T.tent_poll(eng.ctx, h, eng.stream) == 0
            T.tent_release(eng.ctx, h)
    for w in ws:                                              # different geometries through one process
        src, dst0 = W.fill_numpy(w, 0), W.fill_numpy(w, 1)
        with H.Engine(w, src, dst0) as eng:
            for _ in range(2):
                h = eng.declare()
                st, _ = eng.plan()
                eng.execute()
                assert np.array_equal(eng.dst.cpu().numpy(), expected_destination(w, src, dst0))
                T.tent_release(eng.ctx, h)
