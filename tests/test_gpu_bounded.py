"""GPU parity for bounded, pipelined staging (Section 4.1): chunks of the payload pass through an arena that
is smaller than the payload; destination and arena bytes against the CPU oracle, bit for bit."""
import numpy as np
import pytest

from paper_2604_00368_amd import workloads as W

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

MiB = 1 << 20


@pytest.fixture(scope="module")
def H():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import gpu_harness
    return gpu_harness


@pytest.mark.parametrize("slots", [1, 2])
@pytest.mark.parametrize("name,chunk", [("tiny", 1 * MiB), ("tiny", 3 * MiB), ("kv_migration", 2 * MiB),
                                        ("rl_params", 1 * MiB), ("many_small", 1 * MiB)])
def test_bounded_execute_bit_exact(H, oracle, name, chunk, slots):
    from paper_2604_00368_amd import binding as T
    w = W.small_variant(name)
    R = w.rails.shape[0]
    assert chunk < w.payload
    slot = chunk + 256 * R
    cap = slots * slot
    src, dst0 = W.fill_numpy(w, 0), W.fill_numpy(w, 1)
    s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
    b = oracle.bind(s.len, w.rails)
    dst_want, staging_want = dst0.copy(), np.zeros(cap, dtype=np.uint8)
    assert oracle.execute_bounded(w, s, b, [src, dst_want], staging_want, chunk, slots=slots, slot_bytes=slot) == 0
    with H.Engine(w, src, dst0, flags=T.TENT_FLAG_BOUNDED_STAGING, arena_bytes=cap) as eng:
        eng.declare()
        st, info = eng.plan()
        assert st == 0
        H.assert_plan_equal(eng.table(), s, b, info)
        T.tent_execute_bounded(eng.ctx, eng.batch, chunk, eng.stream, slots=slots)
        # no device-wide wait here: the caller's stream alone must see the batch complete
        eng.stream.synchronize()
        assert T.tent_poll(eng.ctx, eng.batch, eng.stream) == 0
        assert np.array_equal(eng.dst.cpu().numpy(), dst_want)
        assert np.array_equal(eng.arena.cpu().numpy(), staging_want)
        assert np.array_equal(eng.src.cpu().numpy(), src)


@pytest.mark.parametrize("slots", [1, 2])
def test_bounded_execute_over_replanning_epochs(H, oracle, slots):
    # every epoch only the slices that stayed bound move (a FIFO prefix per rail), through a 1 MiB buffer
    from paper_2604_00368_amd import binding as T
    w = W.replanning(n_req=6, layers=4, ctx_lo=400, ctx_hi=2000, queued_hi=1 << 20)
    R = w.rails.shape[0]
    chunk = 4 * MiB
    slot = chunk + 256 * R
    cap = slots * slot
    src, dst0 = W.fill_numpy(w, 0), W.fill_numpy(w, 1)
    s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
    dst_want, staging_want = dst0.copy(), np.zeros(cap, dtype=np.uint8)
    pending = np.arange(s.n, dtype=np.uint32)
    with H.Engine(w, src, dst0, flags=T.TENT_FLAG_BOUNDED_STAGING, arena_bytes=cap) as eng:
        eng.declare()
        for e, ep in enumerate(list(w.epochs) + [w.drain]):
            if pending.shape[0] == 0:
                break
            b = oracle.bind(s.len, ep.rails, ids=pending)
            assert b.status == 0
            done = oracle.retire(s, b, ep.rails["queued_bytes"], ep.budget, ids=pending).astype(bool)
            ids = np.ascontiguousarray(pending[done])
            if ids.shape[0]:
                assert oracle.execute_bounded(w, s, b, [src, dst_want], staging_want, chunk, ids=ids, slots=slots,
                                              slot_bytes=slot) == 0
            print("bounded epoch", e, "pending", pending.shape[0], "moved", ids.shape[0], flush=True)
            st, info = eng.plan(rails=ep.rails)
            assert st == 0 and info.n_slices == pending.shape[0]
            assert T.tent_sim_advance(eng.ctx, eng.batch, ep.budget, eng.stream) == ids.shape[0]
            T.tent_execute_bounded(eng.ctx, eng.batch, chunk, eng.stream, slots=slots)
            eng.stream.synchronize()
            assert np.array_equal(eng.dst.cpu().numpy(), dst_want)
            assert np.array_equal(eng.arena.cpu().numpy(), staging_want)
            pending = np.ascontiguousarray(pending[~done])
            assert T.tent_poll(eng.ctx, eng.batch, eng.stream) == pending.shape[0]
        assert pending.shape[0] == 0


def test_bounded_argument_errors(H, oracle):
    from paper_2604_00368_amd import binding as T
    w = W.tiny()
    R = w.rails.shape[0]
    src, dst0 = W.fill_numpy(w, 0), W.fill_numpy(w, 1)
    with H.Engine(w, src, dst0) as eng:                       # context without the flag
        h = eng.declare()
        eng.plan()
        with pytest.raises(T.TentError) as ei:
            T.tent_execute_bounded(eng.ctx, h, MiB, eng.stream)
        assert ei.value.status == T.TENT_ERR_STATE
    cap = 2 * MiB + 256 * R
    with H.Engine(w, src, dst0, flags=T.TENT_FLAG_BOUNDED_STAGING, arena_bytes=cap) as eng:
        h = eng.declare()
        with pytest.raises(T.TentError) as ei:
            T.tent_execute_bounded(eng.ctx, h, MiB, eng.stream)
        assert ei.value.status == T.TENT_ERR_STATE             # not planned yet
        st, _ = eng.plan()                                     # the arena is smaller than the payload: allowed here
        assert st == 0
        for bad in (0, MiB + 4096, MiB // 2):
            with pytest.raises(T.TentError) as ei:
                T.tent_execute_bounded(eng.ctx, h, bad, eng.stream)
            assert ei.value.status == T.TENT_ERR_INVALID
        with pytest.raises(T.TentError) as ei:
            T.tent_execute_bounded(eng.ctx, h, 3 * MiB, eng.stream)     # chunk does not fit the arena
        assert ei.value.status == T.TENT_ERR_RANGE
        with pytest.raises(T.TentError) as ei:
            T.tent_execute_bounded(eng.ctx, h, 2 * MiB, eng.stream, slots=2)   # two slots do not fit either
        assert ei.value.status == T.TENT_ERR_RANGE
        with pytest.raises(T.TentError) as ei:
            T.tent_execute_bounded(eng.ctx, h, MiB, eng.stream, slots=3)
        assert ei.value.status == T.TENT_ERR_INVALID
        with pytest.raises(T.TentError) as ei:
            T.tent_execute(eng.ctx, h, eng.stream)                      # the unbounded execute needs the whole payload
        assert ei.value.status == T.TENT_ERR_RANGE
        assert np.array_equal(eng.dst.cpu().numpy(), dst0)      # nothing has moved so far
        T.tent_execute_bounded(eng.ctx, h, 2 * MiB, eng.stream)
        torch.cuda.synchronize()
        assert T.tent_poll(eng.ctx, h, eng.stream) == 0


@pytest.mark.parametrize("slots", [1, 2])
@pytest.mark.parametrize("seed,kw", [(3, {}), (4, dict(n_desc=9, max_len=1_500_000, slice_bytes=65536 + 3)),
                                     (5, dict(n_desc=40, max_len=90_000, slice_bytes=1, max_ext=7)),
                                     (6, dict(n_desc=6, max_len=3_000_000, slice_bytes=1 << 20, max_ext=1 << 18)),
                                     (7, dict(n_desc=30, max_len=300_000, slice_bytes=5000, align=8))])
def test_bounded_execute_ragged_geometry_bit_exact(H, oracle, seed, kw, slots):
    # lengths that are no multiple of any tile size (1-byte slices, 1-byte extents, source and destination cut
    # differently): the chunks are moved byte-exactly in ranges of 1 KiB; arena and destination against the oracle
    from paper_2604_00368_amd import binding as T
    w = W.ragged(seed, **kw)
    R = w.rails.shape[0]
    chunk = MiB
    assert chunk < w.payload
    slot = chunk + 256 * R
    cap = slots * slot
    src, dst0 = W.fill_numpy(w, 0), W.fill_numpy(w, 1)
    s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
    b = oracle.bind(s.len, w.rails)
    dst_want, staging_want = dst0.copy(), np.zeros(cap, dtype=np.uint8)
    assert oracle.execute_bounded(w, s, b, [src, dst_want], staging_want, chunk, slots=slots, slot_bytes=slot) == 0
    print("ragged bounded", seed, "payload", w.payload, "slices", s.n, "chunks", -(-w.payload // chunk), flush=True)
    with H.Engine(w, src, dst0, flags=T.TENT_FLAG_BOUNDED_STAGING, arena_bytes=cap, arena_skew=seed % 3) as eng:
        eng.declare()
        st, info = eng.plan()
        assert st == 0
        H.assert_plan_equal(eng.table(), s, b, info)
        T.tent_execute_bounded(eng.ctx, eng.batch, chunk, eng.stream, slots=slots)
        eng.stream.synchronize()
        assert T.tent_poll(eng.ctx, eng.batch, eng.stream) == 0
        assert np.array_equal(eng.dst.cpu().numpy(), dst_want)
        assert np.array_equal(eng.arena.cpu().numpy(), staging_want)
        assert np.array_equal(eng.src.cpu().numpy(), src)


def test_bounded_execute_ragged_partial_sets(H, oracle):
    # re-planning epochs on ragged geometry: only the slices that stayed bound move, the rest is re-planned
    from paper_2604_00368_amd import binding as T
    w = W.ragged(11, n_desc=16, max_len=600_000, slice_bytes=30_000 + 1)
    w.rails["health"] = 0
    R = w.rails.shape[0]
    chunk = MiB
    slot = chunk + 256 * R
    src, dst0 = W.fill_numpy(w, 0), W.fill_numpy(w, 1)
    s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
    dst_want, staging_want = dst0.copy(), np.zeros(slot, dtype=np.uint8)
    pending = np.arange(s.n, dtype=np.uint32)
    rng = np.random.Generator(np.random.PCG64(77))
    with H.Engine(w, src, dst0, flags=T.TENT_FLAG_BOUNDED_STAGING, arena_bytes=slot) as eng:
        eng.declare()
        for epoch in range(12):
            if pending.shape[0] == 0:
                break
            rails = w.rails.copy()
            rails["queued_bytes"] = rng.integers(0, 1 << 16, size=R)
            b = oracle.bind(s.len, rails, ids=pending)
            share = 1.0 if epoch >= 6 else 0.4
            budget = (rails["queued_bytes"] + (b.T * share).astype(np.uint64)).astype(np.uint64)
            done = oracle.retire(s, b, rails["queued_bytes"], budget, ids=pending).astype(bool)
            ids = np.ascontiguousarray(pending[done])
            if ids.shape[0]:
                assert oracle.execute_bounded(w, s, b, [src, dst_want], staging_want, chunk, ids=ids, slot_bytes=slot) == 0
            st, info = eng.plan(rails=rails)
            assert st == 0 and info.n_slices == pending.shape[0]
            assert T.tent_sim_advance(eng.ctx, eng.batch, budget, eng.stream) == ids.shape[0]
            T.tent_execute_bounded(eng.ctx, eng.batch, chunk, eng.stream)
            eng.stream.synchronize()
            assert np.array_equal(eng.dst.cpu().numpy(), dst_want)
            assert np.array_equal(eng.arena.cpu().numpy(), staging_want)
            pending = np.ascontiguousarray(pending[~done])
            assert T.tent_poll(eng.ctx, eng.batch, eng.stream) == pending.shape[0]
        assert pending.shape[0] == 0


def test_bounded_execute_after_dispatch_with_odd_addresses(H, oracle):
    # the bounded execute moves whatever is BOUND, whoever planned it: request-level dispatch with deferred
    # transfers, pages and arena at odd addresses, 1 KiB tiles
    from paper_2604_00368_amd import binding as T
    w = W.kv_migration(n_req=5, layers=2, ctx_lo=300, ctx_hi=1200, page_tokens=1, head_dim=64, skew=(3, 5))   # 1 KiB pages
    w.rails = w.rails[:2].copy()
    R = w.rails.shape[0]
    chunk = 2 * MiB
    cap = chunk + 256 * R
    src, dst0 = W.fill_numpy(w, 0), W.fill_numpy(w, 1)
    s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
    prio = W.make_priorities(8, w.n_desc)
    dst_want, staging_want = dst0.copy(), np.zeros(cap, dtype=np.uint8)
    done = np.zeros(s.n, dtype=np.uint8)
    with H.Engine(w, src, dst0, flags=T.TENT_FLAG_BOUNDED_STAGING, arena_bytes=cap, arena_skew=7) as eng:
        eng.declare()
        for window in range(3):
            dp = W.make_dispatch_params(4 * w.slice_bytes, window=window)
            r = oracle.dispatch(s, w.rails, dp, priority=prio, done=done)
            ids = np.flatnonzero(r.bound).astype(np.uint32)
            if ids.shape[0]:
                assert oracle.execute_bounded(w, s, r.binding, [src, dst_want], staging_want, chunk, ids=ids) == 0
            st, info = T.tent_plan_dispatch(eng.ctx, eng.batch, w.rails, dp, prio, True, eng.stream)
            assert st == 0 and info.plan.n_slices == ids.shape[0]
            T.tent_execute_bounded(eng.ctx, eng.batch, chunk, eng.stream)
            torch.cuda.synchronize()
            done[ids] = 1
            assert T.tent_poll(eng.ctx, eng.batch, eng.stream) == int((done == 0).sum())
            assert np.array_equal(eng.dst.cpu().numpy(), dst_want)
            assert np.array_equal(eng.arena.cpu().numpy(), staging_want)
        assert done.all()
