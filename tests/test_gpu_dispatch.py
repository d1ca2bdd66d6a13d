"""GPU parity for the request-level dispatch (Algorithm 1: QoS admission, mice round robin, weighted
spraying of elephants) against the CPU oracle, bit for bit."""
import numpy as np
import pytest

from paper_2604_00368_amd import workloads as W

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

KiB = 1 << 10


@pytest.fixture(scope="module")
def H():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import gpu_harness
    return gpu_harness


def contiguous_requests(lens, S, rails, seed):
    """Contiguous transfers of the given lengths; destination order shuffled."""
    lens = np.asarray(lens, dtype=np.uint64)
    D = lens.shape[0]
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.uint64)
    ptr = np.arange(D + 1, dtype=np.uint32)
    se = np.zeros(D, dtype=W.EXTENT_DTYPE)
    se["seg"], se["len"], se["off"] = W.SRC_SEG, lens, off[:-1]
    order = np.random.Generator(np.random.PCG64(seed)).permutation(D)
    doff = np.zeros(D, dtype=np.uint64)
    doff[order] = np.concatenate([[0], np.cumsum(lens[order])])[:-1]
    de = se.copy()
    de["seg"], de["off"] = W.DST_SEG, doff
    total = int(off[-1])
    return W.Workload("requests", seed, S, [total, total], ptr, se, ptr.copy(), de, rails, "u8")


def dispatch_windows_and_compare(H, oracle, w, theta, gamma_q8, prio, windows, flags=0, bytes_too=True, rr_start=0,
                                 final_check=None):
    """Dispatch the batch window after window (deferred transfers wait for a window that admits them), moving
    what was dealt after every window; everything is compared with the oracle."""
    from paper_2604_00368_amd import binding as T
    R = w.rails.shape[0]
    s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
    src = W.fill_numpy(w, 0) if bytes_too else None
    dst0 = W.fill_numpy(w, 1) if bytes_too else None
    dst_want = dst0.copy() if bytes_too else None
    staging_want = np.zeros(w.staging_bytes, dtype=np.uint8) if bytes_too else None
    eng = H.Engine(w, src, dst0, flags=flags) if bytes_too else H.Engine(w, flags=flags)
    try:
        eng.declare()
        done = np.zeros(s.n, dtype=np.uint8)
        rr = rr_start
        seen_modes = set()
        for window in windows:
            dp = W.make_dispatch_params(theta, gamma_q8=gamma_q8, window=window, rr_start=rr)
            r = oracle.dispatch(s, w.rails, dp, priority=prio, done=done)
            print("dispatch window", window, "pending", int((done == 0).sum()), "dealt", int(r.bound.sum()),
                  "modes", np.bincount(r.mode, minlength=4).tolist(), flush=True)
            st, info = T.tent_plan_dispatch(eng.ctx, eng.batch, w.rails, dp, prio, True, eng.stream)
            assert st == r.binding.status == 0
            tab = eng.table()
            assert np.array_equal(tab["desc"], s.desc) and np.array_equal(tab["len"], s.len)
            ids = np.flatnonzero(r.bound)
            assert np.array_equal(np.flatnonzero(tab["state"] == 1), ids)
            assert np.array_equal(np.flatnonzero(tab["state"] == 2), np.flatnonzero(done))
            assert np.array_equal(tab["rail"][ids], r.binding.rail[ids])
            assert np.array_equal(tab["stage_off"][ids], r.binding.stage_off[ids])
            assert np.array_equal(T.tent_get_modes(eng.ctx, eng.batch, w.n_desc), r.mode)
            b = r.binding
            assert list(info.plan.rail_bytes)[:R] == b.T.tolist()
            assert list(info.plan.rail_slices)[:R] == b.n_slices.tolist()
            assert list(info.plan.queued_after)[:R] == b.A_after.tolist()
            assert list(info.plan.stage_base)[:R] == b.base.tolist()
            assert info.plan.n_slices == ids.shape[0]
            assert (info.n_mice, info.n_elephant, info.n_deferred) == tuple(int((r.mode == k).sum()) for k in (1, 2, 3))
            assert info.rr_next == r.rr_end
            rr = r.rr_end
            seen_modes.update(np.unique(r.mode).tolist())
            if bytes_too and ids.shape[0]:
                oracle.execute(w, s, b, [src, dst_want], staging_want, ids=np.ascontiguousarray(ids.astype(np.uint32)))
            eng.execute()
            done[ids] = 1
            assert T.tent_poll(eng.ctx, eng.batch, eng.stream) == int((done == 0).sum())
            if bytes_too:
                assert np.array_equal(eng.dst.cpu().numpy(), dst_want)
                assert np.array_equal(eng.arena.cpu().numpy(), staging_want)
        if final_check is not None:
            final_check(eng, done)
        return done, seen_modes
    finally:
        eng.close()


@pytest.mark.parametrize("seed", range(6))
def test_random_requests_bit_exact(H, oracle, seed):
    rng = np.random.Generator(np.random.PCG64(700 + seed))
    R = int(rng.choice([1, 3, 9, 16, 40, 64]))
    S = int(rng.choice([4 * KiB, 64 * KiB]))
    D = int(rng.integers(20, 200))
    lens = np.where(rng.random(D) < 0.5, rng.integers(1, 3 * S, D), rng.integers(1, 120 * S, D))
    rails = W.make_rails(rng.integers(1000, 400000, R), lat_ns=rng.integers(0, 20000, R),
                         queued=rng.integers(0, 1 << 22, R), health=rng.choice([0, 0, 0, 1, 2], R),
                         penalty_q8=rng.choice([256, 256, 384], R))
    rails["health"][int(rng.integers(0, R))] = 0
    if seed == 3:                                              # identical idle rails: every cost ties
        rails = W.make_rails([50000] * R)
    w = contiguous_requests(lens, S, rails, seed)
    prio = W.make_priorities(seed, D)
    done, modes = dispatch_windows_and_compare(H, oracle, w, theta=int(rng.choice([S, 2 * S, 8 * S])),
                                               gamma_q8=int(rng.choice([0, 26, 128, 1000])), prio=prio,
                                               windows=[5, 6, 7, 8, 9, 10], rr_start=int(rng.integers(0, 5)))
    assert {1, 2} <= modes
    if R >= 3 and (rails["health"][:3] != 2).all():
        assert done.all()


@pytest.mark.parametrize("name", ["tiny", "kv_migration", "rl_params", "many_small"])
def test_small_configs_dispatch_bit_exact(H, oracle, name):
    w = W.small_variant(name)
    prio = W.make_priorities(11, w.n_desc)
    done, modes = dispatch_windows_and_compare(H, oracle, w, theta=4 * w.slice_bytes, gamma_q8=26, prio=prio,
                                               windows=[0, 1, 2])
    assert done.all()


def test_dispatch_then_cost_model_replan(H, oracle):
    # a window of request-level dispatch, then the per-slice planner finishes what was deferred
    from paper_2604_00368_amd import binding as T
    w = W.small_variant("kv_migration")
    w.rails = w.rails[:2].copy()                               # two rails: in window 0 nothing admits LOW
    s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
    prio = W.make_priorities(4, w.n_desc)
    src, dst0 = W.fill_numpy(w, 0), W.fill_numpy(w, 1)
    dst_want, staging_want = dst0.copy(), np.zeros(w.staging_bytes, dtype=np.uint8)
    dp = W.make_dispatch_params(2 * w.slice_bytes, window=0)
    r = oracle.dispatch(s, w.rails, dp, priority=prio)
    assert (r.mode == 3).any()
    ids = np.flatnonzero(r.bound).astype(np.uint32)
    oracle.execute(w, s, r.binding, [src, dst_want], staging_want, ids=ids)
    rest = np.flatnonzero(r.bound == 0).astype(np.uint32)
    b2 = oracle.bind(s.len, w.rails, ids=rest)
    oracle.execute(w, s, b2, [src, dst_want], staging_want, ids=rest)
    with H.Engine(w, src, dst0) as eng:
        eng.declare()
        st, info = T.tent_plan_dispatch(eng.ctx, eng.batch, w.rails, dp, prio, True, eng.stream)
        assert st == 0 and info.n_deferred == int((r.mode == 3).sum())
        eng.execute()
        st, info2 = eng.plan()
        assert st == 0 and info2.n_slices == rest.shape[0]
        tab = eng.table()
        assert np.array_equal(tab["rail"][rest], b2.rail[rest]) and np.array_equal(tab["stage_off"][rest], b2.stage_off[rest])
        eng.execute()
        assert np.array_equal(eng.dst.cpu().numpy(), dst_want)
        assert np.array_equal(eng.arena.cpu().numpy(), staging_want)


def test_dispatch_argument_errors(H, oracle):
    from paper_2604_00368_amd import binding as T
    w = W.tiny()
    with H.Engine(w, W.fill_numpy(w, 0), W.fill_numpy(w, 1)) as eng:
        h = eng.declare()
        dp = W.make_dispatch_params(4 * w.slice_bytes)
        bad = np.zeros(w.n_desc, dtype=np.uint8); bad[3] = 3
        with pytest.raises(T.TentError) as ei:
            T.tent_plan_dispatch(eng.ctx, h, w.rails, dp, bad)
        assert ei.value.status == T.TENT_ERR_INVALID
        with pytest.raises(T.TentError) as ei:
            T.tent_plan_dispatch(eng.ctx, h, w.rails, W.make_dispatch_params(1, gamma_q8=70000))
        assert ei.value.status == T.TENT_ERR_RANGE
        huge = w.rails.copy(); huge["lat_ns"] = 0xFFFFFFFF; huge["penalty_q8"] = 65535
        with pytest.raises(T.TentError) as ei:
            T.tent_plan_dispatch(eng.ctx, h, huge, W.make_dispatch_params(1, gamma_q8=65535))
        assert ei.value.status == T.TENT_ERR_RANGE
        off = w.rails.copy(); off["health"] = 2
        st, _ = T.tent_plan_dispatch(eng.ctx, h, off, dp)
        assert st == T.TENT_DEFER
        # still usable afterwards, without priorities every transfer is HIGH
        s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
        r = oracle.dispatch(s, w.rails, dp)
        st, info = T.tent_plan_dispatch(eng.ctx, h, w.rails, dp)
        assert st == 0 and info.n_deferred == 0
        tab = eng.table()
        assert np.array_equal(tab["rail"], r.binding.rail) and np.array_equal(tab["stage_off"], r.binding.stage_off)
