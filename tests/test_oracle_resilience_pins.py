"""Pins for the oracle's link-level resilience (Section 4.3): retry rotation, failure marking and the
rail health monitor.  CPU only."""
import numpy as np
import pytest

from helpers import read_golden
from paper_2604_00368_amd import workloads as W

KiB = 1 << 10


def literal_plan(lens, retry, rails, ids):
    """The plan written out in Python integers: rotation for retried slices, then per-slice argmin."""
    R = rails.shape[0]
    health = [int(h) for h in rails["health"]]
    pen = [int(p) for p in rails["penalty_q8"]]
    cand = [d for d in range(R) if health[d] == 0]
    if not cand:
        cand = [d for d in range(R) if health[d] == 1 and pen[d] <= 256]
    if not cand:
        cand = [d for d in range(R) if health[d] == 1]
    if not cand:
        return None
    c0, c1 = [], []
    for r in rails:
        w = 2 if int(r["health"]) == 1 else 1
        c1.append(w * (10**6 * int(r["beta1_q8"]) * int(r["penalty_q8"]) // int(r["bw_MBps"])))
        c0.append(w * ((int(r["lat_ns"]) * 1000 * int(r["penalty_q8"])) >> 8))
    A = [int(q) for q in rails["queued_bytes"]]
    T = [0] * R
    rail, off = {}, {}
    for i in ids:
        if retry[i]:
            d = cand[(int(i) + int(retry[i])) % len(cand)]
            rail[i], off[i] = d, T[d]
            T[d] += int(lens[i]); A[d] += int(lens[i])
    for i in ids:
        if not retry[i]:
            costs = [(c0[d] + (((A[d] + int(lens[i])) * c1[d]) >> 16), d) for d in range(R) if health[d] != 2]
            d = min(costs)[1]
            rail[i], off[i] = d, T[d]
            T[d] += int(lens[i]); A[d] += int(lens[i])
    return rail, off, T, A


def test_worked_example(oracle):
    rows = read_golden("retry_rotation_worked_example.txt")
    rails = W.make_rails([25000] * 4, health=np.array([0, 2, 0, 1]))
    lens = np.full(8, 64 * KiB, dtype=np.uint32)
    retry = np.zeros(8, dtype=np.uint8)
    retry[[2, 5, 6]] = [1, 1, 2]
    b = oracle.plan(lens, retry, rails)
    assert b.status == oracle.OK
    assert b.rail.tolist() == rows[0]
    assert b.stage_off.tolist() == rows[1]
    assert b.T.tolist() == rows[2]


@pytest.mark.parametrize("seed", range(12))
def test_plan_matches_the_literal_python_version(oracle, seed):
    rng = np.random.Generator(np.random.PCG64(4300 + seed))
    R = int(rng.integers(1, 9))
    n = int(rng.integers(1, 120))
    rails = W.make_rails(rng.integers(1000, 400000, R), lat_ns=rng.integers(0, 20000, R),
                         queued=rng.integers(0, 1 << 24, R), health=rng.choice([0, 0, 1, 2], R),
                         penalty_q8=rng.choice([256, 256, 384, 512], R))
    lens = rng.choice([4 * KiB, 64 * KiB, 64 * KiB, 1000], n).astype(np.uint32)
    retry = (rng.integers(0, 4, n) * (rng.random(n) < 0.4)).astype(np.uint8)
    ids = np.flatnonzero(rng.random(n) < 0.8).astype(np.uint32)
    b = oracle.plan(lens, retry, rails, ids=ids)
    want = literal_plan(lens, retry, rails, ids)
    if want is None:
        assert b.status == oracle.DEFER and int(b.T.sum()) == 0
        return
    rail, off, T, A = want
    assert b.status == oracle.OK
    assert [int(b.rail[i]) for i in ids] == [rail[i] for i in ids]
    assert [int(b.stage_off[i]) for i in ids] == [off[i] for i in ids]
    assert b.T.tolist() == T and b.A_after.tolist() == A
    untouched = np.setdiff1d(np.arange(n), ids)
    assert (b.rail[untouched] == 0xFFFFFFFF).all()


def test_candidate_groups(oracle):
    # first pass: HEALTHY rails only, even when DEGRADED ones are faster
    rails = W.make_rails([25000, 400000, 25000, 400000], health=np.array([0, 1, 0, 2]))
    assert oracle.rotation_candidates(rails).tolist() == [0, 2]
    # no HEALTHY rail: DEGRADED rails without topology penalty come before the others
    rails = W.make_rails([25000] * 5, health=np.array([2, 1, 1, 2, 1]), penalty_q8=np.array([256, 512, 256, 256, 200]))
    assert oracle.rotation_candidates(rails).tolist() == [2, 4]
    # only penalised DEGRADED rails left: any reachable one
    rails = W.make_rails([25000] * 3, health=np.array([1, 2, 1]), penalty_q8=np.array([512, 256, 300]))
    assert oracle.rotation_candidates(rails).tolist() == [0, 2]
    # nothing admitted: deferred, nothing bound
    rails = W.make_rails([25000] * 3, health=2)
    assert oracle.rotation_candidates(rails).tolist() == []
    lens = np.full(4, 64 * KiB, dtype=np.uint32)
    b = oracle.plan(lens, np.array([1, 0, 2, 0], dtype=np.uint8), rails)
    assert b.status == oracle.DEFER and (b.rail == 0xFFFFFFFF).all() and int(b.T.sum()) == 0


def test_retried_slices_never_use_the_cost_model(oracle):
    # a retried slice lands on its rotation slot even when that rail is by far the most expensive
    rails = W.make_rails([1000, 400000, 400000], queued=np.array([1 << 30, 0, 0]))
    lens = np.full(6, 64 * KiB, dtype=np.uint32)
    retry = np.array([0, 0, 3, 0, 0, 0], dtype=np.uint8)          # slice 2, third retry: (2+3) mod 3 = 2
    b = oracle.plan(lens, retry, rails)
    assert int(b.rail[2]) == 2 and int(b.stage_off[2]) == 0
    retry[2] = 1                                                  # first retry: (2+1) mod 3 = 0, the slow rail
    b = oracle.plan(lens, retry, rails)
    assert int(b.rail[2]) == 0
    assert (np.delete(b.rail, 2) != 0).all()                      # the cost model keeps everything else off it


def test_successive_retries_walk_round_the_candidate_set(oracle):
    rails = W.make_rails([25000] * 7, health=np.array([0, 2, 0, 0, 1, 0, 0]))
    cand = oracle.rotation_candidates(rails).tolist()
    assert cand == [0, 2, 3, 5, 6]
    lens = np.full(40, 64 * KiB, dtype=np.uint32)
    for i in (0, 7, 39):
        seen = []
        for k in range(1, len(cand) + 1):
            retry = np.zeros(40, dtype=np.uint8)
            retry[i] = k
            seen.append(int(oracle.plan(lens, retry, rails).rail[i]))
        assert sorted(seen) == cand                               # every candidate exactly once in |C| retries
        assert all(seen[k] != seen[k - 1] for k in range(1, len(seen)))


def test_slices_that_fail_together_spread_over_the_candidates(oracle):
    rails = W.make_rails([12500, 100000, 50000], health=0)
    lens = np.full(100, 64 * KiB, dtype=np.uint32)
    retry = np.zeros(100, dtype=np.uint8)
    retry[10:71] = 1                                              # 61 consecutive slices failed once
    b = oracle.plan(lens, retry, rails)
    counts = np.bincount(b.rail[10:71], minlength=3)
    assert counts.max() - counts.min() <= 1                       # bandwidth plays no part in the rotation
    # within a rail the retried slices are packed from offset 0 in slice order, the others follow
    for d in range(3):
        on_d = np.flatnonzero(b.rail == d)
        first = [i for i in on_d if retry[i]] + [i for i in on_d if not retry[i]]
        assert b.stage_off[first].tolist() == (np.arange(len(first)) * 64 * KiB).tolist()


def test_recovery_traffic_counts_in_the_queue_statistics(oracle):
    # Section 4.3: retries bypass the cost model, yet their bytes are part of what the cost model sees.
    # So the second pass must equal a plain cost-model bind whose rails start with the retried bytes queued.
    rng = np.random.Generator(np.random.PCG64(77))
    rails = W.make_rails([25000, 50000, 100000, 25000], queued=rng.integers(0, 1 << 22, 4), health=np.array([0, 0, 1, 0]))
    n = 300
    lens = rng.choice([64 * KiB, 64 * KiB, 3000], n).astype(np.uint32)
    retry = (rng.random(n) < 0.3).astype(np.uint8) * rng.integers(1, 5, n).astype(np.uint8)
    b = oracle.plan(lens, retry, rails)
    cand = oracle.rotation_candidates(rails)
    rot = np.flatnonzero(retry)
    Tr = np.zeros(4, dtype=np.uint64)
    for i in rot:
        d = int(cand[(int(i) + int(retry[i])) % len(cand)])
        assert int(b.rail[i]) == d and int(b.stage_off[i]) == int(Tr[d])
        Tr[d] += lens[i]
    shifted = rails.copy()
    shifted["queued_bytes"] += Tr
    fresh = np.flatnonzero(retry == 0).astype(np.uint32)
    ref = oracle.bind(lens, shifted, ids=fresh)
    assert (b.rail[fresh] == ref.rail[fresh]).all()
    assert (b.stage_off[fresh] == ref.stage_off[fresh] + Tr[ref.rail[fresh]]).all()
    assert (b.T == ref.T + Tr).all()
    assert (b.A_after == rails["queued_bytes"] + b.T).all()
    # and it matters: without the retried bytes the fresh slices would be placed differently
    plain = oracle.bind(lens, rails, ids=fresh)
    assert (plain.rail[fresh] != b.rail[fresh]).any()


def test_without_retries_the_plan_is_the_plain_bind(oracle):
    w = W.tiny()
    s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
    a = oracle.bind(s.len, w.rails)
    b = oracle.plan(s.len, np.zeros(s.n, dtype=np.uint8), w.rails)
    assert (a.rail == b.rail).all() and (a.stage_off == b.stage_off).all()
    assert (a.T == b.T).all() and (a.base == b.base).all() and (a.A_after == b.A_after).all()


def test_fail_marks_exactly_the_slices_of_failed_rails(oracle):
    w = W.tiny()
    s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
    b = oracle.bind(s.len, w.rails)
    retry = np.zeros(s.n, dtype=np.uint8)
    retry[::5] = 254
    before = retry.copy()
    failed, per_rail = oracle.fail(b, [0, 0, 1, 1], retry)
    on = np.isin(b.rail, [2, 3])
    assert (failed.astype(bool) == on).all()
    assert per_rail.tolist() == [0, 0, int((b.rail == 2).sum()), int((b.rail == 3).sum())]
    assert (retry[~on] == before[~on]).all()
    assert (retry[on] == before[on] + 1).all()
    failed, _ = oracle.fail(b, [0, 0, 1, 1], retry)               # counts saturate at 255
    assert (retry[on] == np.minimum(before[on].astype(int) + 2, 255)).all()
    ids = np.flatnonzero(b.rail == 3)[:3].astype(np.uint32)       # listed slices only
    r2 = np.zeros(s.n, dtype=np.uint8)
    failed, per_rail = oracle.fail(b, [0, 0, 0, 1], r2, ids=ids)
    assert failed.tolist() == [1, 1, 1] and int(r2.sum()) == 3 and per_rail.tolist() == [0, 0, 0, 3]


# ------------------------------------------------------------------------------ rail health monitor
def mparams(oracle, err=2, recover=2, cooldown=1, degrade_q8=128):
    return np.array([(err, recover, cooldown, degrade_q8)], dtype=oracle.MONITOR_PARAMS_DTYPE)


def run_windows(oracle, mp, windows, probe=0, bw=1000):
    mon = oracle.monitor_init(1, mp)
    states = []
    for hard, cong in windows:
        oracle.monitor_step(mp, mon, [hard], [cong], [probe], [bw])
        states.append(int(mon["state"][0]))
    return states, mon


def test_monitor_timeline(oracle):
    rows = read_golden("rail_monitor_timeline.txt")
    states, _ = run_windows(oracle, mparams(oracle), [(h, c) for h, c, _ in rows])
    assert states == [s for _, _, s in rows]


@pytest.mark.parametrize("E", [1, 3, 10])
def test_congestion_errors_need_twice_the_threshold(oracle, E):
    mp = mparams(oracle, err=E)
    assert run_windows(oracle, mp, [(E, 0)])[0] == [1]            # at the threshold: degraded, not paused
    assert run_windows(oracle, mp, [(E + 1, 0)])[0] == [2]        # beyond it: paused
    assert run_windows(oracle, mp, [(0, 2 * E)])[0] == [1]
    assert run_windows(oracle, mp, [(0, 2 * E + 1)])[0] == [2]
    assert run_windows(oracle, mp, [(E, 1)])[0] == [2]            # mixed: one hard error weighs two congestion errors
    assert run_windows(oracle, mp, [(E - 1, 2)])[0] == [1]


def test_errors_accumulate_until_a_clean_window(oracle):
    mp = mparams(oracle, err=2, recover=5)
    assert run_windows(oracle, mp, [(1, 0), (1, 0), (1, 0)])[0] == [1, 1, 2]
    assert run_windows(oracle, mp, [(1, 0), (1, 0), (0, 0), (1, 0), (1, 0)])[0] == [1, 1, 1, 1, 1]


def test_cooldown_doubles_and_resets_on_promotion(oracle):
    mp = mparams(oracle, err=0, recover=1, cooldown=3)
    # pause, wait, fail again straight after re-admission: 3, 6, 12 windows of exclusion
    seq, expect = [], []
    for length in (3, 6, 12):
        seq += [(1, 0)] + [(0, 0)] * length
        expect += [2] * length + [1]
    states, mon = run_windows(oracle, mp, seq)
    assert states == expect and int(mon["cooldown_next"][0]) == 24
    # one clean window promotes (recover = 1) and the next pause is short again
    states, mon = run_windows(oracle, mp, seq + [(0, 0), (1, 0), (0, 0), (0, 0), (0, 0)])
    assert states[len(seq):] == [0, 2, 2, 2, 1] and int(mon["cooldown_next"][0]) == 6


def test_errors_on_a_paused_rail_are_ignored(oracle):
    mp = mparams(oracle, err=0, recover=1, cooldown=2)
    assert run_windows(oracle, mp, [(1, 0), (9, 9), (9, 9), (0, 0)])[0] == [2, 2, 1, 0]


@pytest.mark.parametrize("k", [1, 2, 5])
def test_degraded_rail_recovers_after_k_clean_windows(oracle, k):
    mp = mparams(oracle, err=5, recover=k)
    states, _ = run_windows(oracle, mp, [(1, 0)] + [(0, 0)] * (k + 1))
    assert states == [1] + [1] * (k - 1) + [0, 0]
    # an error on the way restarts the count
    states, _ = run_windows(oracle, mp, [(1, 0)] + [(0, 0)] * (k - 1) + [(0, 1)] + [(0, 0)] * k)
    assert states == [1] * (2 * k) + [0]


def test_slow_probe_is_a_degradation_event(oracle):
    mp = mparams(oracle, err=5, recover=1, degrade_q8=128)       # below half the estimate
    mon = oracle.monitor_init(4, mp)
    #             probe: none, just below half, exactly half, above
    oracle.monitor_step(mp, mon, [0] * 4, [0] * 4, [0, 499, 500, 900], [1000] * 4)
    assert mon["state"].tolist() == [0, 1, 0, 0]
    oracle.monitor_step(mp, mon, [0] * 4, [0] * 4, [0, 1000, 0, 0], [1000] * 4)
    assert mon["state"].tolist() == [0, 0, 0, 0]


def test_monitor_states_steer_the_plan(oracle):
    # a paused rail gets nothing, a degraded rail half the share of its healthy twin
    mp = mparams(oracle, err=1, recover=3, cooldown=4)
    mon = oracle.monitor_init(3, mp)
    oracle.monitor_step(mp, mon, [0, 1, 2], [0, 0, 0], [0, 0, 0], [50000] * 3)
    assert mon["state"].tolist() == [0, 1, 2]
    rails = W.make_rails([50000] * 3, lat_ns=0, health=mon["state"].astype(np.uint8))
    lens = np.full(300, 64 * KiB, dtype=np.uint32)
    b = oracle.bind(lens, rails)
    assert b.n_slices.tolist() == [200, 100, 0]


# ------------------------------------------------------------------------------ the loop as a whole
def test_resilient_epochs_deliver_every_byte_exactly_once(oracle):
    # Section 4.3: faults are absorbed below the batch; whatever fails, the destination ends up as the plain
    # definition says and every slice completes exactly once.
    from helpers import expected_destination
    w = W.small_variant("replanning")
    R = w.rails.shape[0]
    s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
    src, dst0 = W.fill_numpy(w, 0), W.fill_numpy(w, 1)
    dst = dst0.copy()
    staging = np.zeros(w.staging_bytes, dtype=np.uint8)
    params = W.make_probe_params(2 * w.rails["bw_MBps"].astype(np.uint64), ewma_q8=128)
    fails, cong = W.failure_schedule(5, len(w.epochs), R)
    assert fails.any() and cong.any()
    recs = oracle.run_epochs_resilient(w, s, params, W.make_monitor_params(), fails, cong, [src, dst], staging)
    assert np.array_equal(dst, expected_destination(w, src, dst0))
    done = np.concatenate([r["done_ids"] for r in recs])
    assert np.array_equal(np.sort(done), np.arange(s.n))
    assert sum(int(r["failed_per_rail"].sum()) for r in recs) == int(recs[-1]["retry_after"].astype(int).sum()) > 0
    states = np.stack([r["mon_after"]["state"] for r in recs])
    assert (states == 1).any() and (states == 2).any()            # the schedule reaches every health state
    for r in recs:
        if r["rail"] is None:
            continue
        # a slice never rides a rail that was excluded when it was planned
        assert (r["rails"]["health"][r["rail"]] != 2).all()
        # retried slices sit on HEALTHY rails whenever one exists
        k = r["retry"][r["pending"]]
        if (r["rails"]["health"] == 0).any():
            assert (r["rails"]["health"][r["rail"][k > 0]] == 0).all()
