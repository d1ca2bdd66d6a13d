"""Pins for the oracle's request-level dispatch (Algorithm 1: QoS admission, mice and elephant modes).  CPU only."""
from fractions import Fraction

import numpy as np
import pytest

from helpers import read_golden
from paper_2604_00368_amd import workloads as W
from test_oracle_pins import one_transfer

KiB, MiB = 1 << 10, 1 << 20


def requests(lens, S, rails):
    """A workload of contiguous transfers with the given byte lengths."""
    lens = np.asarray(lens, dtype=np.uint64)
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.uint64)
    ptr = np.arange(lens.shape[0] + 1, dtype=np.uint32)
    se = np.zeros(lens.shape[0], dtype=W.EXTENT_DTYPE)
    se["seg"], se["len"], se["off"] = 0, lens, off[:-1]
    de = se.copy()
    de["seg"] = 1
    total = int(off[-1])
    return W.Workload("requests", 0, S, [total, total], ptr, se, ptr.copy(), de, rails, "u8")


def literal_dispatch(s, rails, dp, priority, done):
    """Algorithm 1 per request in Python integers (exact rationals for the tolerance test)."""
    R = rails.shape[0]
    theta, gamma, window, rr = (int(dp[f][0]) for f in ("theta_bytes", "gamma_q8", "window", "rr_start"))
    c0, c1 = [], []
    for r in rails:
        w = 2 if int(r["health"]) == 1 else 1
        c1.append(w * (10**6 * int(r["beta1_q8"]) * int(r["penalty_q8"]) // int(r["bw_MBps"])))
        c0.append(w * ((int(r["lat_ns"]) * 1000 * int(r["penalty_q8"])) >> 8))
    A = [int(q) for q in rails["queued_bytes"]]
    T = [0] * R
    rail, off, mode = {}, {}, []
    needs = [2, 1, 0]
    for j in range(s.first.shape[0] - 1):
        ids = [i for i in range(int(s.first[j]), int(s.first[j + 1])) if not done[i]]
        if not ids:
            mode.append(0); continue
        adm = [d for d in range(R) if int(rails["health"][d]) != 2 and int(priority[j]) >= needs[(window + d) % 3]]
        if not adm:
            mode.append(3); continue
        L_req = sum(int(s.len[i]) for i in range(int(s.first[j]), int(s.first[j + 1])))
        if L_req < theta:
            cost = {d: c0[d] + (((A[d] + L_req) * c1[d]) >> 16) for d in adm}
            smin = min(cost.values())
            cand = [d for d in adm if Fraction(cost[d]) <= Fraction(smin) + (smin * gamma) // 256]
            pick = cand[rr % len(cand)]
            rr += 1
            for i in ids:
                rail[i], off[i] = pick, T[pick]
                T[pick] += int(s.len[i]); A[pick] += int(s.len[i])
            mode.append(1)
        else:
            L0 = int(s.len[int(s.first[j])])
            cost = {d: max(1, c0[d] + (((A[d] + L0) * c1[d]) >> 16)) for d in adm}
            m = {d: 0 for d in adm}
            for i in ids:
                d = min(adm, key=lambda x: ((m[x] + 1) * cost[x], x))
                m[d] += 1
                rail[i], off[i] = d, T[d]
                T[d] += int(s.len[i]); A[d] += int(s.len[i])
            mode.append(2)
    return rail, off, T, A, mode, rr


def test_weighted_spray_worked_example(oracle):
    rows = read_golden("weighted_spray_worked_example.txt")
    rails = W.make_rails([25000, 50000], lat_ns=0)
    w = one_transfer(9 * 64 * KiB, 64 * KiB, rails)
    s = oracle.split(w.src_ptr, w.src_ext, 64 * KiB)
    r = oracle.dispatch(s, rails, W.make_dispatch_params(64 * KiB))
    assert r.binding.status == oracle.OK and r.mode.tolist() == [2]
    assert r.binding.rail.tolist() == rows[0]
    assert r.binding.stage_off.tolist() == rows[1]
    assert r.binding.T.tolist() == rows[2]


@pytest.mark.parametrize("seed", range(16))
def test_dispatch_matches_the_literal_python_version(oracle, seed):
    rng = np.random.Generator(np.random.PCG64(9100 + seed))
    R = int(rng.integers(1, 9))
    S = int(rng.choice([4 * KiB, 64 * KiB]))
    D = int(rng.integers(1, 40))
    lens = np.where(rng.random(D) < 0.5, rng.integers(1, 3 * S, D), rng.integers(1, 40 * S, D))
    rails = W.make_rails(rng.integers(1000, 400000, R), lat_ns=rng.integers(0, 20000, R),
                         queued=rng.integers(0, 1 << 22, R), health=rng.choice([0, 0, 0, 1, 2], R),
                         penalty_q8=rng.choice([256, 256, 384], R))
    w = requests(lens, S, rails)
    s = oracle.split(w.src_ptr, w.src_ext, S)
    prio = W.make_priorities(seed, D)
    done = (rng.random(s.n) < 0.2).astype(np.uint8)
    dp = W.make_dispatch_params(int(rng.choice([S, 2 * S, 8 * S])), gamma_q8=int(rng.choice([0, 26, 128, 1000])),
                                window=int(rng.integers(0, 7)), rr_start=int(rng.integers(0, 5)))
    r = oracle.dispatch(s, rails, dp, priority=prio, done=done)
    if (rails["health"] == 2).all():
        assert r.binding.status == oracle.DEFER and not r.bound.any()
        return
    rail, off, T, A, mode, rr = literal_dispatch(s, rails, dp, prio, done)
    assert r.mode.tolist() == mode and r.rr_end == rr
    ids = sorted(rail)
    assert np.flatnonzero(r.bound).tolist() == ids
    assert [int(r.binding.rail[i]) for i in ids] == [rail[i] for i in ids]
    assert [int(r.binding.stage_off[i]) for i in ids] == [off[i] for i in ids]
    assert r.binding.T.tolist() == T and r.binding.A_after.tolist() == A


def test_elephant_shares_follow_the_efficiency_weights(oracle):
    # W_d = 1 / s_d: the number of slices a rail receives stays within one of its proportional share
    rails = W.make_rails([12500, 25000, 50000, 100000, 33000], lat_ns=[0, 5000, 5000, 20000, 0])
    w = one_transfer(1000 * 64 * KiB, 64 * KiB, rails)
    s = oracle.split(w.src_ptr, w.src_ext, 64 * KiB)
    r = oracle.dispatch(s, rails, W.make_dispatch_params(64 * KiB))
    c0, c1, _, _ = oracle.coeffs(rails)
    cost = [Fraction(oracle.cost(int(c0[d]), int(c1[d]), 0, 64 * KiB)) for d in range(5)]
    total_w = sum(1 / c for c in cost)
    for d in range(5):
        share = 1000 * (1 / cost[d]) / total_w
        assert abs(int(r.binding.n_slices[d]) - share) < 1 + 1e-9
    # the order is the merge of the rails' arithmetic slot sequences (k+1) * s_d, ties to the lower rail
    keys = sorted((int((k + 1) * cost[d]), d) for d in range(5) for k in range(int(r.binding.n_slices[d]) + 1))
    assert r.binding.rail.tolist() == [d for _, d in keys[:1000]]


def test_elephants_on_identical_rails_go_round_robin(oracle):
    rails = W.make_rails([50000] * 4)
    w = requests([10 * 64 * KiB, 7 * 64 * KiB + 5], 64 * KiB, rails)
    s = oracle.split(w.src_ptr, w.src_ext, 64 * KiB)
    r = oracle.dispatch(s, rails, W.make_dispatch_params(1))
    assert r.binding.rail[:10].tolist() == [0, 1, 2, 3, 0, 1, 2, 3, 0, 1]
    # the second request sees rails 0 and 1 one slice deeper, so it starts on rails 2 and 3
    assert r.binding.rail[10:].tolist() == [2, 3, 0, 1, 2, 3, 0, 1]
    assert int(r.binding.T.sum()) == w.payload


def test_mice_round_robin_within_the_tolerance(oracle):
    S = 64 * KiB
    # 5 us of fixed latency dominate a 4 KiB request, so rails 0 and 2 stay within 10 % of each other for all
    # six requests; rail 1 carries a topology penalty of 2.0 and never qualifies
    rails = W.make_rails([50000, 50000, 48000], penalty_q8=np.array([256, 512, 256]))
    w = requests([4 * KiB] * 6, S, rails)
    s = oracle.split(w.src_ptr, w.src_ext, S)
    r = oracle.dispatch(s, rails, W.make_dispatch_params(S, gamma_q8=26))
    assert r.mode.tolist() == [1] * 6 and r.rr_end == 6
    assert r.binding.rail.tolist() == [0, 2, 0, 2, 0, 2]
    # no tolerance: always the cheapest rail of the moment (the per-request earliest-completion choice)
    r = oracle.dispatch(s, rails, W.make_dispatch_params(S, gamma_q8=0))
    ref = oracle.bind(s.len, rails)
    assert (r.binding.rail == ref.rail).all() and (r.binding.stage_off == ref.stage_off).all()
    # unbounded tolerance: plain round robin over every admitted rail, from the counter's start value
    r = oracle.dispatch(s, rails, W.make_dispatch_params(S, gamma_q8=60000, rr_start=2))
    assert r.binding.rail.tolist() == [2, 0, 1, 2, 0, 1] and r.rr_end == 8


def test_tolerance_boundary(oracle):
    # s_min = 1,310,720 ps (50 GB/s, 64 KiB); gamma = 128/256 admits costs up to 1,966,080 ps exactly
    S = 64 * KiB
    c1_at = lambda bw: 10**6 * 256 * 256 // bw
    edge_bw = next(bw for bw in range(33000, 34000) if c1_at(bw) <= 1966080 < c1_at(bw - 1))
    for bw, inside in ((edge_bw, True), (edge_bw - 1, False)):
        rails = W.make_rails([50000, bw], lat_ns=0)
        w = requests([S], S, rails)                           # one whole slice, a mice request under theta = S + 1
        s = oracle.split(w.src_ptr, w.src_ext, S)
        # the counter starts at 1: the request lands on rail 1 iff rail 1 is a candidate
        r = oracle.dispatch(s, rails, W.make_dispatch_params(S + 1, gamma_q8=128, rr_start=1))
        assert (int(r.binding.rail[0]) == 1) == inside


def test_mode_follows_the_request_length(oracle):
    S = 64 * KiB
    rails = W.make_rails([25000, 50000, 100000])
    w = requests([S, 3 * S - 1, 3 * S, 3 * S + 1, 20 * S], S, rails)
    s = oracle.split(w.src_ptr, w.src_ext, S)
    r = oracle.dispatch(s, rails, W.make_dispatch_params(3 * S, gamma_q8=0))
    assert r.mode.tolist() == [1, 1, 2, 2, 2]
    for j in (0, 1):                                          # a mice request is not sprayed, whatever its slice count
        assert np.unique(r.binding.rail[int(s.first[j]):int(s.first[j + 1])]).shape[0] == 1
    assert np.unique(r.binding.rail[int(s.first[4]):]).shape[0] == 3


def test_mice_cost_uses_the_request_length(oracle):
    # Algorithm 1 takes the request length L: a 4-slice mice request (256 KiB) is cheaper on the fast rail with
    # the long latency (20 us + 0.66 us = 20.66 us) than on the slow one (5 us + 20.97 us), although a single
    # slice would be cheaper on the slow rail (10.24 us against 20.16 us)
    S = 64 * KiB
    rails = W.make_rails([400000, 12500], lat_ns=np.array([20000, 5000]))
    w = requests([4 * S, S], S, rails)
    s = oracle.split(w.src_ptr, w.src_ext, S)
    r = oracle.dispatch(s, rails, W.make_dispatch_params(8 * S, gamma_q8=0))
    assert r.mode.tolist() == [1, 1]
    assert r.binding.rail.tolist() == [0, 0, 0, 0, 1]


def test_priority_slots(oracle):
    # Section 4.2 "Quality of Service": in window w rail d is in slot (w + d) mod 3; HIGH-only, HIGH+MID, all
    S = 64 * KiB
    rails = W.make_rails([50000] * 6)
    w = requests([30 * S] * 3, S, rails)
    s = oracle.split(w.src_ptr, w.src_ext, S)
    prio = np.array([0, 1, 2], dtype=np.uint8)                # LOW, MID, HIGH
    for window in range(4):
        r = oracle.dispatch(s, rails, W.make_dispatch_params(1, window=window), priority=prio)
        slot = [(window + d) % 3 for d in range(6)]
        used = [set(r.binding.rail[int(s.first[j]):int(s.first[j + 1])].tolist()) for j in range(3)]
        assert used[0] == {d for d in range(6) if slot[d] == 2}
        assert used[1] == {d for d in range(6) if slot[d] >= 1}
        assert used[2] == set(range(6))
    # one rail only: a LOW request waits for the window in which the rail accepts it
    rails = W.make_rails([50000])
    w = requests([S, 5 * S], S, rails)
    s = oracle.split(w.src_ptr, w.src_ext, S)
    prio = np.array([0, 1], dtype=np.uint8)
    modes = [oracle.dispatch(s, rails, W.make_dispatch_params(2 * S, window=k), priority=prio).mode.tolist() for k in range(3)]
    assert modes == [[3, 3], [3, 2], [1, 2]]
    r = oracle.dispatch(s, rails, W.make_dispatch_params(2 * S, window=0), priority=prio)
    assert r.binding.status == oracle.OK and not r.bound.any() and int(r.binding.T.sum()) == 0
    # without priorities every request counts as HIGH
    assert oracle.dispatch(s, rails, W.make_dispatch_params(2 * S, window=0)).mode.tolist() == [1, 2]


def test_dispatch_bookkeeping(oracle):
    w = W.small_variant("kv_migration")
    s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
    rng = np.random.Generator(np.random.PCG64(3))
    done = (rng.random(s.n) < 0.3).astype(np.uint8)
    prio = W.make_priorities(3, w.n_desc)
    # two rails in the HIGH-only and the HIGH+MID window: LOW requests find no admitted rail
    rails = W.make_rails([50000, 400000], queued=rng.integers(0, 1 << 20, 2))
    r = oracle.dispatch(s, rails, W.make_dispatch_params(4 * w.slice_bytes, window=0), priority=prio, done=done)
    b = r.binding
    dealt = np.flatnonzero(r.bound)
    assert not (done[dealt]).any()
    deferred = np.flatnonzero(r.mode == 3)
    assert deferred.shape[0] > 0
    pending_of_deferred = np.concatenate([np.arange(s.first[j], s.first[j + 1]) for j in deferred]).astype(int)
    assert not r.bound[pending_of_deferred].any()
    assert set(np.flatnonzero((done == 0) & (r.bound == 0)).tolist()) == set(pending_of_deferred[done[pending_of_deferred] == 0].tolist())
    for d in range(rails.shape[0]):
        on = dealt[b.rail[dealt] == d]
        assert int(s.len[on].astype(np.uint64).sum()) == int(b.T[d]) and on.shape[0] == int(b.n_slices[d])
        assert np.array_equal(np.sort(b.stage_off[on]), np.concatenate([[0], np.cumsum(s.len[on][np.argsort(b.stage_off[on])].astype(np.uint64))[:-1]]).astype(np.uint64))
    assert (b.A_after == rails["queued_bytes"] + b.T).all()
    # all rails excluded: deferred as a whole
    r = oracle.dispatch(s, W.make_rails(w.rails["bw_MBps"], health=2), W.make_dispatch_params(1))
    assert r.binding.status == oracle.DEFER and not r.bound.any()
