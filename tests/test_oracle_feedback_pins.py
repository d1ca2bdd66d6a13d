"""Pins for the oracle's telemetry feedback (Eq. 2 peak picking and the smoothed bandwidth update)
and for the rail simulator's latencies.  CPU only."""
from fractions import Fraction

import numpy as np
import pytest

from paper_2604_00368_amd import workloads as W
from test_oracle_pins import one_transfer

KiB, MiB = 1 << 10, 1 << 20


def plan_one(oracle, nbytes, S, rails):
    w = one_transfer(nbytes, S, rails)
    s = oracle.split(w.src_ptr, w.src_ext, S)
    return w, s, oracle.bind(s.len, rails)


def test_simulated_latency_closed_form(oracle):
    # one idle 50 GB/s rail, 5 us latency: slice k finishes after (k+1) * 256 KiB / 50 GB/s + 5 us
    rails = W.make_rails([50000])
    w, s, b = plan_one(oracle, 8 * 256 * KiB, 256 * KiB, rails)
    tau = oracle.sim_latency(s, b, rails, [50000])
    for k in range(8):
        exact = Fraction(5000) + Fraction((k + 1) * 256 * KiB * 1000, 50000)      # ns
        assert 0 <= int(tau[k]) - exact < 1                                       # ceiling of the drain time
    # bytes queued before the plan drain first
    rails = W.make_rails([50000], queued=10 * MiB)
    tau_q = oracle.sim_latency(s, oracle.bind(s.len, rails), rails, [50000])
    assert int(tau_q[0]) == 5000 + -(-(10 * MiB + 256 * KiB) * 1000 // 50000)


def test_peak_picking_recovers_true_bandwidth_on_a_clean_rail(oracle):
    # Eq. 2 with alpha = 1, delta = fixed latency: the first slice of an idle rail saw no queueing, so
    # L / (tau - delta) is the rail's bandwidth; every later slice reports bw / (k+1) and the maximum picks the first
    for true_bw in (12500, 50000, 400000):
        rails = W.make_rails([true_bw])
        w, s, b = plan_one(oracle, 16 * 256 * KiB, 256 * KiB, rails)
        tau = oracle.sim_latency(s, b, rails, [true_bw])
        params = W.make_probe_params([2 * true_bw], alpha_q8=256, delta_ns=5000, ewma_q8=256)
        est, probe = oracle.probe(s, b, tau, params, [true_bw // 3])
        drain_ns = -(-256 * KiB * 1000 // true_bw)
        assert int(probe[0]) == 256 * KiB * 1000 // drain_ns
        assert 0 <= true_bw - int(probe[0]) <= true_bw // drain_ns + 1            # ceiling of tau costs < 1/tau relative
        assert int(est[0]) == int(probe[0])                                       # weight 1.0 replaces the estimate
        # the sample of slice k alone is bw/(k+1)
        for k in (1, 5):
            ids = np.array([k], dtype=np.uint32)
            _, pk = oracle.probe(s, b, tau, params, [1], ids=ids)
            # the ceiling of tau (in ns) costs at most one part in tau - delta
            exact_k = true_bw / (k + 1)
            assert 0 <= exact_k - int(pk[0]) <= exact_k / ((k + 1) * drain_ns - 1) + 2


def test_probe_formula_exact_rational(oracle):
    rng = np.random.Generator(np.random.PCG64(21))
    for _ in range(200):
        bw = int(rng.integers(1000, 400000))
        queued = int(rng.integers(0, 1 << 26))
        alpha = int(rng.integers(64, 1024))
        delta = int(rng.integers(0, 9000))
        L = int(rng.integers(1, 1 << 22))
        rails = W.make_rails([bw], lat_ns=int(rng.integers(0, 20000)), queued=queued)
        w, s, b = plan_one(oracle, L, 1 << 22, rails)
        tau = oracle.sim_latency(s, b, rails, [bw])
        lat = int(rails["lat_ns"][0])
        assert int(tau[0]) == lat + -(-(queued + L) * 1000 // bw)
        params = W.make_probe_params([1 << 31], alpha_q8=alpha, delta_ns=delta, ewma_q8=256)
        _, probe = oracle.probe(s, b, tau, params, [bw])
        if int(tau[0]) > delta:
            exact = Fraction(alpha, 256) * L * 1000 / (int(tau[0]) - delta)       # alpha * L / (tau - delta) in 1e6 B/s
            assert int(probe[0]) == min(1 << 31, int(exact))
        else:
            assert int(probe[0]) == 1 << 31


def test_hardware_bandwidth_caps_the_probe(oracle):
    rails = W.make_rails([50000])
    w, s, b = plan_one(oracle, 4 * 256 * KiB, 256 * KiB, rails)
    tau = oracle.sim_latency(s, b, rails, [50000])
    params = W.make_probe_params([25000], ewma_q8=256)
    est, probe = oracle.probe(s, b, tau, params, [10000])
    assert int(probe[0]) == 25000 and int(est[0]) == 25000
    # a latency at or below delta carries no rate information: it counts as the hardware bandwidth
    params = W.make_probe_params([25000], delta_ns=10**9, ewma_q8=256)
    _, probe = oracle.probe(s, b, tau, params, [10000])
    assert int(probe[0]) == 25000


def test_smoothing_recurrence_and_untouched_rails(oracle):
    # two rails, only rail 1 is admitted: rail 0 completes nothing and keeps its estimate
    rails = W.make_rails([50000, 50000], health=[2, 0])
    w, s, b = plan_one(oracle, 8 * 256 * KiB, 256 * KiB, rails)
    tau = oracle.sim_latency(s, b, rails, [50000, 40000])
    for weight in (0, 64, 128, 256):
        params = W.make_probe_params([10**6, 10**6], ewma_q8=weight)
        est = np.array([7777, 20000], dtype=np.uint32)
        probes = []
        for _ in range(12):
            new, probe = oracle.probe(s, b, tau, params, est)
            assert int(new[0]) == 7777 and int(probe[0]) == 0
            assert int(new[1]) == (weight * int(probe[1]) + (256 - weight) * int(est[1])) >> 8
            est = new
            probes.append(int(probe[1]))
        assert len(set(probes)) == 1                                             # same window, same peak
        target = probes[0]
        if weight == 0:
            assert int(est[1]) == 20000
        elif weight == 256:
            assert int(est[1]) == target
        else:
            # geometric approach from below; the floor keeps it within 256/weight of the target
            bound = target - (target - 20000) * (1 - weight / 256) ** 12
            assert bound - 256 / weight - 1 <= int(est[1]) <= target


def test_congested_window_underestimates_and_clean_slice_wins(oracle):
    # foreign bytes ahead of the plan inflate every latency; the window's best sample is still its first slice
    rails = W.make_rails([50000], queued=4 * MiB)
    w, s, b = plan_one(oracle, 32 * 256 * KiB, 256 * KiB, rails)
    tau = oracle.sim_latency(s, b, rails, [50000])
    params = W.make_probe_params([10**6], ewma_q8=256)
    _, probe = oracle.probe(s, b, tau, params, [50000])
    first = np.array([0], dtype=np.uint32)
    _, p_first = oracle.probe(s, b, tau, params, [50000], ids=first)
    assert int(probe[0]) == int(p_first[0])
    assert abs(int(probe[0]) - 50000 * 256 * KiB / (4 * MiB + 256 * KiB)) <= 3


def test_closed_loop_epochs(oracle):
    # the estimates follow the epochs' true bandwidths; every slice still completes exactly once
    w = W.small_variant("replanning")
    s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
    params = W.make_probe_params(2 * w.rails["bw_MBps"].astype(np.uint64), ewma_q8=128)
    records, left = oracle.run_epochs_closed_loop(w, s, params)
    assert left.shape[0] == 0
    done_all = np.concatenate([r["done_ids"] for r in records])
    assert np.array_equal(np.sort(done_all), np.arange(s.n))
    moved = 0
    for r, ep in zip(records, list(w.epochs) + [w.drain]):
        if r["probe"] is None:
            continue
        true_bw = ep.rails["bw_MBps"].astype(np.int64)
        seen = r["probe"] > 0
        assert (r["probe"][seen].astype(np.int64) <= true_bw[seen]).all()          # alpha = 1 never overshoots
        assert np.array_equal(r["est_after"][~seen], r["est"][~seen])
        lo = np.minimum(r["est"], r["probe"])[seen]
        hi = np.maximum(r["est"], r["probe"])[seen]
        assert ((r["est_after"][seen] >= lo - 1) & (r["est_after"][seen] <= hi)).all()   # between old and probe
        moved += int(seen.sum())
    assert moved > 10
