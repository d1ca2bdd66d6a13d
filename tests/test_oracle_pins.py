"""Pins for the CPU oracle: printed values, closed forms, invariants, special cases and
brute force.  None of these tests touches the HIP engine.

Each test names the passage of the paper (or the reading of it) that fixes the expected value.
"""
from fractions import Fraction

import numpy as np
import pytest

from paper_2604_00368_amd import workloads as W
from helpers import (check_greedy_choice, exact_cost, expected_destination, int_cost, logical_bytes,
                     read_golden)

KiB, MiB = 1 << 10, 1 << 20


def one_transfer(nbytes, S, rails):
    ptr = np.array([0, 1], dtype=np.uint32)
    se = W._extents(0, [0], nbytes)
    de = W._extents(1, [0], nbytes)
    return W.Workload("one", 0, S, [nbytes, nbytes], ptr, se, ptr.copy(), de, rails, "u8")


# ---------------------------------------------------------------- slice geometry
def test_slice_count_printed_in_paper(oracle):
    # Section 4.2, figure "Spraying 1MB data (16 slices) among two devices"
    for payload, S, n_expected, n_dev in read_golden("paper_fig_slice_spraying.txt"):
        w = one_transfer(payload, S, W.make_rails([25000] * n_dev))
        s = oracle.split(w.src_ptr, w.src_ext, S)
        assert s.n == n_expected
        assert int(s.len.astype(np.uint64).sum()) == payload


@pytest.mark.parametrize("name", ["tiny", "kv_migration", "rl_params", "many_small"])
def test_slices_tile_every_transfer_exactly_once(oracle, name):
    # Section 4.2 "Slice Decomposition": slices partition the payload; each carries its offset.
    w = W.CONFIGS[name]()
    S = w.slice_bytes
    s = oracle.split(w.src_ptr, w.src_ext, S)
    seg_sum = np.add.reduceat(w.src_ext["len"].astype(np.uint64), w.src_ptr[:-1].astype(np.int64))
    cnt = (seg_sum + np.uint64(S - 1)) // np.uint64(S)
    first = np.concatenate([[0], np.cumsum(cnt)]).astype(np.uint64)       # textbook exclusive scan
    assert np.array_equal(s.first, first)
    assert s.n == int(cnt.sum())
    # per descriptor: offsets 0, S, 2S, ...; all full but the last; lengths sum to the transfer length
    assert np.array_equal(s.desc, np.repeat(np.arange(w.n_desc, dtype=np.uint32), cnt.astype(np.int64)))
    k = np.arange(s.n, dtype=np.uint64) - first[s.desc]
    assert np.array_equal(s.off, k * np.uint64(S))
    rest = seg_sum[s.desc] - s.off
    assert np.array_equal(s.len.astype(np.uint64), np.minimum(rest, np.uint64(S)))
    assert (s.len > 0).all()
    assert np.array_equal(np.add.reduceat(s.len.astype(np.uint64), first[:-1].astype(np.int64)), seg_sum)


def test_config_sizes_match_the_published_shapes(oracle):
    w = W.rl_params()
    assert w.notes["params"] == 7_504_924_672 and w.payload == 15_009_849_344
    s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
    assert s.n == 14_379 and int((s.len == 8 * KiB).sum()) == 65
    w5 = W.many_small(layers=6)
    n5 = oracle.split(w5.src_ptr, w5.src_ext, w5.slice_bytes).n
    assert 0.9e6 < n5 < 1.1e6                                   # "~1M slices planned per call"


def test_short_transfer_is_one_short_slice(oracle):
    w = one_transfer(100, 64 * KiB, W.make_rails([25000]))
    s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
    assert s.n == 1 and int(s.len[0]) == 100 and int(s.off[0]) == 0


# ---------------------------------------------------------------- cost model
def test_idle_rail_costs_closed_form(oracle):
    # Eq. 1 with A = 0: beta0 + L / B; 200 Gbps = 25.0 GB/s (Table "peak-bandwidth")
    for bw, expected in read_golden("idle_rail_costs.txt"):
        c0, c1, ex, A = oracle.coeffs(W.make_rails([bw]))
        assert oracle.cost(int(c0[0]), int(c1[0]), 0, 64 * KiB) == expected
        assert Fraction(expected) == Fraction(5_000_000) + Fraction(64 * KiB * 10**12, bw * 10**6)


def test_cost_tracks_exact_rational_eq1(oracle):
    # fixed point floors three times (c0, c1, the shift): 0 <= exact - fixed < (A+L)/2^16 + 2 ps
    rng = np.random.Generator(np.random.PCG64(11))
    for _ in range(400):
        rails = W.make_rails([int(rng.integers(1000, 400001))], lat_ns=int(rng.integers(0, 50000)),
                             beta1_q8=int(rng.integers(1, 2048)), penalty_q8=int(rng.integers(1, 2048)))
        A = int(rng.integers(0, 1 << 30))      # keeps (A+L)*c1 inside 63 bits (the engine's precondition)
        L = int(rng.integers(1, 1 << 24))
        c0, c1, ex, _ = oracle.coeffs(rails)
        fixed = oracle.cost(int(c0[0]), int(c1[0]), A, L)
        exact = exact_cost(rails[0], A, L)
        assert 0 <= exact - fixed < Fraction(A + L, 1 << 16) + 2
        assert fixed == int_cost(c0[0], c1[0], A, L)


def test_penalty_and_beta1_scale_the_cost(oracle):
    # Section 4.2: s = P * t.  P = 5.0 (cross-NUMA example) multiplies both terms; beta1 only the queue term.
    base = W.make_rails([50000])
    pen = W.make_rails([50000], penalty_q8=5 * 256)
    b1 = W.make_rails([50000], beta1_q8=2 * 256)
    cost = {}
    for k, r in (("base", base), ("pen", pen), ("b1", b1)):
        c0, c1, _, _ = oracle.coeffs(r)
        cost[k] = oracle.cost(int(c0[0]), int(c1[0]), 3 * MiB, MiB)
    assert cost["pen"] == 5 * cost["base"]
    assert cost["b1"] - 5_000_000 == 2 * (cost["base"] - 5_000_000)


# ---------------------------------------------------------------- rail choice
def test_two_rail_worked_example(oracle):
    rows = read_golden("two_rail_worked_example.txt")
    w = one_transfer(MiB, 64 * KiB, W.make_rails([25000, 100000]))
    s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
    b = oracle.bind(s.len, w.rails)
    assert b.status == oracle.OK
    assert b.rail.tolist() == rows[0]
    assert b.T.tolist() == rows[1]
    c0, c1, _, _ = oracle.coeffs(w.rails)
    assert [oracle.cost(int(c0[1]), int(c1[1]), k * 64 * KiB, 64 * KiB) for k in range(4)] == rows[2]
    # each rail's staging offsets count its own bytes, in index order
    for d in (0, 1):
        assert b.stage_off[b.rail == d].tolist() == [k * 64 * KiB for k in range(int(b.n_slices[d]))]


@pytest.mark.parametrize("seed", range(6))
def test_greedy_choice_brute_force(oracle, seed):
    # Section 4.2, opening rule: a slice is bound to the rail whose predicted completion, from current telemetry, is earliest.
    w = W.ragged(seed, n_desc=10, max_len=60_000, slice_bytes=4096 + 7 * seed, n_rails=3 + seed)
    s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
    b = oracle.bind(s.len, w.rails)
    c0, c1, ex, _ = oracle.coeffs(w.rails)
    A, T = check_greedy_choice(s.len, w.rails, b.rail, b.stage_off, c0, c1, ex)
    assert b.A_after.tolist() == A and b.T.tolist() == T


def test_greedy_choice_on_tiny_config(oracle):
    w = W.tiny()
    s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
    b = oracle.bind(s.len, w.rails)
    c0, c1, ex, _ = oracle.coeffs(w.rails)
    check_greedy_choice(s.len, w.rails, b.rail, b.stage_off, c0, c1, ex)
    assert not (b.rail == 1).any()                               # rail 1 is marked unhealthy


def test_single_admitted_rail_takes_everything(oracle):
    w = W.tiny()
    rails = w.rails.copy()
    rails["health"] = [2, 2, 0, 2]
    s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
    b = oracle.bind(s.len, rails)
    assert (b.rail == 2).all()
    assert np.array_equal(b.stage_off, np.concatenate([[0], np.cumsum(s.len.astype(np.uint64))[:-1]]))


def test_identical_idle_rails_round_robin(oracle):
    R = 7
    w = one_transfer(40 * 64 * KiB, 64 * KiB, W.make_rails([50000] * R))
    s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
    b = oracle.bind(s.len, w.rails)
    assert b.rail.tolist() == [i % R for i in range(40)]


def test_no_admitted_rail_defers(oracle):
    # Algorithm 1, Stage 1: empty admitted set -> defer, nothing is bound
    w = W.tiny()
    rails = w.rails.copy()
    rails["health"] = 2
    s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
    b = oracle.bind(s.len, rails)
    assert b.status == oracle.DEFER
    assert (b.rail == 0xFFFFFFFF).all() and int(b.T.sum()) == 0
    assert np.array_equal(b.A_after, rails["queued_bytes"])


@pytest.mark.parametrize("name", ["kv_migration", "rl_params", "many_small"])
def test_plan_invariants_full_configs(oracle, name):
    w = W.CONFIGS[name]()
    s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
    b = oracle.bind(s.len, w.rails)
    R = w.rails.shape[0]
    lens = s.len.astype(np.uint64)
    # totals: per-rail bytes are the summed slice lengths; all bytes are bound; queue feedback
    T = np.bincount(b.rail, weights=None, minlength=R)
    assert np.array_equal(T.astype(np.uint64), b.n_slices)
    bytes_per_rail = np.array([int(lens[b.rail == d].sum()) for d in range(R)], dtype=np.uint64)
    assert np.array_equal(bytes_per_rail, b.T)
    assert int(b.T.sum()) == w.payload
    assert np.array_equal(b.A_after, w.rails["queued_bytes"] + b.T)
    # staging offsets inside a rail: gap-free, in index order
    for d in range(R):
        sel = b.rail == d
        assert np.array_equal(b.stage_off[sel], np.concatenate([[0], np.cumsum(lens[sel])[:-1]]).astype(np.uint64))
    # region bases: exclusive sum of 256-byte-rounded totals
    rounded = (b.T + np.uint64(255)) // np.uint64(256) * np.uint64(256)
    assert np.array_equal(b.base, np.concatenate([[0], np.cumsum(rounded)[:-1]]).astype(np.uint64))
    # equal latencies: the rails' predicted drain times end within one largest-slice time of each other,
    # so byte shares track bandwidth shares (Section 5.2 "Device-to-Device": per-NIC byte counters)
    bw = w.rails["bw_MBps"].astype(np.float64)
    finish = b.A_after.astype(np.float64) / bw
    assert finish.max() - finish.min() <= w.slice_bytes / bw.min() * 1.0001
    share = b.T.astype(np.float64) / w.payload
    assert np.abs(share - bw / bw.sum()).max() < 0.01


@pytest.mark.parametrize("seed", range(4))
def test_uniform_run_is_a_merge_of_sorted_rail_sequences(oracle, seed):
    # For equal-length slices the greedy picks the m smallest of all (cost, rail, slot) triples:
    # no bound slot costs more than any still-free slot.
    rng = np.random.Generator(np.random.PCG64(100 + seed))
    R = int(rng.integers(2, 12))
    rails = W.make_rails(rng.integers(5000, 400000, size=R), lat_ns=rng.integers(0, 9000, size=R),
                         queued=rng.integers(0, 1 << 24, size=R))
    m, L = int(rng.integers(50, 400)), int(rng.integers(1, 1 << 20))
    w = one_transfer(m * L, L, rails)
    s = oracle.split(w.src_ptr, w.src_ext, L)
    b = oracle.bind(s.len, rails)
    c0, c1, _, A0 = oracle.coeffs(rails)
    slot_cost = lambda d, k: int_cost(c0[d], c1[d], int(A0[d]) + k * L, L)
    n = [int(x) for x in b.n_slices]
    taken = [(slot_cost(d, k), d, k) for d in range(R) for k in range(n[d])]
    free = [(slot_cost(d, n[d]), d, n[d]) for d in range(R)]
    assert max(taken) < min(free)
    # and the order in which slots were taken is the sorted order of those triples
    order = sorted(taken)
    assert b.rail.tolist() == [d for (_, d, _) in order]


# ---------------------------------------------------------------- bytes
@pytest.mark.parametrize("name", ["tiny", "kv_migration", "rl_params", "many_small"])
def test_destination_bytes_match_the_definition(oracle, name):
    w = W.small_variant(name)
    s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
    b = oracle.bind(s.len, w.rails)
    src = W.fill_numpy(w, 0)
    dst = np.full(w.seg_bytes[1], 0xA5, dtype=np.uint8)
    want = expected_destination(w, src, dst)
    staging = np.zeros(w.staging_bytes, dtype=np.uint8)
    oracle.execute(w, s, b, [src, dst], staging)
    assert np.array_equal(dst, want)
    # staging region of rail d = its slices' source bytes, concatenated in index order
    for d in range(w.rails.shape[0]):
        parts = []
        for i in np.nonzero(b.rail == d)[0]:
            j = int(s.desc[i])
            data = logical_bytes({0: src}, w.src_ext[w.src_ptr[j]:w.src_ptr[j + 1]])
            parts.append(data[int(s.off[i]):int(s.off[i]) + int(s.len[i])])
        region = np.concatenate(parts) if parts else np.zeros(0, np.uint8)
        lo = int(b.base[d])
        assert np.array_equal(staging[lo:lo + region.shape[0]], region)


@pytest.mark.parametrize("seed", range(5))
def test_ragged_bytes_and_untouched_gaps(oracle, seed):
    # odd lengths, 1-byte extents, source and destination cut differently; gaps must keep their bytes
    w = W.ragged(seed, slice_bytes=[1, 17, 4096, 5000, 65536][seed], n_desc=8, max_len=30_000, max_ext=700)
    s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
    b = oracle.bind(s.len, w.rails)
    src = W.fill_numpy(w, 0)
    dst = W.fill_numpy(w, 1)
    want = expected_destination(w, src, dst)
    staging = np.zeros(w.staging_bytes, dtype=np.uint8)
    oracle.execute(w, s, b, [src, dst], staging)
    assert np.array_equal(dst, want)
    assert not np.array_equal(want, W.fill_numpy(w, 1))


def test_destination_is_independent_of_rails_and_idempotent(oracle):
    # Section 4.2 / 4.3: absolute destination offsets make delivery order- and rail-independent; retries are safe
    w = W.small_variant("many_small")
    s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
    src = W.fill_numpy(w, 0)
    outs = []
    for variant in range(3):
        rails = w.rails.copy()
        if variant == 1:
            rails = rails[::-1].copy()
        if variant == 2:
            rails["health"][::2] = 2
        b = oracle.bind(s.len, rails)
        dst = np.zeros(w.seg_bytes[1], dtype=np.uint8)
        staging = np.zeros(w.staging_bytes, dtype=np.uint8)
        oracle.execute(w, s, b, [src, dst], staging)
        once = dst.copy()
        oracle.execute(w, s, b, [src, dst], staging)
        assert np.array_equal(dst, once)
        outs.append(once)
    assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[0], outs[2])


# ---------------------------------------------------------------- re-planning epochs
def test_replanning_epochs(oracle):
    w = W.small_variant("replanning")
    s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
    src = W.fill_numpy(w, 0)
    dst = np.full(w.seg_bytes[1], 0x5A, dtype=np.uint8)
    want = expected_destination(w, src, dst)
    staging = np.zeros(w.staging_bytes, dtype=np.uint8)
    records, left = oracle.run_epochs(w, s, [src, dst], staging)
    assert left.shape[0] == 0
    assert np.array_equal(dst, want)
    done_all = np.concatenate([r["done_ids"] for r in records])
    assert np.array_equal(np.sort(done_all), np.arange(s.n))      # every slice completes exactly once
    assert int(s.len[done_all].astype(np.uint64).sum()) == w.payload
    assert sum(r["done_ids"].shape[0] > 0 for r in records[:-1]) >= 3   # progress spreads over epochs
    eps = list(w.epochs) + [w.drain]
    for e, (r, ep) in enumerate(zip(records, eps)):
        if r["rail"] is None:
            continue
        ex = ep.rails["health"] == 2
        assert not ex[r["rail"]].any()                           # nothing lands on a failed rail
        if e >= 5:
            assert not (r["rail"] == 3).any()
        if e >= 11:
            assert not (r["rail"] == 6).any()
        # FIFO drain: on each rail the completed slices are a prefix of its staging order
        done_mask = np.isin(r["pending"], r["done_ids"])
        for d in range(ep.rails.shape[0]):
            sel = r["rail"] == d
            so, dm = r["stage_off"][sel], done_mask[sel]
            assert (np.diff(so.astype(np.int64)) > 0).all()
            assert not (dm[1:] & ~dm[:-1]).any()
        c0, c1, exc, _ = oracle.coeffs(ep.rails)
        if r["pending"].shape[0] <= 400:
            rail_full = np.zeros(s.n, np.uint32); rail_full[r["pending"]] = r["rail"]
            so_full = np.zeros(s.n, np.uint64); so_full[r["pending"]] = r["stage_off"]
            check_greedy_choice(s.len, ep.rails, rail_full, so_full, c0, c1, exc, ids=r["pending"])


def test_degraded_rail_costs_twice(oracle):
    # Section 4.3: a DEGRADED rail keeps half its weight and can still be chosen
    healthy = W.make_rails([50000, 50000])
    degraded = W.make_rails([50000, 50000], health=[1, 0])
    c0h, c1h, exh, _ = oracle.coeffs(healthy)
    c0d, c1d, exd, _ = oracle.coeffs(degraded)
    assert int(c0d[0]) == 2 * int(c0h[0]) and int(c1d[0]) == 2 * int(c1h[0]) and not exd[0]
    assert int(c0d[1]) == int(c0h[1]) and int(c1d[1]) == int(c1h[1])
    # the degraded rail still takes traffic, about half as many bytes as its healthy twin would
    w = one_transfer(600 * 64 * KiB, 64 * KiB, degraded)
    s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
    b = oracle.bind(s.len, degraded)
    share = int(b.T[0]) / w.payload
    assert 0.30 < share < 0.36                                   # 1/3 of the bytes: weights 1 : 2
    c0, c1, ex, _ = oracle.coeffs(degraded)
    check_greedy_choice(s.len, degraded, b.rail, b.stage_off, c0, c1, ex)
    # with a healthy rail of half the bandwidth and half... the latency term doubles too: compare with P = 2
    same = W.make_rails([50000, 50000], penalty_q8=[512, 256])
    b2 = oracle.bind(s.len, same)
    assert np.array_equal(b.rail, b2.rail)


def test_region_bases_round_each_total_up_to_256(oracle):
    # odd byte totals: base_d = sum over d' < d of ceil(T_d' / 256) * 256
    w = W.ragged(3, n_desc=10, max_len=60_000, slice_bytes=4099, n_rails=6)
    s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
    b = oracle.bind(s.len, w.rails)
    assert (b.T % 256 != 0).any()
    want, at = [], 0
    for t in b.T.tolist():
        want.append(at)
        at += -(-t // 256) * 256
    assert b.base.tolist() == want


def test_retire_boundary_is_inclusive(oracle):
    # FIFO drain: queued bytes first, then the plan's slices; a slice whose last byte lands exactly on the budget completes
    rails = W.make_rails([50000], queued=100)
    w = one_transfer(3000, 1000, rails)
    s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
    b = oracle.bind(s.len, rails)
    for budget, n_done in [(99, 0), (1099, 0), (1100, 1), (2099, 1), (2100, 2), (3099, 2), (3100, 3), (10**9, 3)]:
        done = oracle.retire(s, b, rails["queued_bytes"], [budget])
        assert done.tolist() == [1] * n_done + [0] * (3 - n_done), budget
