"""Pins for the oracle's bounded, pipelined staging (Section 4.1: chunks through a buffer of fixed size).  CPU only."""
import numpy as np
import pytest

from helpers import expected_destination, logical_bytes
from paper_2604_00368_amd import workloads as W

KiB, MiB = 1 << 10, 1 << 20


def brute_force_staging(w, s, b, src, ids, chunk_bytes, cap):
    """The staging buffer after a bounded execute, byte by byte with numpy from the definition: every payload
    byte knows its rail, its offset in the rail's region and its value; chunk after chunk the bytes of each rail
    are packed from the rail's chunk base in region order."""
    R = b.T.shape[0]
    P = np.concatenate([[0], np.cumsum(s.len.astype(np.int64))])
    payload = int(P[-1])
    rail = np.full(payload, -1, dtype=np.int64)
    reg = np.zeros(payload, dtype=np.int64)
    val = np.zeros(payload, dtype=np.uint8)
    for i in ids:
        j = int(s.desc[i])
        data = logical_bytes({0: src}, w.src_ext[w.src_ptr[j]:w.src_ptr[j + 1]])
        lo, n = int(P[i]), int(s.len[i])
        rail[lo:lo + n] = int(b.rail[i])
        reg[lo:lo + n] = int(b.stage_off[i]) + np.arange(n)
        val[lo:lo + n] = data[int(s.off[i]):int(s.off[i]) + n]
    staging = np.zeros(cap, dtype=np.uint8)
    peak = 0
    for c_lo in range(0, payload, chunk_bytes):
        sl = slice(c_lo, min(payload, c_lo + chunk_bytes))
        at = 0
        for d in range(R):
            m = rail[sl] == d
            if not m.any():
                continue
            r = reg[sl][m]
            staging[at + r - r.min()] = val[sl][m]
            at += -(-(int(r.max()) + 1 - int(r.min())) // 256) * 256
        peak = max(peak, at)
    return staging, peak


@pytest.mark.parametrize("name,chunk", [("tiny", 256 * KiB), ("tiny", 1 * MiB), ("kv_migration", 2 * MiB), ("many_small", 1 * MiB)])
def test_bounded_execute_against_the_definition(oracle, name, chunk):
    w = W.small_variant(name)
    s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
    b = oracle.bind(s.len, w.rails)
    src, dst0 = W.fill_numpy(w, 0), W.fill_numpy(w, 1)
    cap = chunk + 256 * w.rails.shape[0]
    dst = dst0.copy()
    staging = np.zeros(cap + 4096, dtype=np.uint8)
    staging[cap:] = 0xA5                                       # guard zone behind the buffer
    assert oracle.execute_bounded(w, s, b, [src, dst], staging[:cap], chunk) == 0
    assert np.array_equal(dst, expected_destination(w, src, dst0))      # Section 4.4: every byte at its final offset
    assert (staging[cap:] == 0xA5).all()
    want, peak = brute_force_staging(w, s, b, src, np.arange(s.n), chunk, cap)
    assert np.array_equal(staging[:cap], want)
    assert peak <= cap and chunk < w.payload


@pytest.mark.parametrize("seed", [0, 1])
def test_bounded_execute_with_odd_lengths(oracle, seed):
    # lengths, slice size and chunk size share no factor: chunks cut slices anywhere and the per-rail regions of a
    # chunk need their 256-byte rounding
    w = W.ragged(seed, n_desc=12, max_len=60_000)
    w.rails = W.make_rails([50000, 40000, 60000], lat_ns=0)   # every rail takes its share
    s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
    b = oracle.bind(s.len, w.rails)
    assert (b.T > 0).all()
    src, dst0 = W.fill_numpy(w, 0), W.fill_numpy(w, 1)
    chunk = 50_001
    cap = chunk + 256 * w.rails.shape[0]
    dst, staging = dst0.copy(), np.zeros(cap, dtype=np.uint8)
    assert oracle.execute_bounded(w, s, b, [src, dst], staging, chunk) == 0
    assert np.array_equal(dst, expected_destination(w, src, dst0))
    want, peak = brute_force_staging(w, s, b, src, np.arange(s.n), chunk, cap)
    assert np.array_equal(staging, want) and peak > chunk


def test_slots_hold_alternating_chunks(oracle):
    # two slots: even chunks in the first, odd chunks in the second; each slot ends up exactly as a one-slot
    # run over only its own chunks would leave it, and the destination is the same
    w = W.small_variant("kv_migration")
    s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
    b = oracle.bind(s.len, w.rails)
    src, dst0 = W.fill_numpy(w, 0), W.fill_numpy(w, 1)
    chunk = 2 * MiB
    slot = chunk + 256 * w.rails.shape[0]
    dst, staging = dst0.copy(), np.zeros(2 * slot, dtype=np.uint8)
    assert oracle.execute_bounded(w, s, b, [src, dst], staging, chunk, slots=2, slot_bytes=slot) == 0
    assert np.array_equal(dst, expected_destination(w, src, dst0))
    P = np.concatenate([[0], np.cumsum(s.len.astype(np.int64))])
    for parity in (0, 1):
        # brute force over the payload with the other parity's chunks blanked out
        ids = [i for i in range(s.n)]
        want = np.zeros(slot, dtype=np.uint8)
        full, _ = None, None
        rail = np.full(int(P[-1]), -1, dtype=np.int64)
        reg = np.zeros(int(P[-1]), dtype=np.int64)
        val = np.zeros(int(P[-1]), dtype=np.uint8)
        for i in ids:
            j = int(s.desc[i])
            data = logical_bytes({0: src}, w.src_ext[w.src_ptr[j]:w.src_ptr[j + 1]])
            lo, n = int(P[i]), int(s.len[i])
            rail[lo:lo + n] = int(b.rail[i]); reg[lo:lo + n] = int(b.stage_off[i]) + np.arange(n)
            val[lo:lo + n] = data[int(s.off[i]):int(s.off[i]) + n]
        for c, c_lo in enumerate(range(0, int(P[-1]), chunk)):
            if c % 2 != parity:
                continue
            sl = slice(c_lo, min(int(P[-1]), c_lo + chunk))
            at = 0
            for d in range(w.rails.shape[0]):
                m = rail[sl] == d
                if m.any():
                    r = reg[sl][m]
                    want[at + r - r.min()] = val[sl][m]
                    at += -(-(int(r.max()) + 1 - int(r.min())) // 256) * 256
        assert np.array_equal(staging[parity * slot:(parity + 1) * slot], want)
    # slots that do not fit the buffer are refused
    assert oracle.execute_bounded(w, s, b, [src, dst0.copy()], staging[:slot], chunk, slots=2, slot_bytes=slot) == -1


def test_one_chunk_is_the_unbounded_execute(oracle):
    w = W.small_variant("kv_migration")
    s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
    b = oracle.bind(s.len, w.rails)
    src, dst0 = W.fill_numpy(w, 0), W.fill_numpy(w, 1)
    d1, d2 = dst0.copy(), dst0.copy()
    st1 = np.zeros(w.staging_bytes, dtype=np.uint8)
    st2 = np.zeros(w.staging_bytes, dtype=np.uint8)
    oracle.execute(w, s, b, [src, d1], st1)
    assert oracle.execute_bounded(w, s, b, [src, d2], st2, w.payload) == 0
    assert np.array_equal(d1, d2) and np.array_equal(st1, st2)


def test_partial_sets_and_capacity(oracle):
    # only the slices that stayed bound move (a FIFO prefix of every rail, as after the rail simulator)
    w = W.small_variant("kv_migration")
    s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
    b = oracle.bind(s.len, w.rails)
    done = oracle.retire(s, b, w.rails["queued_bytes"], b.T // 2).astype(bool)      # every rail drains half its bytes
    ids = np.flatnonzero(done).astype(np.uint32)
    assert s.n // 4 < ids.shape[0] < s.n
    src, dst0 = W.fill_numpy(w, 0), W.fill_numpy(w, 1)
    chunk = 1 * MiB
    cap = chunk + 256 * w.rails.shape[0]
    dst, staging = dst0.copy(), np.zeros(cap, dtype=np.uint8)
    assert oracle.execute_bounded(w, s, b, [src, dst], staging, chunk, ids=ids) == 0
    want, _ = brute_force_staging(w, s, b, src, ids, chunk, cap)
    assert np.array_equal(staging, want)
    # destination: moved slices by definition, everything else untouched
    full = expected_destination(w, src, dst0)
    mask = np.zeros(dst.shape[0], dtype=bool)
    for i in ids:
        j = int(s.desc[i])
        pos = 0
        for e in w.dst_ext[w.dst_ptr[j]:w.dst_ptr[j + 1]]:
            lo = max(pos, int(s.off[i])); hi = min(pos + int(e["len"]), int(s.off[i]) + int(s.len[i]))
            if lo < hi:
                mask[int(e["off"]) + lo - pos:int(e["off"]) + hi - pos] = True
            pos += int(e["len"])
    assert np.array_equal(dst[mask], full[mask]) and np.array_equal(dst[~mask], dst0[~mask])
    # a buffer smaller than a chunk's need is refused and nothing moves
    dst2, small = dst0.copy(), np.zeros(chunk // 2, dtype=np.uint8)
    assert oracle.execute_bounded(w, s, b, [src, dst2], small, chunk) == -1
    assert np.array_equal(dst2, dst0) and not small.any()
