"""Checker-side helpers: results written out from their plain definitions (numpy / Python ints).

None of this is used by the engine or by the oracle; tests use it to pin both.
"""
from __future__ import annotations

import os
from fractions import Fraction

import numpy as np

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def read_golden(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append([int(x) for x in line.split()])
    return rows


def logical_bytes(pools, ext):
    """The byte string a descriptor side denotes: its extents concatenated in list order."""
    parts = [pools[int(e["seg"])][int(e["off"]):int(e["off"]) + int(e["len"])] for e in ext]
    return np.concatenate(parts) if parts else np.zeros(0, dtype=np.uint8)


def expected_destination(w, src_pool, dst_before):
    """Destination pool after the transfer, by definition: DST_j[x] = SRC_j[x] for every
    descriptor j and logical byte x; every byte outside declared extents keeps its value."""
    out = dst_before.copy()
    pools = {0: src_pool, 1: out}
    for j in range(w.n_desc):
        data = logical_bytes({0: src_pool}, w.src_ext[w.src_ptr[j]:w.src_ptr[j + 1]])
        pos = 0
        for e in w.dst_ext[w.dst_ptr[j]:w.dst_ptr[j + 1]]:
            n = int(e["len"])
            pools[int(e["seg"])][int(e["off"]):int(e["off"]) + n] = data[pos:pos + n]
            pos += n
        assert pos == data.shape[0]
    return out


def exact_cost(rail, A, L):
    """Eq. 1 scaled by the penalty, in exact rationals, in picoseconds, from the quantised telemetry."""
    beta0 = Fraction(int(rail["lat_ns"]) * 1000)
    beta1 = Fraction(int(rail["beta1_q8"]), 256)
    P = Fraction(int(rail["penalty_q8"]), 256)
    B = Fraction(int(rail["bw_MBps"]) * 10**6, 10**12)          # bytes per picosecond
    return P * (beta0 + beta1 * Fraction(A + L) / B)


def int_cost(c0, c1, A, L):
    return int(c0) + (((int(A) + int(L)) * int(c1)) >> 16)


def check_greedy_choice(lens, rails, rail_of, stage_off, c0, c1, excluded, ids=None):
    """Every slice sits on the admitted rail whose predicted completion cost, under the bytes
    in flight at its turn, is smallest (lowest index on ties); its staging offset is the
    number of bytes bound to that rail before it.  Python ints throughout."""
    R = len(c0)
    A = [int(x) for x in rails["queued_bytes"]]
    T = [0] * R
    order = range(len(lens)) if ids is None else [int(i) for i in ids]
    for i in order:
        L = int(lens[i])
        costs = [(int_cost(c0[d], c1[d], A[d], L), d) for d in range(R) if not excluded[d]]
        best = min(costs)[1]
        assert int(rail_of[i]) == best, (i, int(rail_of[i]), best, costs)
        assert int(stage_off[i]) == T[best], (i, int(stage_off[i]), T[best])
        A[best] += L
        T[best] += L
    return A, T
