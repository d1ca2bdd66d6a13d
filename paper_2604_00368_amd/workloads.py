"""Seeded synthetic transfer workloads.

This module only *describes* inputs: descriptor lists (CSR pointer arrays plus
extent records), rail telemetry vectors, and how the byte pools are filled.
It contains none of the engine's arithmetic (no slicing, no cost model, no
copying); both the HIP engine and the CPU checker consume the same arrays.

Shapes follow the workloads the paper evaluates on: paged KVCache migration
(Section 5.1.1), bulk parameter updates for RL pipelines (Section 5.1.2), the
fail-stop / degradation timeline of Section 5.3, and many small flows
(Section 2.2).  The production traffic itself is not available, so every
value is drawn from ``numpy.random.Generator(PCG64(seed))``.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

KiB = 1 << 10
MiB = 1 << 20

# struct { uint32 seg; uint32 len; uint64 off; }  -- 16 bytes
EXTENT_DTYPE = np.dtype(
    {"names": ["seg", "len", "off"], "formats": ["<u4", "<u4", "<u8"],
     "offsets": [0, 4, 8], "itemsize": 16})

# struct { uint32 bw_MBps; uint32 lat_ns; uint64 queued_bytes;
#          uint16 beta1_q8; uint16 penalty_q8; uint8 health; }  -- 24 bytes
RAIL_DTYPE = np.dtype(
    {"names": ["bw_MBps", "lat_ns", "queued_bytes", "beta1_q8", "penalty_q8", "health"],
     "formats": ["<u4", "<u4", "<u8", "<u2", "<u2", "u1"],
     "offsets": [0, 4, 8, 16, 18, 20], "itemsize": 24})

# struct { uint32 hw_MBps; uint32 alpha_q8; uint32 delta_ns; uint32 ewma_q8; }  -- 16 bytes
DISPATCH_PARAMS_DTYPE = np.dtype([("theta_bytes", "<u8"), ("gamma_q8", "<u4"), ("window", "<u4"), ("rr_start", "<u8")])
MONITOR_PARAMS_DTYPE = np.dtype([("err_threshold", "<u4"), ("recover_windows", "<u4"),
                                 ("cooldown_windows", "<u4"), ("degrade_q8", "<u4")])
PROBE_DTYPE = np.dtype(
    {"names": ["hw_MBps", "alpha_q8", "delta_ns", "ewma_q8"], "formats": ["<u4"] * 4,
     "offsets": [0, 4, 8, 12], "itemsize": 16})

HEALTHY = 0
DEGRADED = 1
EXCLUDED = 2

SRC_SEG = 0
DST_SEG = 1


def make_rails(bw_MBps, lat_ns=5000, queued=0, health=0, beta1_q8=256, penalty_q8=256):
    """Rail telemetry vector; scalars broadcast over rails."""
    bw = np.asarray(bw_MBps, dtype=np.uint64)
    r = np.zeros(bw.shape[0], dtype=RAIL_DTYPE)
    r["bw_MBps"] = bw
    r["lat_ns"] = lat_ns
    r["queued_bytes"] = queued
    r["beta1_q8"] = beta1_q8
    r["penalty_q8"] = penalty_q8
    r["health"] = health
    return r


def make_dispatch_params(theta_bytes, gamma_q8=26, window=0, rr_start=0):
    """Parameters of the request-level dispatch: mice/elephant threshold, cost tolerance (Q8.8, 26 = 10 %),
    index of the current priority window, start value of the round-robin counter."""
    return np.array([(theta_bytes, gamma_q8, window, rr_start)], dtype=DISPATCH_PARAMS_DTYPE)


def make_priorities(seed, n_desc, p_high=0.3, p_mid=0.3):
    """Seeded request priorities: 2 HIGH, 1 MID, 0 LOW."""
    rng = np.random.Generator(np.random.PCG64(seed))
    u = rng.random(n_desc)
    return np.where(u < p_high, 2, np.where(u < p_high + p_mid, 1, 0)).astype(np.uint8)


def make_monitor_params(err_threshold=8, recover_windows=2, cooldown_windows=1, degrade_q8=128):
    """Parameters of the rail health monitor (thresholds in events, times in measurement windows)."""
    return np.array([(err_threshold, recover_windows, cooldown_windows, degrade_q8)], dtype=MONITOR_PARAMS_DTYPE)


def failure_schedule(seed, n_windows, n_rails, p_fail=0.08, p_congestion=0.15, max_congestion=12):
    """Seeded fault injection: per window and rail, whether the rail reports a hard error and how many
    congestion errors it reports.  Returns (uint8[n_windows, n_rails], uint32[n_windows, n_rails])."""
    rng = np.random.Generator(np.random.PCG64(seed))
    fails = (rng.random((n_windows, n_rails)) < p_fail).astype(np.uint8)
    cong = (rng.integers(1, max_congestion + 1, size=(n_windows, n_rails)) *
            (rng.random((n_windows, n_rails)) < p_congestion)).astype(np.uint32)
    return fails, cong


def make_probe_params(hw_MBps, alpha_q8=256, delta_ns=5000, ewma_q8=64):
    """Per-rail calibration of the bandwidth probe: hardware bandwidth, alpha, delta, smoothing weight."""
    hw = np.asarray(hw_MBps, dtype=np.uint64)
    p = np.zeros(hw.shape[0], dtype=PROBE_DTYPE)
    p["hw_MBps"] = hw
    p["alpha_q8"] = alpha_q8
    p["delta_ns"] = delta_ns
    p["ewma_q8"] = ewma_q8
    return p


@dataclass
class Epoch:
    rails: np.ndarray          # RAIL_DTYPE[R] telemetry seen by the planner
    budget: np.ndarray         # uint64[R] bytes each rail drains this epoch


@dataclass
class Workload:
    name: str
    seed: int
    slice_bytes: int
    seg_bytes: List[int]       # [source pool bytes, destination pool bytes]
    src_ptr: np.ndarray        # uint32[D+1]
    src_ext: np.ndarray        # EXTENT_DTYPE[E_src]
    dst_ptr: np.ndarray        # uint32[D+1]
    dst_ext: np.ndarray        # EXTENT_DTYPE[E_dst]
    rails: np.ndarray          # RAIL_DTYPE[R]
    fill: str                  # "u8" uniform bytes | "bf16" normal values
    epochs: Optional[List[Epoch]] = None
    drain: Optional[Epoch] = None
    notes: dict = field(default_factory=dict)

    @property
    def n_desc(self) -> int:
        return int(self.src_ptr.shape[0] - 1)

    @property
    def payload(self) -> int:
        return int(self.src_ext["len"].astype(np.uint64).sum())

    @property
    def staging_bytes(self) -> int:
        # payload plus one 256-byte alignment gap per possible rail
        return self.payload + 64 * 256


def _extents(seg, off, length):
    off = np.asarray(off, dtype=np.uint64)
    e = np.zeros(off.shape[0], dtype=EXTENT_DTYPE)
    e["seg"] = seg
    e["off"] = off
    e["len"] = length
    return e


def _csr(counts):
    ptr = np.zeros(len(counts) + 1, dtype=np.uint64)
    np.cumsum(np.asarray(counts, dtype=np.uint64), out=ptr[1:])
    assert int(ptr[-1]) < (1 << 32)
    return ptr.astype(np.uint32)


# --------------------------------------------------------------------------
# Config 1: tiny, runs through every checker in seconds
# --------------------------------------------------------------------------
def tiny(seed: int = 1, n_desc: int = 64, block: int = 16 * KiB,
         slice_bytes: int = 64 * KiB) -> Workload:
    rng = np.random.Generator(np.random.PCG64(seed))
    n_blocks = rng.integers(4, 17, size=n_desc)
    total = int(n_blocks.sum())
    src_blocks = rng.permutation(total)
    dst_blocks = rng.permutation(total)
    ptr = _csr(n_blocks)
    src_ext = _extents(SRC_SEG, src_blocks.astype(np.uint64) * block, block)
    dst_ext = _extents(DST_SEG, dst_blocks.astype(np.uint64) * block, block)
    rails = make_rails([25000, 25000, 50000, 100000], lat_ns=5000,
                       queued=rng.integers(0, (1 << 20) + 1, size=4),
                       health=[HEALTHY, EXCLUDED, HEALTHY, HEALTHY])
    return Workload("tiny", seed, slice_bytes, [total * block, total * block],
                    ptr, src_ext, ptr.copy(), dst_ext, rails, "u8")


# --------------------------------------------------------------------------
# Config 2: paged KVCache migration (Llama-3-8B shaped)
# --------------------------------------------------------------------------
def _paged_kv(rng, n_req, pages_per_req, planes, page_bytes):
    """Descriptors (request, plane) over a pool laid out [plane][page][page_bytes].

    One random permutation of page ids is dealt to the requests and shared by
    all planes; source and destination pools use independent permutations.
    """
    P = int(pages_per_req.sum())
    starts = np.concatenate([[0], np.cumsum(pages_per_req)]).astype(np.int64)
    out = []
    for seg in (SRC_SEG, DST_SEG):
        perm = rng.permutation(P).astype(np.uint64)
        chunks = []
        for r in range(n_req):
            pages = perm[starts[r]:starts[r + 1]]
            plane_base = (np.arange(planes, dtype=np.uint64) * np.uint64(P))[:, None]
            chunks.append(((plane_base + pages[None, :]) * np.uint64(page_bytes)).ravel())
        out.append(_extents(seg, np.concatenate(chunks), page_bytes))
    counts = np.repeat(pages_per_req, planes)
    ptr = _csr(counts)
    pool = planes * P * page_bytes
    return ptr, out[0], out[1], pool, P


def kv_migration(seed: int = 2, n_req: int = 32, layers: int = 32,
                 ctx_lo: int = 2048, ctx_hi: int = 8192, page_tokens: int = 16,
                 kv_heads: int = 8, head_dim: int = 128,
                 slice_bytes: int = 256 * KiB, skew=(0, 0)) -> Workload:
    """skew = (source, destination) byte shift of every page, to exercise unaligned addresses."""
    rng = np.random.Generator(np.random.PCG64(seed))
    page_bytes = page_tokens * kv_heads * head_dim * 2          # bf16
    ctx = rng.integers(ctx_lo, ctx_hi + 1, size=n_req)
    pages = -(-ctx // page_tokens)
    ptr, src_ext, dst_ext, pool, P = _paged_kv(rng, n_req, pages, layers * 2, page_bytes)
    rails = make_rails([50000] * 8 + [400000])
    if skew != (0, 0):
        src_ext["off"] += np.uint64(skew[0])
        dst_ext["off"] += np.uint64(skew[1])
        pool += 16
    return Workload("kv_migration", seed, slice_bytes, [pool, pool], ptr, src_ext,
                    ptr.copy(), dst_ext, rails, "bf16",
                    notes={"pages": int(P), "page_bytes": page_bytes, "ctx": ctx.tolist()})


# --------------------------------------------------------------------------
# Config 3: RL parameter update (bulk contiguous tensors)
# --------------------------------------------------------------------------
def rl_params(seed: int = 3, layers: int = 32, hidden: int = 4096, ffn: int = 14336,
              vocab: int = 128256, kv_dim: int = 1024,
              slice_bytes: int = 1 * MiB) -> Workload:
    rng = np.random.Generator(np.random.PCG64(seed))
    shapes = [(vocab, hidden)]
    for _ in range(layers):
        shapes += [(hidden,), (hidden, hidden), (kv_dim, hidden), (kv_dim, hidden),
                   (hidden, hidden), (hidden,), (ffn, hidden), (ffn, hidden), (hidden, ffn)]
    shapes.append((hidden,))
    nbytes = np.array([int(np.prod(s)) * 2 for s in shapes], dtype=np.uint64)
    assert int(nbytes.max()) < (1 << 32)
    n = len(shapes)
    src_off = np.concatenate([[0], np.cumsum(nbytes)[:-1]]).astype(np.uint64)
    # destination pool holds the same tensors in an independently shuffled order
    order = rng.permutation(n)
    dst_off = np.zeros(n, dtype=np.uint64)
    dst_off[order] = np.concatenate([[0], np.cumsum(nbytes[order])[:-1]]).astype(np.uint64)
    ptr = _csr(np.ones(n, dtype=np.int64))
    src_ext = _extents(SRC_SEG, src_off, nbytes)
    dst_ext = _extents(DST_SEG, dst_off, nbytes)
    bw = np.rint(np.exp(rng.uniform(np.log(12500.0), np.log(100000.0), size=8))).astype(np.uint64)
    rails = make_rails(bw)
    pool = int(nbytes.sum())
    return Workload("rl_params", seed, slice_bytes, [pool, pool], ptr, src_ext,
                    ptr.copy(), dst_ext, rails, "bf16",
                    notes={"params": pool // 2, "tensors": n})


# --------------------------------------------------------------------------
# Config 4: congestion / failure re-planning over telemetry epochs
# --------------------------------------------------------------------------
def replanning(seed: int = 4, n_epochs: int = 16, fail_at=((5, 3), (11, 6)),
               queued_hi: int = 64 * MiB, epoch_share: int = 16, **kv_kwargs) -> Workload:
    """KV migration replayed over telemetry epochs.  Every epoch lasts t_us, the time the nominal
    rails need for 1/epoch_share of the payload; rail d drains bw_d * t_us bytes per epoch, so the
    transfer spans all epochs (both rail failures happen while slices are still pending) and a final
    drain pass with unlimited budget finishes what is left."""
    kv_kwargs.setdefault("seed", 2)
    w = kv_migration(**kv_kwargs)
    rng = np.random.Generator(np.random.PCG64(seed))
    nominal = w.rails["bw_MBps"].astype(np.float64)
    R = nominal.shape[0]
    t_us = -(-w.payload // int(epoch_share * int(w.rails["bw_MBps"].astype(np.uint64).sum())))
    epochs = []
    health = np.zeros(R, dtype=np.uint8)
    for e in range(n_epochs):
        for (at, rail) in fail_at:
            if e == at and rail < R:
                health[rail] = EXCLUDED          # a failed rail stays failed
        bw = np.maximum(1, np.rint(nominal * np.exp(0.5 * rng.standard_normal(R)))).astype(np.uint64)
        queued = rng.integers(0, queued_hi + 1, size=R).astype(np.uint64)
        rails = make_rails(bw, queued=queued, health=health.copy())
        epochs.append(Epoch(rails, bw * np.uint64(t_us)))
    drain = Epoch(epochs[-1].rails.copy(), np.full(R, np.iinfo(np.uint64).max, dtype=np.uint64))
    w.name, w.seed, w.epochs, w.drain = "replanning", seed, epochs, drain
    w.notes["t_us"] = int(t_us)
    return w


# --------------------------------------------------------------------------
# Config 5: many small flows (MLA-style latent KV, slices straddle pages)
# --------------------------------------------------------------------------
def many_small(seed: int = 5, n_req: int = 4096, layers: int = 1, pages_lo: int = 8,
               pages_hi: int = 64, latent_dim: int = 576, page_tokens: int = 16,
               slice_bytes: int = 16 * KiB) -> Workload:
    rng = np.random.Generator(np.random.PCG64(seed))
    page_bytes = latent_dim * page_tokens * 2                   # 18 KiB
    pages = rng.integers(pages_lo, pages_hi + 1, size=n_req)
    ptr, src_ext, dst_ext, pool, P = _paged_kv(rng, n_req, pages, layers, page_bytes)
    rails = make_rails([25000, 50000] * 8)
    return Workload("many_small" + ("" if layers == 1 else f"_x{layers}"), seed, slice_bytes,
                    [pool, pool], ptr, src_ext, ptr.copy(), dst_ext, rails, "bf16",
                    notes={"pages": int(P), "page_bytes": page_bytes})


# --------------------------------------------------------------------------
# Slice-size sweep: fixed payload, contiguous or paged layout (shapes of the
# paper's block-size sweeps, Section 5.2)
# --------------------------------------------------------------------------
def sweep(slice_bytes: int, paged: bool, payload: int = 4 << 30, n_desc: int = 64, page_bytes: int = 32 * KiB,
          seed: int = 6) -> Workload:
    """n_desc equal transfers; contiguous = one extent each, paged = shuffled pages on both sides."""
    rng = np.random.Generator(np.random.PCG64(seed))
    per = payload // n_desc
    rails = make_rails([50000] * 8 + [400000])
    if not paged:
        off = (np.arange(n_desc, dtype=np.uint64) * np.uint64(per))
        ptr = np.arange(n_desc + 1, dtype=np.uint32)
        order = rng.permutation(n_desc)
        doff = np.zeros(n_desc, dtype=np.uint64)
        doff[order] = off
        return Workload("sweep_contiguous", seed, slice_bytes, [payload, payload], ptr, _extents(SRC_SEG, off, per),
                        ptr.copy(), _extents(DST_SEG, doff, per), rails, "u8")
    pages = np.full(n_desc, per // page_bytes, dtype=np.int64)
    ptr, se, de, pool, _ = _paged_kv(rng, n_desc, pages, 1, page_bytes)
    return Workload("sweep_paged", seed, slice_bytes, [pool, pool], ptr, se, ptr.copy(), de, rails, "u8")


# --------------------------------------------------------------------------
# Arbitrary-geometry descriptors for property tests (odd lengths, 1-byte
# extents, independent source and destination block structure)
# --------------------------------------------------------------------------
def ragged(seed: int, n_desc: int = 24, max_len: int = 200_000, max_ext: int = 4096,
           slice_bytes: int = 4096 + 7, n_rails: int = 5, align: int = 1) -> Workload:
    rng = np.random.Generator(np.random.PCG64(seed))
    lens = rng.integers(1, max_len + 1, size=n_desc) // align * align
    lens = np.maximum(lens, align)

    def cut(total):
        parts = []
        left = int(total)
        while left > 0:
            p = int(rng.integers(1, max_ext + 1)) // align * align
            p = max(align, min(p, left))
            parts.append(p)
            left -= p
        return parts

    def layout(seg):
        counts, sizes = [], []
        for L in lens:
            parts = cut(L)
            counts.append(len(parts))
            sizes += parts
        sizes = np.array(sizes, dtype=np.uint64)
        # scatter extents over the pool in random order with random gaps
        order = rng.permutation(sizes.shape[0])
        gaps = rng.integers(0, 64, size=sizes.shape[0]).astype(np.uint64) // np.uint64(align) * np.uint64(align)
        pos = np.zeros(sizes.shape[0], dtype=np.uint64)
        run = np.cumsum(sizes[order] + gaps[order])
        pos[order] = run - sizes[order]
        pool = int(run[-1]) + 64
        return _csr(counts), _extents(seg, pos, sizes), pool

    sp, se, spool = layout(SRC_SEG)
    dp, de, dpool = layout(DST_SEG)
    bw = rng.integers(1000, 400000, size=n_rails)
    u = rng.random(n_rails)
    health = np.where(u < 0.25, EXCLUDED, np.where(u < 0.45, DEGRADED, HEALTHY)).astype(np.uint8)
    if (health == EXCLUDED).all():
        health[int(rng.integers(0, n_rails))] = HEALTHY
    rails = make_rails(bw, lat_ns=rng.integers(0, 20000, size=n_rails),
                       queued=rng.integers(0, 1 << 22, size=n_rails), health=health,
                       beta1_q8=rng.integers(128, 1024, size=n_rails),
                       penalty_q8=rng.integers(26, 1280, size=n_rails))
    return Workload(f"ragged{seed}", seed, slice_bytes, [spool, dpool], sp, se, dp, de, rails, "u8")


# --------------------------------------------------------------------------
# Pool contents
# --------------------------------------------------------------------------
def fill_numpy(w: Workload, which: int = SRC_SEG) -> np.ndarray:
    """Host byte pool for one segment (small workloads / CPU tests)."""
    rng = np.random.Generator(np.random.PCG64([w.seed, 1000 + which]))
    n = w.seg_bytes[which]
    if w.fill == "u8" or n % 2:
        return rng.integers(0, 256, size=n, dtype=np.uint8)
    vals = rng.standard_normal(n // 2, dtype=np.float32)
    return (vals.view(np.uint32) >> 16).astype(np.uint16).view(np.uint8)   # bf16 bit patterns


def fill_torch(w: Workload, which: int, device, chunk_bytes: int = 1 << 30, out=None):
    """Device byte pool for one segment, filled in place by a seeded torch generator (`out`: a uint8
    tensor of the segment's size to fill instead of a new allocation)."""
    import torch
    n = w.seg_bytes[which]
    g = torch.Generator(device=device)
    g.manual_seed(w.seed * 7919 + which)
    if out is not None and (out.dtype != torch.uint8 or out.numel() != n):
        raise ValueError("out must be a uint8 tensor of the segment's size")
    buf = torch.empty(n, dtype=torch.uint8, device=device) if out is None else out
    for lo in range(0, n, chunk_bytes):
        hi = min(n, lo + chunk_bytes)
        if w.fill == "u8" or (hi - lo) % 2:
            buf[lo:hi] = torch.randint(0, 256, (hi - lo,), dtype=torch.uint8, device=device, generator=g)
        else:
            v = torch.randn((hi - lo) // 2, dtype=torch.bfloat16, device=device, generator=g)
            buf[lo:hi] = v.view(torch.uint8)
    return buf


CONFIGS = {
    "tiny": tiny,
    "kv_migration": kv_migration,
    "rl_params": rl_params,
    "replanning": replanning,
    "many_small": many_small,
}


def small_variant(name: str) -> Workload:
    """Reduced-size instance of a named config that still spans several tiles and tails."""
    if name == "tiny":
        return tiny()
    if name == "kv_migration":
        return kv_migration(n_req=4, layers=2, ctx_lo=200, ctx_hi=900)
    if name == "rl_params":
        return rl_params(layers=2, hidden=512, ffn=1792, vocab=4001, kv_dim=128, slice_bytes=256 * KiB)
    if name == "replanning":
        return replanning(n_req=4, layers=2, ctx_lo=200, ctx_hi=900, queued_hi=256 * KiB)
    if name == "many_small":
        return many_small(n_req=96, layers=2)
    raise KeyError(name)
