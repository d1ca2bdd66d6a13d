"""Where the byte pools of a transfer engine sit in device memory.

Measured on MI355X (288 GiB of HBM3E): device memory behaves as three regions of 96 GiB, and a
copy kernel whose read side and write side lie in the same region runs 4-9 % slower than one that
reads from one region and writes to another (20 GiB gathered from 32 KiB pages in random order:
7.2 ms when the source pool and the staging arena share the first region, 6.5 ms when they do
not; contiguous copies differ by 2 %).  Which region an address belongs to is a property of the
physical address.  Allocations made one after the other on an idle device come out of the same
region, so three pools of 20 GiB allocated in the ordinary way all share one.  Nothing in the
copy kernels can make up for that; the remedy is a layout decision of the caller, who owns the
pools: gather should read one region and write another, and so should scatter.

The runtime does not tell physical addresses, and a large allocation is not laid out in address
order (a 212 GiB allocation was found to be made of five pieces from the three regions in the
order 1, 2, 3, 1, 2).  So the layout is found by measurement: reserve most of the device in one
allocation, cut it into chunks, and time a small probe copy (32 KiB pages of one chunk in a
scattered order into another chunk: tent_probe_copy) for pairs of chunks -- same-region pairs are 6-7 %
slower than the others, far outside the noise of 0.5 % -- which labels every chunk with its
region after about sixty such probes (well under a second).  The pools are then carved from runs
of chunks with one label: source pool and staging arena in different regions, staging arena and
destination pool in different regions.

The engine itself takes the pools as plain device pointers and does not care where they came
from; the reservation stays alive as long as any pool carved from it does.
"""
from __future__ import annotations

from dataclasses import dataclass, field

GiB = 1 << 30
CHUNK = 8 * GiB          # granularity of the region map
ALIGN = 2 << 20          # verification probes start on 2 MiB boundaries
PROBE = 2 * GiB          # bytes a probe moves (from the start of one chunk to the start of another)
SAME_REGION_RATIO = 1.032   # a pair this much slower than the fastest pair seen shares a region


@dataclass
class Layout:
    mode: str                       # "regions" (pools carved by measured region) or "plain" (ordinary allocations)
    note: str
    reserved_bytes: int = 0
    chunk_bytes: int = 0
    labels: list = field(default_factory=list)      # region label of every chunk of the reservation
    offsets: tuple = ()                             # byte offsets of (src, arena, dst) inside the reservation
    probes: int = 0
    verified: bool = False          # probes between the carved pools themselves (first and last bytes) say "different regions"


def split_level(times, min_spread: float = 1.02):
    """Where a set of probe times falls into a fast and a slow group: the middle of the widest gap between
    neighbours of the sorted times, or None when the slowest is within `min_spread` of the fastest (one group)."""
    ts = sorted(times)
    if len(ts) < 2 or ts[-1] < min_spread * ts[0]:
        return None
    k = max(range(len(ts) - 1), key=lambda n: ts[n + 1] - ts[n])
    return 0.5 * (ts[k] + ts[k + 1])


def label_chunks(n_chunks: int, pair_ms, ratio: float = SAME_REGION_RATIO):
    """Region label (0, 1, ...) for each of n_chunks chunks.  pair_ms(i, j) times one probe that reads
    chunk i and writes chunk j.  Same-region pairs are the slow group: the level between the groups is
    taken from the first reference chunk whose probes show two groups and kept for the rest (later
    references may see one group only); until then a pair counts as same-region when it takes `ratio`
    times the fastest pair seen.  Returns (labels, number of probes, fastest pair time, the level or None)."""
    labels = [-1] * n_chunks
    fastest = None
    level = None
    probes = 0
    next_label = 0
    for i in range(n_chunks):
        if labels[i] != -1:
            continue
        labels[i] = next_label
        todo = [j for j in range(i + 1, n_chunks) if labels[j] == -1]
        times = {}
        for j in todo:
            times[j] = pair_ms(i, j)
            probes += 1
            fastest = times[j] if fastest is None else min(fastest, times[j])
        if level is None:
            level = split_level(list(times.values()))
        cut = level if level is not None else ratio * fastest
        for j in todo:
            if times[j] >= cut:
                labels[j] = next_label
        next_label += 1
    return labels, probes, fastest, level


def uniform_runs(labels):
    """Maximal runs of equal labels as (first chunk, number of chunks, label)."""
    runs = []
    for k, lab in enumerate(labels):
        if runs and runs[-1][2] == lab and runs[-1][0] + runs[-1][1] == k:
            runs[-1] = (runs[-1][0], runs[-1][1] + 1, lab)
        else:
            runs.append((k, 1, lab))
    return runs


def choose_windows(labels, chunk_bytes: int, probe_bytes: int, sizes):
    """Byte offsets for pools of `sizes` = (src, arena, dst) bytes, each inside a run of chunks with one
    label, arena in another region than src and dst in another region than arena (and, if possible,
    than src).  Only the first `probe_bytes` of a chunk are known to carry its label, so a pool must
    end within the probed part of its run's last chunk.  Returns None when no such choice exists."""
    runs = uniform_runs(labels)

    def fits(run, nbytes, taken):
        first, count, _ = run
        lo = first * chunk_bytes
        for t_lo, t_hi in taken:                      # a run may host two pools, one after the other
            if t_lo < (first + count) * chunk_bytes and t_hi > lo:
                lo = max(lo, (t_hi + chunk_bytes - 1) // chunk_bytes * chunk_bytes)
        hi_ok = (first + count - 1) * chunk_bytes + probe_bytes
        return lo if lo + nbytes <= hi_ok else None

    best = None
    for ra in runs:                                   # arena first: it is the partner of both others
        o_arena = fits(ra, sizes[1], [])
        if o_arena is None:
            continue
        taken_a = [(o_arena, o_arena + sizes[1])]
        for rs in runs:
            if rs[2] == ra[2]:
                continue
            o_src = fits(rs, sizes[0], taken_a)
            if o_src is None:
                continue
            taken_s = taken_a + [(o_src, o_src + sizes[0])]
            for rd in runs:
                if rd[2] == ra[2]:
                    continue
                o_dst = fits(rd, sizes[2], taken_s)
                if o_dst is None:
                    continue
                score = 1 if rd[2] != rs[2] else 0    # three different regions preferred
                if best is None or score > best[0]:
                    best = (score, (o_src, o_arena, o_dst))
                if score == 1:
                    return best[1]
    return None if best is None else best[1]


def _probe_factory(block, chunk_bytes, probe_bytes, repeats):
    """(pair_ms, window_ms): pair_ms(i, j) for label_chunks is the library's timed probe copy (32 KiB pages of
    the start of chunk i in a scattered order, written front to back to the start of chunk j); window_ms(a, b)
    is the same probe between two byte offsets of the reservation.  Every probe is the shortest of `repeats`
    runs: what disturbs a timing (a profiler, another process) only ever makes it longer."""
    import torch
    from . import binding as T
    if probe_bytes > chunk_bytes or probe_bytes & (probe_bytes - 1):
        raise ValueError("the probe must be a power of two and fit a chunk")
    stream = torch.cuda.current_stream(block.device)
    base = block.data_ptr()

    def window_ms(read_off, write_off):
        return T.tent_probe_copy(base + read_off, base + write_off, probe_bytes, 32768, repeats, stream)

    def pair_ms(i, j):
        return window_ms(i * chunk_bytes, j * chunk_bytes)
    return pair_ms, window_ms


def verify_windows(offsets, sizes, probe_bytes, window_ms, cut) -> bool:
    """Probes between the pools as carved -- source to arena and arena to destination, at the pools' first
    bytes and at their last -- must all be faster than `cut`, i.e. as fast as pairs from different regions."""
    (o_src, o_arena, o_dst), (n_src, n_arena, n_dst) = offsets, sizes
    def last(o, n):
        return o + (max(n - probe_bytes, 0) // ALIGN) * ALIGN
    pairs = [(o_src, o_arena), (last(o_src, n_src), last(o_arena, n_arena)),
             (o_arena, o_dst), (last(o_arena, n_arena), last(o_dst, n_dst))]
    return all(window_ms(a, b) < cut for a, b in pairs)


def place_pools(device, src_bytes: int, arena_bytes: int, dst_bytes: int, mode: str = "regions",
                keep_free: int = 24 * GiB, chunk_bytes: int = CHUNK, probe_bytes: int = PROBE, reserve_bytes=None):
    """Allocate the three pools on `device` (uint8 tensors).  Returns (src, arena, dst, layout).

    mode "regions": reserve the device memory but `keep_free` bytes (or `reserve_bytes`), measure the
    region of every chunk and carve the pools as the module's header describes; falls back to
    ordinary allocations (and says so in the layout's note) when the reservation fails, when the
    measurement finds one region only, or when no placement exists.
    mode "plain": three ordinary allocations."""
    import torch
    if mode not in ("regions", "plain"):
        raise ValueError(f"unknown placement mode {mode!r}")
    lay = Layout("plain", "ordinary allocations")
    if mode == "regions":
        sizes = (src_bytes, arena_bytes, dst_bytes)
        torch.cuda.empty_cache()                          # blocks the caching allocator still holds count as used
        free, _total = torch.cuda.mem_get_info(device)
        first = (free - keep_free if reserve_bytes is None else reserve_bytes) // chunk_bytes * chunk_bytes
        # A reservation of nearly the whole device can fail (or map one region only) in a process that has
        # allocated and freed a lot before; smaller reservations are tried before giving up, and every
        # attempt leaves its reason in the layout's note.
        attempts, notes = [], []
        for num, den in ((1, 1), (3, 4), (1, 2)):
            want = first * num // den // chunk_bytes * chunk_bytes
            if want not in attempts:
                attempts.append(want)
        for want in attempts:
            if want < sum(sizes) or want < 2 * chunk_bytes:
                notes.append(f"{want >> 30} GiB: too small for the pools")
                continue
            try:
                block = torch.empty(want, dtype=torch.uint8, device=device)
            except RuntimeError as exc:                   # out of memory
                notes.append(f"{want >> 30} GiB: reservation failed ({type(exc).__name__})")
                torch.cuda.empty_cache()
                continue
            n_chunks = want // chunk_bytes
            total_probes = 0
            for repeats in (3, 8):                        # a second, more patient pass if the first map does not hold up
                pair_ms, window_ms = _probe_factory(block, chunk_bytes, probe_bytes, repeats)
                labels, probes, fastest, level = label_chunks(n_chunks, pair_ms)
                total_probes += probes
                offs = choose_windows(labels, chunk_bytes, probe_bytes, sizes)
                verified = False
                if offs is not None and min(sizes) >= probe_bytes:
                    verified = verify_windows(offs, sizes, probe_bytes, window_ms,
                                              level if level is not None else SAME_REGION_RATIO * fastest)
                    total_probes += 4
                if offs is not None and (verified or min(sizes) < probe_bytes):
                    break
            if offs is None:
                notes.append(f"{want >> 30} GiB: " + ("one region found (map " + "".join(str(x) for x in labels) + ")"
                                                      if len(set(labels)) < 2 else
                                                      "no placement with the partners in different regions (map "
                                                      + "".join(str(x) for x in labels) + ")"))
                del block
                torch.cuda.empty_cache()
                continue
            lay = Layout("regions", "pools carved from one reservation by measured region: source and staging arena "
                         "in different regions, staging arena and destination in different regions"
                         + ("" if not notes else "; earlier attempts: " + "; ".join(notes)),
                         want, chunk_bytes, labels, offs, total_probes, verified)
            o_src, o_arena, o_dst = offs
            return (block[o_src:o_src + src_bytes], block[o_arena:o_arena + arena_bytes],
                    block[o_dst:o_dst + dst_bytes], lay)
        lay.note = "ordinary allocations, no region layout: " + "; ".join(notes)
    src = torch.empty(src_bytes, dtype=torch.uint8, device=device)
    dst = torch.empty(dst_bytes, dtype=torch.uint8, device=device)
    arena = torch.empty(arena_bytes, dtype=torch.uint8, device=device)
    return src, arena, dst, lay


def main(argv=None):
    """python -m paper_2604_00368_amd.placement [--step GiB]: reserve the device memory, print the probe time
    of every pair of windows `step` GiB apart (rows read, columns write) and the region map."""
    import argparse
    import torch
    ap = argparse.ArgumentParser(description=main.__doc__)
    ap.add_argument("--step", type=int, default=16, help="distance between probed windows in GiB (a multiple of 8)")
    ap.add_argument("--keep-free", type=int, default=24, help="GiB left outside the reservation")
    args = ap.parse_args(argv)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    free, total = torch.cuda.mem_get_info(dev)
    want = (free - args.keep_free * GiB) // CHUNK * CHUNK
    block = torch.empty(want, dtype=torch.uint8, device=dev)
    print(f"device memory {total / GiB:.1f} GiB, reservation {want / GiB:.0f} GiB; probe: {PROBE >> 30} GiB, 32 KiB pages "
          "in scattered order -> sequential writes; ms, shortest of 3")
    pair_ms, _ = _probe_factory(block, CHUNK, PROBE, 3)
    per = max(1, args.step * GiB // CHUNK)
    idx = list(range(0, want // CHUNK, per))
    print("read\\write " + " ".join(f"{k * (CHUNK >> 30):6d}" for k in idx))
    for i in idx:
        print(f"{i * (CHUNK >> 30):9d}  " + " ".join("    --" if i == j else f"{pair_ms(i, j):6.3f}" for j in idx), flush=True)
    labels, probes, fastest, level = label_chunks(want // CHUNK, pair_ms)
    print(f"region of each {CHUNK >> 30} GiB chunk: {''.join(str(x) for x in labels)}  ({probes} probes, fastest pair {fastest:.3f} ms, "
          f"level between the groups {level if level is None else round(level, 3)} ms)")


if __name__ == "__main__":
    main()
