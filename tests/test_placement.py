"""Pool placement helper: the region map from pairwise probe times and the carving (CPU), the carved pools on
the device (GPU)."""
import numpy as np
import pytest

from paper_2604_00368_amd import placement as P
from paper_2604_00368_amd import workloads as W

GiB = 1 << 30


def fake_probe(regions, same=0.729, cross=0.683, jitter=0.004, seed=0):
    rng = np.random.Generator(np.random.PCG64(seed))
    def pair_ms(i, j):
        return (same if regions[i] == regions[j] else cross) + float(rng.uniform(-jitter, jitter))
    return pair_ms


def test_region_labels_from_pair_times():
    # a reservation made of five pieces from three regions, as found on the device: 1, 2, 3, 1, 2
    regions = [0] * 8 + [1] * 8 + [2] * 4 + [0] * 4 + [1] * 2
    labels, probes, fastest, level = P.label_chunks(len(regions), fake_probe(regions))
    assert 0.679 <= fastest <= 0.687 and 0.69 < level < 0.72
    assert labels == regions                      # labels are numbered in order of first appearance
    assert probes == 25 + 13 + 3
    # address-ordered thirds
    regions = [0] * 12 + [1] * 12 + [2] * 8
    labels, _, _, _ = P.label_chunks(len(regions), fake_probe(regions, seed=3))
    assert labels == regions
    # a narrower gap than the fixed ratio would separate (the level adapts to what the first reference sees)
    regions = [0] * 12 + [1] * 12 + [2] * 8
    labels, _, _, level = P.label_chunks(len(regions), fake_probe(regions, same=0.700, cross=0.676, jitter=0.004, seed=9))
    assert labels == regions and 0.68 < level < 0.70
    # one region only: no pair is slower than the fastest by the ratio, so no two chunks are reported as sharing a
    # region, no run is long enough for a pool, and the caller falls back to ordinary allocations
    labels, _, _, level = P.label_chunks(6, fake_probe([0] * 6))
    assert level is None
    assert len(set(labels)) == 6
    assert P.choose_windows(labels, 8 * GiB, 2 * GiB, (20 * GiB, 20 * GiB, 20 * GiB)) is None


def test_windows_keep_partners_in_different_regions():
    chunk, probe = 8 * GiB, 2 * GiB
    sizes = (21_179_138_048, 21_179_140_352, 21_179_138_048)
    def region_of(labels, off, n):
        ks = set(labels[k] for k in range(off // chunk, (off + n - 1) // chunk + 1))
        assert len(ks) == 1, "pool crosses a region boundary"
        return ks.pop()
    for labels in ([0] * 8 + [1] * 8 + [2] * 4 + [0] * 4 + [1] * 2, [0] * 12 + [1] * 12 + [2] * 9, [0] * 12 + [1] * 20):
        offs = P.choose_windows(labels, chunk, probe, sizes)
        assert offs is not None
        r_src, r_arena, r_dst = (region_of(labels, o, n) for o, n in zip(offs, sizes))
        assert r_src != r_arena and r_dst != r_arena
        if len(set(labels)) >= 3:
            assert r_src != r_dst
        spans = sorted((o, o + n) for o, n in zip(offs, sizes))
        assert spans[0][1] <= spans[1][0] and spans[1][1] <= spans[2][0]          # no overlap
        for o, n in zip(offs, sizes):                                            # ends inside the probed part of a chunk
            assert (o + n - 1) % chunk < probe or labels[(o + n - 1) // chunk] == labels[min(len(labels) - 1, (o + n - 1) // chunk + 1)]
        # the carved pools verify against the same region map, and a pool pushed across a boundary does not
        chunk_region = lambda off: labels[off // chunk]
        window_ms = lambda a, b: 0.729 if chunk_region(a) == chunk_region(b) else 0.683
        assert P.verify_windows(offs, sizes, probe, window_ms, 0.706)
        bad = (offs[1], offs[1], offs[2])
        assert not P.verify_windows(bad, sizes, probe, window_ms, 0.706)
    # runs too short for the pools
    assert P.choose_windows([0, 0, 1, 1, 2, 2], chunk, probe, sizes) is None
    # two regions, the second one must host nothing but the arena
    offs = P.choose_windows([0] * 8 + [1] * 4, chunk, probe, sizes)
    assert offs is not None and offs[1] == 8 * chunk and offs[0] != offs[2]


@pytest.mark.gpu
def test_carved_pools_run_the_engine(oracle):
    torch = pytest.importorskip("torch")
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import gpu_harness as H
    w = W.small_variant("kv_migration")
    dev = torch.device("cuda:0")
    # a small reservation exercises the probing and the carving; whether it spans regions is up to the device
    need = max(w.seg_bytes[0], w.staging_bytes, w.seg_bytes[1])
    chunk = 64 << 20
    src, arena, dst, lay = P.place_pools(dev, w.seg_bytes[0], w.staging_bytes, w.seg_bytes[1], chunk_bytes=chunk,
                                         probe_bytes=16 << 20, reserve_bytes=12 * chunk + 3 * need)
    assert lay.mode in ("regions", "plain")
    assert (src.numel(), arena.numel(), dst.numel()) == (w.seg_bytes[0], w.staging_bytes, w.seg_bytes[1])
    if lay.mode == "regions":
        base = src.data_ptr() - lay.offsets[0]
        assert (arena.data_ptr() - base, dst.data_ptr() - base) == lay.offsets[1:]
    with H.Engine(w, pools=(src, arena, dst)) as eng:
        eng.declare()
        st, info = eng.plan()
        assert st == 0
        eng.execute()
        s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
        b = oracle.bind(s.len, w.rails)
        H.assert_plan_equal(eng.table(), s, b, info)
        src_h = eng.src.cpu().numpy()
        dst_want = np.zeros(w.seg_bytes[1], dtype=np.uint8)
        stg_want = np.zeros(w.staging_bytes, dtype=np.uint8)
        oracle.execute(w, s, b, [src_h, dst_want], stg_want)
        assert np.array_equal(eng.dst.cpu().numpy(), dst_want)
        assert np.array_equal(eng.arena.cpu().numpy(), stg_want)
    s2, a2, d2, lay2 = P.place_pools(dev, 1 << 20, 1 << 20, 1 << 20, mode="plain")
    assert lay2.mode == "plain" and s2.numel() == a2.numel() == d2.numel() == 1 << 20


@pytest.mark.gpu
def test_probe_copy_moves_every_page_once():
    torch = pytest.importorskip("torch")
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2604_00368_amd import binding as T
    dev = torch.device("cuda:0")
    page, n_pages = 32768, 256
    g = torch.Generator(device=dev)
    g.manual_seed(12)
    a = torch.randint(0, 256, (page * n_pages,), dtype=torch.uint8, device=dev, generator=g)
    b = torch.zeros_like(a)
    ms = T.tent_probe_copy(a.data_ptr(), b.data_ptr(), a.numel(), page, 2, torch.cuda.current_stream(dev))
    assert ms > 0
    torch.cuda.synchronize(dev)
    # block w (4 KiB) reads block (w mod 8) of a permuted page and lands in one of eight write frontiers
    m1, bits = 0x9E3779B97F4A7C15, n_pages.bit_length() - 1
    m2 = (m1 >> 7) | 1
    bpp = page // 4096
    n_blocks = n_pages * bpp
    src_block, dst_block = [], []
    for w in range(n_blocks):
        v = ((w // bpp) * m1) % n_pages               # multiply by an odd constant,
        v ^= v >> (bits // 2)                         # xor with the upper half,
        v = (v * m2) % n_pages                        # multiply by another odd constant
        src_block.append(v * bpp + w % bpp)
        dst_block.append((w % 8) * (n_blocks // 8) + w // 8)
    assert sorted(src_block) == list(range(n_blocks)) and sorted(dst_block) == list(range(n_blocks))
    av, bv = a.view(n_blocks, 4096), b.view(n_blocks, 4096)
    want = torch.empty_like(bv)
    want[torch.tensor(dst_block, device=dev)] = av[torch.tensor(src_block, device=dev)]
    assert torch.equal(bv, want)
    # argument checks
    for bad in [dict(nbytes=page * 3), dict(page_bytes=5000), dict(page_bytes=2048), dict(repeats=0)]:
        kw = dict(nbytes=a.numel(), page_bytes=page, repeats=1)
        kw.update(bad)
        with pytest.raises(T.TentError):
            T.tent_probe_copy(a.data_ptr(), b.data_ptr(), kw["nbytes"], kw["page_bytes"], kw["repeats"])
