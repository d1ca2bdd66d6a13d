"""GPU parity: the HIP engine (through its C ABI) against the CPU oracle, bit for bit."""
import numpy as np
import pytest

from paper_2604_00368_amd import workloads as W

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def H():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import gpu_harness
    return gpu_harness


def run_and_compare(H, oracle, w, flags=0):
    src = W.fill_numpy(w, 0)
    dst0 = W.fill_numpy(w, 1)
    s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
    b = oracle.bind(s.len, w.rails)
    dst_want = dst0.copy()
    staging_want = np.zeros(w.staging_bytes, dtype=np.uint8)
    oracle.execute(w, s, b, [src, dst_want], staging_want)
    with H.Engine(w, src, dst0, flags=flags) as eng:
        eng.declare()
        st, info = eng.plan()
        assert st == 0
        H.assert_plan_equal(eng.table(), s, b, info)
        eng.execute()
        assert np.array_equal(eng.dst.cpu().numpy(), dst_want)
        assert np.array_equal(eng.arena.cpu().numpy(), staging_want)
        assert np.array_equal(eng.src.cpu().numpy(), src)
        tab = eng.table()
        assert (tab["state"] == 2).all()


@pytest.mark.parametrize("name", ["tiny", "kv_migration", "rl_params", "many_small"])
def test_small_configs_bit_exact(H, oracle, name):
    print("case", name, flush=True)
    run_and_compare(H, oracle, W.small_variant(name))


@pytest.mark.parametrize("seed", range(8))
def test_ragged_bit_exact(H, oracle, seed):
    print("ragged seed", seed, flush=True)
    S = [1, 17, 4096, 5000, 65536, 4099, 333, 16][seed]
    align = [1, 1, 1, 1, 1, 4, 1, 16][seed]
    run_and_compare(H, oracle, W.ragged(seed, slice_bytes=S, n_desc=12, max_len=40_000, max_ext=900, align=align))


@pytest.mark.parametrize("S", [1024, 3072, 4096, 6144, 8192 + 2048, 65536 + 1024])
def test_tile_sizes_and_partial_blocks(H, oracle, S):
    # slice sizes that give 1 KiB / 2 KiB / 4 KiB tiles, partial last blocks and extent boundaries inside blocks
    print("tile case S", S, flush=True)
    w = W.ragged(7, slice_bytes=S, n_desc=10, max_len=300_000, max_ext=20_000, align=1024)
    run_and_compare(H, oracle, w)
    w = W.many_small(n_req=24, layers=2, slice_bytes=S)
    run_and_compare(H, oracle, w)


def test_serial_binding_flag_matches_oracle(H, oracle):
    from paper_2604_00368_amd import binding as T
    print("serial binding", flush=True)
    for name in ["tiny", "many_small", "kv_migration"]:
        run_and_compare(H, oracle, W.small_variant(name), flags=T.TENT_FLAG_SERIAL_BINDING)


def _runs_workload(rng, kind):
    """Transfers that produce runs of equal-length slices of arbitrary length and count, with tails."""
    S = int(rng.integers(1, 1 << int(rng.integers(4, 17))))
    lens = []
    for _ in range(int(rng.integers(1, 12))):
        m = int(rng.integers(1, 200 if kind != 5 else 1500))
        if rng.random() < 0.6:
            lens.append(m * S + (int(rng.integers(1, S)) if (S > 1 and rng.random() < 0.7) else 0))
        else:
            lens += [int(rng.integers(1, S + 1))] * m          # m short transfers: a run of equal tails
    lens = np.array(lens, dtype=np.uint64)
    off = np.concatenate([[0], np.cumsum(lens)[:-1]]).astype(np.uint64)
    ptr = np.arange(len(lens) + 1, dtype=np.uint32)
    total = int(lens.sum())
    R = int(rng.integers(1, 20))
    bw = rng.integers(1000, 400000, size=R)
    lat = rng.integers(0, 20000, size=R)
    queued = rng.integers(0, 1 << 24, size=R)
    b1 = rng.integers(128, 1024, size=R)
    pen = rng.integers(26, 1280, size=R)
    if kind == 1:                                              # identical rails: every cost ties
        bw[:], lat[:], queued[:], b1[:], pen[:] = 50000, 5000, 0, 256, 256
    if kind == 2:                                              # cost grows by less than 1 ps per slot
        bw, lat = rng.integers(3_000_000_000, 4_000_000_000, size=R), np.zeros(R, dtype=np.int64)
    if kind == 3:                                              # latencies spread over the whole range
        lat = rng.integers(0, 2**32 - 1, size=R)
    if kind == 4:                                              # long queues
        queued = rng.integers(0, 1 << 31, size=R)                # (max A + payload) * max c1 stays below 2^63
    health = np.where(rng.random(R) < 0.2, 2, 0).astype(np.uint8)
    if (health == 2).all():
        health[0] = 0
    rails = W.make_rails(bw, lat_ns=lat, queued=queued, health=health, beta1_q8=b1, penalty_q8=pen)
    return W.Workload("runs", 0, S, [total, total], ptr, W._extents(0, off, lens), ptr.copy(),
                      W._extents(1, off, lens), rails, "u8")


@pytest.mark.parametrize("kind", range(6))
def test_run_parallel_binding_matches_oracle(H, oracle, kind):
    # plan-only: degenerate telemetry (ties, sub-picosecond steps, huge latencies and queues)
    rng = np.random.Generator(np.random.PCG64(1000 + kind))
    for trial in range(25):
        w = _runs_workload(rng, kind)
        print("runs kind", kind, "trial", trial, "S", w.slice_bytes, "D", w.n_desc, "R", w.rails.shape[0], flush=True)
        s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
        b = oracle.bind(s.len, w.rails)
        with H.Engine(w, np.zeros(w.seg_bytes[0], np.uint8), np.zeros(w.seg_bytes[1], np.uint8)) as eng:
            eng.declare()
            st, info = eng.plan()
            assert st == 0
            H.assert_plan_equal(eng.table(), s, b, info)
