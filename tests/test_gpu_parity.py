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
