"""The plan and execute entry points allocate nothing and copy nothing from the host, so a caller can record
them into a HIP graph.  Every replay must give the oracle's result."""
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


@pytest.mark.parametrize("name", ["tiny", "many_small"])
def test_reset_plan_execute_replayed_from_a_graph(H, oracle, name):
    from paper_2604_00368_amd import binding as T
    w = W.small_variant(name)
    src, dst0 = W.fill_numpy(w, 0), W.fill_numpy(w, 1)
    s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
    b = oracle.bind(s.len, w.rails)
    dst_want, staging_want = dst0.copy(), np.zeros(w.staging_bytes, dtype=np.uint8)
    oracle.execute(w, s, b, [src, dst_want], staging_want)
    with H.Engine(w, src, dst0) as eng:
        eng.declare()
        st, _ = eng.plan()                                     # eager run first: builds nothing lazily afterwards
        assert st == 0
        eng.execute()
        assert np.array_equal(eng.dst.cpu().numpy(), dst_want)
        dst_reset = torch.from_numpy(dst0).to(eng.dev)
        side = torch.cuda.Stream(eng.dev)
        side.wait_stream(torch.cuda.current_stream(eng.dev))
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                cap = torch.cuda.current_stream(eng.dev)
                T.tent_reset(eng.ctx, eng.batch, cap)
                st, _ = T.tent_plan(eng.ctx, eng.batch, w.rails, want_info=False, stream=cap)
                assert st == 0
                T.tent_execute(eng.ctx, eng.batch, cap)
        torch.cuda.synchronize(eng.dev)
        for replay in range(4):
            # the program's own eager work between replays: put the pools back, scribble over the arena
            eng.dst.copy_(dst_reset)
            eng.arena.fill_(replay + 1)
            torch.cuda.synchronize(eng.dev)
            graph.replay()
            torch.cuda.synchronize(eng.dev)
            assert np.array_equal(eng.dst.cpu().numpy(), dst_want), replay
            got = eng.arena.cpu().numpy()
            used = staging_want != 0
            assert np.array_equal(got[used], staging_want[used]), replay
            H.assert_plan_equal(eng.table(), s, b)
            assert T.tent_poll(eng.ctx, eng.batch, eng.stream) == 0
        # eager calls still work after the graph
        T.tent_reset(eng.ctx, eng.batch, eng.stream)
        eng.dst.copy_(dst_reset)
        st, info = eng.plan()
        H.assert_plan_equal(eng.table(), s, b, info)
        eng.execute()
        assert np.array_equal(eng.dst.cpu().numpy(), dst_want)
