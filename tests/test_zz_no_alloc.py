"""tent_declare_static (the declaration for callers that cannot allocate) against tent_declare: the batch it
creates must plan and move exactly as the batch of the ordinary entry point does -- slice table, rails, staging
offsets, arena bytes and destination bytes bit for bit -- on two calls in a row, the second with a smaller input."""
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


def run_batch(T, eng, declare):
    """Declare with `declare`, plan, execute; returns (handle, plan info, slice table, arena bytes, destination bytes)."""
    eng.arena.zero_()
    torch.cuda.synchronize()
    h = declare(eng.ctx, eng.w.src_ptr, eng.w.src_ext, eng.w.dst_ptr, eng.w.dst_ext)
    st, info = T.tent_plan(eng.ctx, h, eng.w.rails, True, eng.stream)
    assert st == T.TENT_OK
    T.tent_execute(eng.ctx, h, eng.stream)
    assert T.tent_poll(eng.ctx, h, eng.stream) == 0
    return h, info, T.tent_get_plan(eng.ctx, h), eng.arena.cpu().numpy().copy(), eng.dst.cpu().numpy().copy()


def test_static_declare_matches_declare_twice_in_a_row(H, oracle):
    from paper_2604_00368_amd import binding as T
    from helpers import expected_destination
    first, second = W.small_variant("many_small"), W.tiny()            # the second input is the smaller one
    sizes = [(w.payload, int(w.src_ext.shape[0]), w.n_desc) for w in (first, second)]
    assert all(b < a for a, b in zip(*sizes)), sizes
    for w in (first, second):
        src, dst0 = W.fill_numpy(w, 0), W.fill_numpy(w, 1)
        with H.Engine(w, src, dst0) as eng:
            h_ref, info_ref, tab_ref, arena_ref, dst_ref = run_batch(T, eng, T.tent_declare)
            eng.dst.copy_(torch.from_numpy(dst0))
            free_before, _ = torch.cuda.mem_get_info()
            h_st = T.tent_declare_static(eng.ctx, w.src_ptr, w.src_ext, w.dst_ptr, w.dst_ext)
            free_after, _ = torch.cuda.mem_get_info()
            assert free_after == free_before                          # no device memory was taken
            assert (h_st & 0xFFFFFFFF) == 0xFFFFFFFF and h_st != h_ref
            st, info = T.tent_plan(eng.ctx, h_st, w.rails, True, eng.stream)
            assert st == T.TENT_OK
            T.tent_execute(eng.ctx, h_st, eng.stream)
            assert T.tent_poll(eng.ctx, h_st, eng.stream) == 0
            tab = T.tent_get_plan(eng.ctx, h_st)
            for f in tab.dtype.names:
                assert np.array_equal(tab[f], tab_ref[f]), f
            for f in ("n_slices", "n_pending_before"):
                assert getattr(info, f) == getattr(info_ref, f)
            for f in ("rail_bytes", "rail_slices", "queued_after", "stage_base"):
                assert list(getattr(info, f)) == list(getattr(info_ref, f)), f
            assert np.array_equal(eng.arena.cpu().numpy(), arena_ref)
            got = eng.dst.cpu().numpy()
            assert np.array_equal(got, dst_ref)
            assert np.array_equal(got, expected_destination(w, src, dst0))
            # the same handle keeps working with the other entry points: reset, plan, execute once more
            eng.dst.copy_(torch.from_numpy(dst0))
            T.tent_reset(eng.ctx, h_st, eng.stream)
            st, _ = T.tent_plan(eng.ctx, h_st, w.rails, True, eng.stream)
            T.tent_execute(eng.ctx, h_st, eng.stream)
            assert T.tent_poll(eng.ctx, h_st, eng.stream) == 0
            assert np.array_equal(eng.dst.cpu().numpy(), dst_ref)
            # a second static declaration in the same context replaces the first: the old handle dies
            h_st2 = T.tent_declare_static(eng.ctx, w.src_ptr, w.src_ext, w.dst_ptr, w.dst_ext)
            assert h_st2 != h_st
            with pytest.raises(T.TentError) as ei:
                T.tent_slice_count(eng.ctx, h_st)
            assert ei.value.status == T.TENT_ERR_INVALID
            assert T.tent_slice_count(eng.ctx, h_st2) == tab_ref.shape[0]
            T.tent_release(eng.ctx, h_st2)
            T.tent_release(eng.ctx, h_ref)


def test_static_declare_across_contexts_and_limits(H, oracle):
    from paper_2604_00368_amd import binding as T
    from helpers import expected_destination
    wa, wb = W.small_variant("many_small"), W.tiny()
    src_a, dst_a = W.fill_numpy(wa, 0), W.fill_numpy(wa, 1)
    src_b, dst_b = W.fill_numpy(wb, 0), W.fill_numpy(wb, 1)
    with H.Engine(wa, src_a, dst_a) as ea, H.Engine(wb, src_b, dst_b) as eb:
        ha = T.tent_declare_static(ea.ctx, wa.src_ptr, wa.src_ext, wa.dst_ptr, wa.dst_ext)
        st, _ = T.tent_plan(ea.ctx, ha, wa.rails, True, ea.stream)
        T.tent_execute(ea.ctx, ha, ea.stream)
        assert T.tent_poll(ea.ctx, ha, ea.stream) == 0
        assert np.array_equal(ea.dst.cpu().numpy(), expected_destination(wa, src_a, dst_a))
        # another context on the same GPU takes the static workspace over: the first context's handle is dead
        hb = T.tent_declare_static(eb.ctx, wb.src_ptr, wb.src_ext, wb.dst_ptr, wb.dst_ext)
        with pytest.raises(T.TentError) as ei:
            T.tent_plan(ea.ctx, ha, wa.rails, True, ea.stream)
        assert ei.value.status == T.TENT_ERR_INVALID
        st, _ = T.tent_plan(eb.ctx, hb, wb.rails, True, eb.stream)
        T.tent_execute(eb.ctx, hb, eb.stream)
        assert T.tent_poll(eb.ctx, hb, eb.stream) == 0
        assert np.array_equal(eb.dst.cpu().numpy(), expected_destination(wb, src_b, dst_b))
        # malformed input is rejected exactly as by tent_declare
        se = wb.src_ext.copy(); se["len"][3] = 0
        with pytest.raises(T.TentError) as ei:
            T.tent_declare_static(eb.ctx, wb.src_ptr, se, wb.dst_ptr, wb.dst_ext)
        assert ei.value.status == T.TENT_ERR_INVALID
        de = wb.dst_ext.copy(); de["off"][1] = de["off"][0] + 100          # overlap: reported by the first plan
        hx = T.tent_declare_static(eb.ctx, wb.src_ptr, wb.src_ext, wb.dst_ptr, de)
        with pytest.raises(T.TentError) as ei:
            T.tent_plan(eb.ctx, hx, wb.rails, True, eb.stream)
        assert ei.value.status == T.TENT_ERR_INVALID
    # a batch whose tables exceed the static workspace is refused with a range error; nothing is touched on the
    # device before that, so the segments only need the right lengths
    big = W.kv_migration(n_req=8)
    assert big.payload > (4 << 30)
    small = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda:0")
    ctx = T.tent_create(big.slice_bytes, small.data_ptr(), big.staging_bytes)
    try:
        T.tent_register_segment(ctx, small.data_ptr(), big.seg_bytes[0])
        T.tent_register_segment(ctx, small.data_ptr(), big.seg_bytes[1])
        with pytest.raises(T.TentError) as ei:
            T.tent_declare_static(ctx, big.src_ptr, big.src_ext, big.dst_ptr, big.dst_ext)
        assert ei.value.status == T.TENT_ERR_RANGE
    finally:
        T.tent_destroy(ctx)


def test_static_declare_uploads_large_arrays_in_pieces(H, oracle):
    # descriptor arrays larger than the context's pinned buffers (which the static entry point may not replace:
    # they hold 1 MiB each in a fresh context) travel through one of them piece by piece; the batch must still
    # equal the ordinary one
    from paper_2604_00368_amd import binding as T
    w = W.kv_migration(n_req=4)
    assert w.src_ext.shape[0] * 16 > (1 << 20)                         # one array alone needs more than one piece
    eng = H.Engine(w)                                                  # pools filled on the device
    try:
        free_before, _ = torch.cuda.mem_get_info()
        h_st = T.tent_declare_static(eng.ctx, w.src_ptr, w.src_ext, w.dst_ptr, w.dst_ext)
        free_after, _ = torch.cuda.mem_get_info()
        assert free_after == free_before
        st, info = T.tent_plan(eng.ctx, h_st, w.rails, True, eng.stream)
        assert st == T.TENT_OK
        T.tent_execute(eng.ctx, h_st, eng.stream)
        assert T.tent_poll(eng.ctx, h_st, eng.stream) == 0
        tab = T.tent_get_plan(eng.ctx, h_st)
        dst_st, arena_st = eng.dst.clone(), eng.arena.clone()
        eng.dst.zero_()
        eng.arena.zero_()
        h_ref = T.tent_declare(eng.ctx, w.src_ptr, w.src_ext, w.dst_ptr, w.dst_ext)
        st, info_ref = T.tent_plan(eng.ctx, h_ref, w.rails, True, eng.stream)
        T.tent_execute(eng.ctx, h_ref, eng.stream)
        assert T.tent_poll(eng.ctx, h_ref, eng.stream) == 0
        tab_ref = T.tent_get_plan(eng.ctx, h_ref)
        for f in tab.dtype.names:
            assert np.array_equal(tab[f], tab_ref[f]), f
        assert list(info.stage_base) == list(info_ref.stage_base)
        assert torch.equal(eng.dst, dst_st) and torch.equal(eng.arena, arena_st)
        s = oracle.split(w.src_ptr, w.src_ext, w.slice_bytes)
        b = oracle.bind(s.len, w.rails)
        H.assert_plan_equal(tab, s, b, info)
    finally:
        eng.close()
