"""Drives the engine through its C ABI on cuda:0 for the GPU parity tests."""
from __future__ import annotations

import numpy as np
import torch

from paper_2604_00368_amd import binding as T
from paper_2604_00368_amd import workloads as W


class Engine:
    """Device pools + one engine context for one workload (torch only provides memory and the stream)."""

    def __init__(self, w, src_host=None, dst_host=None, flags=0, device="cuda:0", arena_skew=0, arena_bytes=None,
                 pools=None):
        self.w = w
        self.dev = torch.device(device)
        torch.cuda.set_device(self.dev)
        if pools is not None:                       # (src, arena, dst) allocated by the caller; src is filled here
            self.src, arena, self.dst = pools
            W.fill_torch(w, 0, self.dev, out=self.src)
            self.dst.zero_()
            arena.zero_()
        elif src_host is not None:
            self.src = torch.from_numpy(src_host).to(self.dev)
        else:
            self.src = W.fill_torch(w, 0, self.dev)
        if pools is not None:
            pass
        elif dst_host is not None:
            self.dst = torch.from_numpy(dst_host).to(self.dev)
        else:
            self.dst = torch.zeros(w.seg_bytes[1], dtype=torch.uint8, device=self.dev)
        # arena_skew > 0 hands the engine a staging arena that starts at an odd address
        n_arena = w.staging_bytes if arena_bytes is None else arena_bytes
        if pools is not None:
            self.arena_full = self.arena = arena
        else:
            self.arena_full = torch.zeros(n_arena + arena_skew, dtype=torch.uint8, device=self.dev)
            self.arena = self.arena_full[arena_skew:]
        self.stream = torch.cuda.current_stream(self.dev)
        self.ctx = T.tent_create(w.slice_bytes, self.arena.data_ptr(), self.arena.numel(), flags)
        s0 = T.tent_register_segment(self.ctx, self.src.data_ptr(), self.src.numel())
        s1 = T.tent_register_segment(self.ctx, self.dst.data_ptr(), self.dst.numel())
        assert (s0, s1) == (W.SRC_SEG, W.DST_SEG)
        self.batch = None

    def declare(self):
        self.batch = T.tent_declare(self.ctx, self.w.src_ptr, self.w.src_ext, self.w.dst_ptr, self.w.dst_ext)
        return self.batch

    def plan(self, rails=None, want_info=True):
        return T.tent_plan(self.ctx, self.batch, self.w.rails if rails is None else rails, want_info, self.stream)

    def execute(self):
        T.tent_execute(self.ctx, self.batch, self.stream)
        torch.cuda.synchronize(self.dev)

    def table(self):
        return T.tent_get_plan(self.ctx, self.batch)

    def close(self):
        if self.ctx is not None:
            T.tent_destroy(self.ctx)
            self.ctx = None

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()


def assert_plan_equal(table, s, b, info=None, ids=None):
    """Slice table, rails and staging offsets are bit-identical to the oracle's."""
    assert table.shape[0] == s.n
    assert np.array_equal(table["desc"], s.desc)
    assert np.array_equal(table["off"], s.off)
    assert np.array_equal(table["len"], s.len)
    sel = slice(None) if ids is None else ids
    assert np.array_equal(table["rail"][sel], b.rail[sel])
    assert np.array_equal(table["stage_off"][sel], b.stage_off[sel])
    if info is not None:
        R = b.T.shape[0]
        assert list(info.rail_bytes)[:R] == b.T.tolist()
        assert list(info.rail_slices)[:R] == b.n_slices.tolist()
        assert list(info.queued_after)[:R] == b.A_after.tolist()
        assert list(info.stage_base)[:R] == b.base.tolist()
        assert info.n_slices == int(b.n_slices.sum())
