"""Slice-size sweep of the plan and copy stages on cuda:0 (prints one table row per slice size and layout).

    python -m paper_2604_00368_amd.sweep [--payload-gib 4]

Fixed payload in 64 equal transfers, 9 rails as in the KV-migration workload; layouts: one contiguous extent per
transfer, and 32 KiB pages shuffled on both sides.  GB/s counts bytes read plus bytes written."""
from __future__ import annotations

import argparse

import numpy as np


def main():
    import torch
    from . import binding as T
    from . import placement
    from . import workloads as W
    ap = argparse.ArgumentParser()
    ap.add_argument("--payload-gib", type=int, default=4)
    ap.add_argument("--reps", type=int, default=4)
    ap.add_argument("--placement", default="regions", choices=["regions", "plain"],
                    help="regions: pools carved so that either copy crosses memory regions (placement.py); plain: "
                         "ordinary allocations")
    args = ap.parse_args()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    payload = args.payload_gib << 30
    stream = torch.cuda.current_stream(dev)
    # one set of pools for the whole sweep, large enough for every layout (the paged pools carry some slack)
    biggest = [W.sweep(kib * 1024, paged, payload=payload) for paged in (False, True) for kib in (4, 65536)]
    n_src = max(w.seg_bytes[0] for w in biggest)
    n_dst = max(w.seg_bytes[1] for w in biggest)
    n_arena = max(w.staging_bytes for w in biggest)
    src_pool, arena_pool, dst_pool, layout = placement.place_pools(dev, n_src, n_arena, n_dst, mode=args.placement)
    print(f"placement: {layout.mode} ({layout.note}); region map {''.join(str(x) for x in layout.labels)}, "
          f"offsets GiB {[round(o / 2**30, 1) for o in layout.offsets]}")
    print(f"{'layout':12s} {'slice':>8s} {'slices':>9s} {'plan ms':>9s} {'M slices/s':>11s} {'gather GB/s':>12s} "
          f"{'scatter GB/s':>13s} {'execute GB/s':>13s}")
    for paged in (False, True):
        for kib in (4, 16, 64, 256, 1024, 4096, 16384, 65536):
            w = W.sweep(kib * 1024, paged, payload=payload)
            src = src_pool[:w.seg_bytes[0]]
            dst = dst_pool[:w.seg_bytes[1]]
            arena = arena_pool[:w.staging_bytes]
            W.fill_torch(w, 0, dev, out=src)
            dst.zero_()
            ctx = T.tent_create(w.slice_bytes, arena.data_ptr(), arena.numel(), T.TENT_FLAG_PROFILE)
            T.tent_register_segment(ctx, src.data_ptr(), src.numel())
            T.tent_register_segment(ctx, dst.data_ptr(), dst.numel())
            h = T.tent_declare(ctx, w.src_ptr, w.src_ext, w.dst_ptr, w.dst_ext)
            n = T.tent_slice_count(ctx, h)
            for rep in range(args.reps + 1):
                T.tent_reset(ctx, h, stream)
                T.tent_plan(ctx, h, w.rails, want_info=False, stream=stream)
                T.tent_execute(ctx, h, stream)
                if rep == 0:
                    torch.cuda.synchronize(dev)
                    T.tent_get_timings(ctx)                     # drop the warm-up
            torch.cuda.synchronize(dev)
            tm = T.tent_get_timings(ctx)
            assert T.tent_poll(ctx, h, stream) == 0
            plan = sum(tm[k][0] for k in ("extent_scan", "slice_scan", "expand", "compact", "bind")) / args.reps
            g = tm["gather"][0] / tm["gather"][1]
            s = tm["scatter"][0] / tm["scatter"][1]
            print(f"{'paged 32K' if paged else 'contiguous':12s} {kib:6d}Ki {n:9d} {plan:9.3f} {n / plan / 1e3:11.1f} "
                  f"{2 * w.payload / g / 1e6:12.0f} {2 * w.payload / s / 1e6:13.0f} {4 * w.payload / (g + s) / 1e6:13.0f}",
                  flush=True)
            T.tent_destroy(ctx)


if __name__ == "__main__":
    main()
