// Tile tables of the copy kernels (slice decomposition of Section 4.2 carried down to tiles of
// 1-4 KiB): for every tile the device address of its bytes on the paged side, so that the copy
// kernels reach their bytes with one table load.  The builders are device functions over a
// virtual grid (block `vb` of `nb`, any block size), because they run in two places: as kernels of
// their own, and in the spare workgroups of the launch whose first workgroup walks the binding
// chain -- the chain is one wavefront and leaves the rest of the device idle, and the tables
// depend on the slice table only, not on the binding.
#pragma once

#include "tent_internal.h"

namespace tent {

// Largest index i in [lo, hi) with a[i] <= key (a is nondecreasing and a[lo] <= key).
__device__ __forceinline__ uint64_t last_not_above(const uint64_t* a, uint64_t lo, uint64_t hi, uint64_t key)
{
    while (hi - lo > 1) {
        uint64_t mid = lo + ((hi - lo) >> 1);
        if (a[mid] <= key) lo = mid; else hi = mid;
    }
    return lo;
}

// Geometry whose tiles may cross extent boundaries.  One thread per (slice, tile): locate the extent
// that holds the tile's first byte on either side; tiles that cross a boundary are flagged.
__device__ __forceinline__ void slice_tile_tables(const BatchDev& b, uint64_t vb, uint64_t nb)
{
    const uint64_t n = b.n_slices * (uint64_t)b.tiles_per_slice;
    const uint64_t stride = nb * blockDim.x;
    for (uint64_t q = vb * blockDim.x + threadIdx.x; q < n; q += stride) {
        const uint64_t i = q / b.tiles_per_slice;
        const uint64_t x = (q - i * b.tiles_per_slice) * b.tile_bytes;      // byte offset inside the slice
        const uint32_t len = b.s_len[i];
        if (x >= len) { b.src_tile[q] = kTileSlow; b.dst_tile[q] = kTileSlow; continue; }
        const uint64_t n_tile = len - x < b.tile_bytes ? len - x : b.tile_bytes;
        const uint32_t j = b.s_desc[i];
        {
            const uint32_t hi = b.src_ptr[j + 1];
            const uint64_t pos = b.src_pre[b.src_ptr[j]] + b.s_off[i] + x;
            const uint32_t e = (uint32_t)last_not_above(b.src_pre, b.s_src_e0[i], hi, pos);
            const tent_extent ex = b.src_ext[e];
            const uint64_t addr = b.seg_base[ex.seg] + ex.off + (pos - b.src_pre[e]);
            const bool slow = pos + n_tile > b.src_pre[e + 1];
            b.src_tile[q] = addr | (slow ? kTileSlow : 0);
        }
        {
            const uint32_t hi = b.dst_ptr[j + 1];
            const uint64_t pos = b.dst_pre[b.dst_ptr[j]] + b.s_off[i] + x;
            const uint32_t e = (uint32_t)last_not_above(b.dst_pre, b.s_dst_e0[i], hi, pos);
            const tent_extent ex = b.dst_ext[e];
            const uint64_t addr = b.seg_base[ex.seg] + ex.off + (pos - b.dst_pre[e]);
            const bool slow = pos + n_tile > b.dst_pre[e + 1];
            b.dst_tile[q] = addr | (slow ? kTileSlow : 0);
        }
    }
}

// Destination-ordered tiles: tile q covers bytes [q*tile, (q+1)*tile) of the destination extents
// laid end to end in ascending device address.  For each tile: its destination address, the slice
// that owns it and its offset inside that slice (independent of the binding).
__device__ __forceinline__ void scatter_tile_table(const BatchDev& b, uint64_t vb, uint64_t nb)
{
    const uint64_t stride = nb * blockDim.x;
    for (uint64_t q = vb * blockDim.x + threadIdx.x; q < b.n_sc_tiles; q += stride) {
        const uint64_t at = q * b.tile_bytes;
        const uint64_t r = last_not_above(b.ord_pre, 0, b.n_dst_ext, at);
        const uint32_t e = b.dst_order[r];
        const uint64_t within = at - b.ord_pre[r];
        const tent_extent ex = b.dst_ext[e];
        // owning transfer: last j with dst_ptr[j] <= e
        uint32_t lo = 0, hi = b.n_desc;
        while (hi - lo > 1) {
            const uint32_t mid = lo + ((hi - lo) >> 1);
            if (b.dst_ptr[mid] <= e) lo = mid; else hi = mid;
        }
        const uint64_t off = b.dst_pre[e] + within - b.dst_pre[b.dst_ptr[lo]];   // offset inside the transfer
        const uint64_t k = off / b.slice_bytes;
        b.sc_dst[q] = b.seg_base[ex.seg] + ex.off + within;
        b.sc_slice[q] = (uint32_t)(b.first[lo] + k);
        b.sc_x[q] = (uint32_t)(off - k * b.slice_bytes);
    }
}

// Source-ordered tiles: tile q covers bytes [q*tile, (q+1)*tile) of the source extents laid end to
// end in declaration order, i.e. of the transfers' logical bytes one after the other.
__device__ __forceinline__ void gather_tile_table(const BatchDev& b, uint64_t vb, uint64_t nb)
{
    const uint64_t stride = nb * blockDim.x;
    for (uint64_t q = vb * blockDim.x + threadIdx.x; q < b.n_sc_tiles; q += stride) {
        const uint64_t at = q * b.tile_bytes;
        const uint64_t e = last_not_above(b.src_pre, 0, b.n_src_ext, at);
        const tent_extent ex = b.src_ext[e];
        uint32_t lo = 0, hi = b.n_desc;                   // owning transfer: last j with src_ptr[j] <= e
        while (hi - lo > 1) {
            const uint32_t mid = lo + ((hi - lo) >> 1);
            if (b.src_ptr[mid] <= e) lo = mid; else hi = mid;
        }
        const uint64_t off = at - b.src_pre[b.src_ptr[lo]];
        const uint64_t k = off / b.slice_bytes;
        b.ga_src[q] = b.seg_base[ex.seg] + ex.off + (at - b.src_pre[e]);
        b.ga_slice[q] = (uint32_t)(b.first[lo] + k);
        b.ga_x[q] = (uint32_t)(off - k * b.slice_bytes);
        if (b.ga_dst) {                                   // same tile on the destination side
            const uint64_t dpos = b.dst_pre[b.dst_ptr[lo]] + off;
            const uint64_t de = last_not_above(b.dst_pre, b.dst_ptr[lo], b.dst_ptr[lo + 1], dpos);
            const tent_extent dx = b.dst_ext[de];
            b.ga_dst[q] = b.seg_base[dx.seg] + dx.off + (dpos - b.dst_pre[de]);
        }
    }
}

// All tile tables of a batch, whichever its geometry.
__device__ __forceinline__ void build_tile_tables(const BatchDev& b, uint64_t vb, uint64_t nb)
{
    if (b.n_sc_tiles == 0) {
        slice_tile_tables(b, vb, nb);
    } else {
        gather_tile_table(b, vb, nb);
        scatter_tile_table(b, vb, nb);
    }
}

// Workgroups of 256 lanes that the table builders are launched with.
inline uint32_t tile_table_blocks(const BatchDev& b)
{
    const uint64_t n = b.n_sc_tiles ? b.n_sc_tiles : b.n_slices * (uint64_t)b.tiles_per_slice;
    const uint64_t blocks = (n + 255) / 256;
    return (uint32_t)(blocks > 65536 ? 65536 : (blocks ? blocks : 1));
}

}  // namespace tent
