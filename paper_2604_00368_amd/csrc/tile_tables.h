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

// Geometry in which no tile crosses an extent boundary: two enumerations of the payload in tiles.
//   Source-ordered:      tile q covers bytes [q*tile, (q+1)*tile) of the source extents laid end to end in
//                        declaration order, i.e. of the transfers' logical bytes one after the other.
//   Destination-ordered: tile q' covers bytes [q'*tile, (q'+1)*tile) of the destination extents laid end
//                        to end in ascending device address.
// For each tile of either enumeration: its address on the paged side, the slice that owns it and its
// offset inside that slice (independent of the binding).  One thread per (slice, tile of the slice):
// the slice table already holds the first source and destination extent of the slice, so each side
// costs a search over the few extents of one slice; the tile's place in the destination order
// follows from the rank of its extent in that order and the prefix of the extent lengths.
__device__ __forceinline__ void ordered_tile_tables(const BatchDev& b, uint64_t vb, uint64_t nb)
{
    const uint32_t tps = b.tiles_per_slice;
    const uint32_t tile = b.tile_bytes;
    const uint64_t n = b.n_slices * (uint64_t)tps;
    const uint64_t stride = nb * blockDim.x;
    for (uint64_t idx = vb * blockDim.x + threadIdx.x; idx < n; idx += stride) {
        const uint64_t i = idx / tps;
        const uint64_t x = (idx - i * tps) * tile;                 // byte offset inside the slice
        if (x >= b.s_len[i]) continue;
        const uint32_t j = b.s_desc[i];
        const uint64_t off = b.s_off[i] + x;                       // byte offset inside the transfer
        const uint64_t s_pos = b.src_pre[b.src_ptr[j]] + off;
        const uint64_t se = last_not_above(b.src_pre, b.s_src_e0[i], b.src_ptr[j + 1], s_pos);
        const tent_extent sx = b.src_ext[se];
        const uint64_t q = s_pos / tile;
        b.ga_src[q] = b.seg_base[sx.seg] + sx.off + (s_pos - b.src_pre[se]);
        b.ga_slice[q] = (uint32_t)i;
        b.ga_x[q] = (uint32_t)x;
        const uint64_t d_pos = b.dst_pre[b.dst_ptr[j]] + off;
        const uint64_t de = last_not_above(b.dst_pre, b.s_dst_e0[i], b.dst_ptr[j + 1], d_pos);
        const tent_extent dx = b.dst_ext[de];
        const uint64_t within = d_pos - b.dst_pre[de];
        const uint64_t dst_addr = b.seg_base[dx.seg] + dx.off + within;
        if (b.ga_dst) b.ga_dst[q] = dst_addr;                      // same tile on the destination side
        const uint64_t qd = (b.ord_pre[b.dst_rank[de]] + within) / tile;
        b.sc_dst[qd] = dst_addr;
        b.sc_slice[qd] = (uint32_t)i;
        b.sc_x[qd] = (uint32_t)x;
    }
}

// All tile tables of a batch, whichever its geometry.
__device__ __forceinline__ void build_tile_tables(const BatchDev& b, uint64_t vb, uint64_t nb)
{
    if (b.n_sc_tiles == 0) {
        slice_tile_tables(b, vb, nb);
    } else {
        ordered_tile_tables(b, vb, nb);
    }
}

// Workgroups of 256 lanes that the table builders are launched with.
inline uint32_t tile_table_blocks(const BatchDev& b)
{
    const uint64_t n = b.n_slices * (uint64_t)b.tiles_per_slice;
    const uint64_t blocks = (n + 255) / 256;
    return (uint32_t)(blocks > 65536 ? 65536 : (blocks ? blocks : 1));
}

}  // namespace tent
