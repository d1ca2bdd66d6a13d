// Gather / scatter of slice bytes between paged extents and per-rail staging regions.
//
// Gather: slice bytes are read from the transfer's source extents (the paged side) and written
// contiguously at the slice's staging address (the staging hop of Section 4.1 of the paper).
// Scatter: the same bytes are read back from staging and written to the destination extents at
// the slice's absolute offset inside the transfer (direct-to-offset writes, Section 4.4), so the
// result does not depend on the order in which slices are moved.
//
// Work decomposition: one 256-lane workgroup per 4 KiB block of a slice, one 16-byte vector per
// lane, and the workgroup ends after its store.  Consecutive workgroups touch consecutive staging
// addresses, so the set of DRAM pages open at any time stays small; on MI355X this one-shot shape
// sustains more bandwidth than persistent workgroups that loop over larger chunks.  The paged-side
// address comes from the tile table built by the splitter (one 8-byte entry per tile of 1-4 KiB),
// looked up per lane, so extent boundaries inside a block cost nothing as long as they fall on
// tile boundaries, at any address alignment.  A wavefront that meets a flagged tile (extent
// boundary inside the tile) or a slice that ends inside a lane's vector takes the
// generic path, which walks the extent list, aligns its stores and loads at any alignment.
#include "copy_generic.h"

namespace tent {

// One workgroup moves kLanes*16 bytes of one slice; every wavefront is independent of the others
// (no barrier): it moves 1 KiB with one 16-byte vector per lane.  The slice record (scalar load)
// and the tile entry (one load per lane) are fetched together before the first branch, so a
// wavefront sees two memory round trips before its data load: kernel arguments, then metadata.
template <bool kGather, int kLanes>
__global__ void __launch_bounds__(kLanes) copy_kernel(const SliceRec* __restrict__ rec, const uint64_t* __restrict__ tab,
                                                      uint64_t n_slices, uint32_t bps, uint32_t bps_shift,
                                                      uint32_t tiles_per_slice, uint32_t tile_shift,
                                                      const BatchDev* __restrict__ batch)
{
    constexpr uint32_t kBlockBytes = kLanes * 16;
    const uint64_t w = (uint64_t)blockIdx.y * gridDim.x + blockIdx.x;
    const uint64_t i = bps_shift != 0xFFFFFFFFu ? (w >> bps_shift)
                       : (w >> 32) == 0 ? (uint64_t)((uint32_t)w / bps) : w / bps;
    if (i >= n_slices) return;
    const uint32_t c = (uint32_t)(w - i * bps);
    const uint32_t x = c * kBlockBytes + threadIdx.x * 16;   // this lane's byte offset inside the slice
    uint32_t t = x >> tile_shift;
    if (t >= tiles_per_slice) t = tiles_per_slice - 1;
    const uint64_t entry = tab[i * tiles_per_slice + t];
    const SliceRec r = rec[i];
    const bool in_range = x + 16 <= r.len;
    const bool ragged = x < r.len && !in_range;              // slice ends inside this lane's vector
    const bool bad = ragged || (x < r.len && (entry & kTileSlow));
    if (__any(bad)) {
        const uint32_t wave_lo = c * kBlockBytes + (threadIdx.x & ~63u) * 16;
        const uint32_t wave_hi = wave_lo + 1024 < r.len ? wave_lo + 1024 : r.len;
        copy_range_generic<kGather>(*batch, i, wave_lo, wave_hi, (uint8_t*)(r.lin + wave_lo));
        return;
    }
    if (!in_range) return;
    const uint64_t paged = entry + (x & ((1u << tile_shift) - 1));
    const uint64_t mine = r.lin + x;
    if (kGather) {
        vec4u v = __builtin_nontemporal_load((const vec4u_any*)paged);
        __builtin_nontemporal_store(v, (vec4u_any*)mine);
    } else {
        vec4u v = __builtin_nontemporal_load((const vec4u_any*)mine);
        __builtin_nontemporal_store(v, (vec4u_any*)paged);
    }
}

template <bool kGather, int kLanes>
static hipError_t launch_copy_lanes(const BatchDev& b, hipStream_t s)
{
    const uint32_t block_bytes = kLanes * 16;
    const uint32_t bps = (uint32_t)((b.slice_bytes + block_bytes - 1) / block_bytes);
    uint32_t bps_shift = 0xFFFFFFFFu;
    if ((bps & (bps - 1)) == 0) { bps_shift = 0; while ((1u << bps_shift) < bps) ++bps_shift; }
    uint32_t tile_shift = 0;
    while ((1u << tile_shift) < b.tile_bytes) ++tile_shift;
    const uint64_t blocks = b.n_slices * (uint64_t)bps;
    if (blocks == 0) return hipSuccess;
    // 2-D grid so that the block count is not capped by the 1-D limit
    const uint32_t gx = blocks < 65536 ? (uint32_t)blocks : 65536u;
    const uint64_t gy = (blocks + gx - 1) / gx;
    if (gy > 0x7FFFFFFFull) return hipErrorInvalidValue;
    hipLaunchKernelGGL((copy_kernel<kGather, kLanes>), dim3(gx, (uint32_t)gy), dim3(kLanes), 0, s,
                       b.s_rec, kGather ? b.src_tile : b.dst_tile, b.n_slices, bps, bps_shift,
                       b.tiles_per_slice, tile_shift, b.self);
    return hipGetLastError();
}

// Table-driven copy: workgroup w moves block w (kOrderedLanes x 16 bytes) of an enumeration of the payload in tiles;
// `from` and `to` hold the two addresses of every tile (0 = tile not to be moved).  Gather walks the
// source bytes in declaration order (reads hop between pages, every rail region is written front to
// back); scatter walks the destination bytes in ascending device address (reads hop between the
// rail regions, writes are sequential) -- HBM tolerates scattered reads better than scattered
// writes.  Only used when no tile crosses an extent boundary.  kGather only names the direction
// (the two launches show up separately in a kernel trace); the code is the same.
template <bool kGather>
__global__ void __launch_bounds__(kOrderedLanes) ordered_copy_kernel(const uint64_t* __restrict__ from,
                                                                     const uint64_t* __restrict__ to,
                                                                     uint64_t n_tiles, uint32_t tile_shift)
{
    const uint64_t w = (uint64_t)blockIdx.y * gridDim.x + blockIdx.x;
    const uint64_t at = w * (kOrderedLanes * 16) + (uint64_t)threadIdx.x * 16;   // byte in enumeration order
    // The tile index is the same for all lanes of a wavefront, but the table entries are fetched with
    // ordinary per-lane loads (one cache line per wavefront): scalar loads measured 1 % faster on the
    // KV-migration workload and 2-4 % slower on contiguous tensors and on 2 KiB tiles.
    const uint64_t q = at >> tile_shift;
    if (q >= n_tiles) return;
    const uint64_t src = from[q];
    const uint64_t dst = to[q];
    if (src == 0 || dst == 0) return;
    const uint64_t in_tile = at & ((1ull << tile_shift) - 1);
    vec4u v = __builtin_nontemporal_load((const vec4u_dev*)(src + in_tile));
    __builtin_nontemporal_store(v, (vec4u_dev*)(dst + in_tile));
}

hipError_t launch_copy_ordered(const BatchDev& b, bool gather, hipStream_t s)
{
    uint32_t tile_shift = 0;
    while ((1u << tile_shift) < b.tile_bytes) ++tile_shift;
    const uint64_t bytes = b.n_sc_tiles * (uint64_t)b.tile_bytes;
    const uint64_t block_bytes = kOrderedLanes * 16;
    const uint64_t blocks = (bytes + block_bytes - 1) / block_bytes;
    if (blocks == 0) return hipSuccess;
    const uint32_t gx = blocks < 65536 ? (uint32_t)blocks : 65536u;
    const uint64_t gy = (blocks + gx - 1) / gx;
    if (gy > 0x7FFFFFFFull) return hipErrorInvalidValue;
    const dim3 grid(gx, (uint32_t)gy);
    if (gather)
        hipLaunchKernelGGL(ordered_copy_kernel<true>, grid, dim3(kOrderedLanes), 0, s, b.ga_src, b.ga_lin, b.n_sc_tiles,
                           tile_shift);
    else
        hipLaunchKernelGGL(ordered_copy_kernel<false>, grid, dim3(kOrderedLanes), 0, s, b.sc_lin, b.sc_dst, b.n_sc_tiles,
                           tile_shift);
    return hipGetLastError();
}

// The same copy over a list of tiles (one workgroup per listed tile, tile_bytes / 16 lanes): used when
// few slices of the batch move, so that the launch is sized by what moves.  The grid is an upper
// bound known to the host; workgroups beyond the device-side count leave at once.
template <bool kGather>
__global__ void __launch_bounds__(256) compact_copy_kernel(const uint64_t* __restrict__ from,
                                                           const uint64_t* __restrict__ to,
                                                           const uint64_t* __restrict__ n_act)
{
    const uint64_t w = (uint64_t)blockIdx.y * gridDim.x + blockIdx.x;
    if (w >= *n_act) return;
    const uint64_t src = from[w];
    const uint64_t dst = to[w];
    const uint64_t in_tile = (uint64_t)threadIdx.x * 16;
    vec4u v = __builtin_nontemporal_load((const vec4u_dev*)(src + in_tile));
    __builtin_nontemporal_store(v, (vec4u_dev*)(dst + in_tile));
}

hipError_t launch_copy_compact(const BatchDev& b, bool gather, uint64_t max_tiles, hipStream_t s)
{
    if (max_tiles > b.act_capacity) max_tiles = b.act_capacity;
    if (max_tiles == 0) return hipSuccess;
    const uint32_t gx = max_tiles < 65536 ? (uint32_t)max_tiles : 65536u;
    const uint64_t gy = (max_tiles + gx - 1) / gx;
    if (gy > 0x7FFFFFFFull) return hipErrorInvalidValue;
    const dim3 grid(gx, (uint32_t)gy), block(b.tile_bytes / 16);
    if (gather)
        hipLaunchKernelGGL(compact_copy_kernel<true>, grid, block, 0, s, b.act_src, b.act_lin, &b.plan->n_act);
    else
        hipLaunchKernelGGL(compact_copy_kernel<false>, grid, block, 0, s, b.act_lin, b.act_dst, &b.plan->n_act);
    return hipGetLastError();
}

hipError_t launch_copy(const BatchDev& b, bool gather, hipStream_t s)
{
    // 256 lanes (4 KiB per workgroup) measured best among 64/128/256/512 on MI355X
    return gather ? launch_copy_lanes<true, 256>(b, s) : launch_copy_lanes<false, 256>(b, s);
}

}  // namespace tent
