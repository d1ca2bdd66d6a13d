// Device side of tent_declare: destination extents in ascending device address (the order in which
// the scatter kernel walks them) and the overlap check between extents.
//
// All extents get a 64-bit key (device address of their first byte) and are sorted with rocPRIM's
// radix sort (the one library primitive of the build).  Over the sorted order, "furthest end seen so
// far" is an exclusive max-scan; a destination extent overlaps something iff it starts before the
// furthest end of everything before it, a source extent overlaps a destination iff it starts before
// the furthest end of the destinations before it.  The scans are the engine's own (scan.h).
//
// Nothing here allocates, copies to the host or waits: the caller hands in a workspace and reads
// the verdict from device memory when the stream has got that far.
#include <cstring>

#include <rocprim/rocprim.hpp>

#include "scan.h"

namespace tent {

namespace {

// value = index into [destinations | sources]: v < n_dst is destination extent v
__global__ void __launch_bounds__(256) declare_keys_kernel(const tent_extent* dst_ext, uint64_t n_dst,
                                                           const tent_extent* src_ext, uint64_t n_src,
                                                           const uint64_t* seg_base, uint64_t* keys, uint32_t* vals,
                                                           uint32_t* overlap)
{
    const uint64_t n = n_dst + n_src;
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t v = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; v < n; v += stride) {
        const tent_extent x = v < n_dst ? dst_ext[v] : src_ext[v - n_dst];
        keys[v] = seg_base[x.seg] + x.off;
        vals[v] = (uint32_t)v;
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) *overlap = 0;
}

// End of the extent at sorted position p (all extents / destinations only).
struct EndAny {
    const tent_extent* dst_ext; const tent_extent* src_ext; uint64_t n_dst;
    const uint64_t* keys; const uint32_t* vals;
    __device__ uint64_t operator()(uint64_t p) const
    {
        const uint32_t v = vals[p];
        return keys[p] + (v < n_dst ? dst_ext[v].len : src_ext[v - n_dst].len);
    }
};
struct EndDst {
    const tent_extent* dst_ext; uint64_t n_dst;
    const uint64_t* keys; const uint32_t* vals;
    __device__ uint64_t operator()(uint64_t p) const
    {
        const uint32_t v = vals[p];
        return v < n_dst ? keys[p] + dst_ext[v].len : 0;
    }
};
struct IsDst {
    const uint32_t* vals; uint64_t n_dst;
    __device__ uint64_t operator()(uint64_t p) const { return vals[p] < n_dst; }
};

__global__ void __launch_bounds__(256) declare_check_kernel(uint64_t n_dst, uint64_t n, const uint64_t* keys,
                                                            const uint32_t* vals, const uint64_t* far_any,
                                                            const uint64_t* far_dst, uint32_t* overlap)
{
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    bool bad = false;
    for (uint64_t p = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; p < n; p += stride) {
        const bool is_dst = vals[p] < n_dst;
        bad |= keys[p] < (is_dst ? far_any[p] : far_dst[p]);
    }
    if (bad) atomicOr(overlap, 1u);
}

// destinations in sorted order: stable compaction of the sorted values
__global__ void __launch_bounds__(256) declare_order_kernel(uint64_t n_dst, uint64_t n, const uint32_t* vals,
                                                            const uint64_t* pos, uint32_t* order, uint32_t* rank)
{
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t p = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; p < n; p += stride)
        if (vals[p] < n_dst) {
            order[pos[p]] = vals[p];
            if (rank) rank[vals[p]] = (uint32_t)pos[p];    // the inverse: position of every extent in address order
        }
}

uint32_t grid_for(uint64_t n)
{
    uint64_t blocks = (n + 255) / 256;
    return (uint32_t)(blocks < 1 ? 1 : (blocks > 8192 ? 8192 : blocks));
}

size_t up256(size_t x) { return (x + 255) & ~(size_t)255; }

// Carves the workspace: two key arrays, two value arrays, three scan outputs, scan partials, the
// sort's own temporary storage.
struct OrderWorkspace {
    uint64_t *keys_in, *keys, *far_any, *far_dst, *pos, *partials;
    uint32_t *vals_in, *vals;
    void* sort_tmp;
    size_t sort_bytes, total;
};

hipError_t layout(uint64_t n, uint8_t* base, OrderWorkspace* w)
{
    size_t sort_bytes = 0;
    hipError_t e = rocprim::radix_sort_pairs(nullptr, sort_bytes, (uint64_t*)nullptr, (uint64_t*)nullptr,
                                             (uint32_t*)nullptr, (uint32_t*)nullptr, n, 0, 64, nullptr);
    if (e != hipSuccess) return e;
    const size_t n8 = up256((size_t)(n + 1) * 8), n4 = up256((size_t)n * 4);
    size_t at = 0;
    auto take = [&](size_t bytes) { uint8_t* p = base ? base + at : nullptr; at += up256(bytes); return p; };
    w->keys_in = (uint64_t*)take(n8);
    w->keys = (uint64_t*)take(n8);
    w->far_any = (uint64_t*)take(n8);
    w->far_dst = (uint64_t*)take(n8);
    w->pos = (uint64_t*)take(n8);
    w->partials = (uint64_t*)take(scan_partials_capacity(n) * 8);
    w->vals_in = (uint32_t*)take(n4);
    w->vals = (uint32_t*)take(n4);
    w->sort_tmp = take(sort_bytes);
    w->sort_bytes = sort_bytes;
    w->total = at;
    return hipSuccess;
}

}  // namespace

// Bytes of workspace device_order_destinations needs for n_dst destination and n_src source extents.
hipError_t order_workspace_bytes(uint64_t n_dst, uint64_t n_src, bool check, uint64_t* bytes_out)
{
    OrderWorkspace w;
    hipError_t e = layout(n_dst + (check ? n_src : 0), nullptr, &w);
    *bytes_out = w.total;
    return e;
}

// Fills order_out[n_dst] with destination extent indices in ascending address, rank_out[n_dst] (if
// not null) with the inverse (position of every extent in that order) and, when `check` is set,
// *overlap_dev (device) with 1 if a destination extent overlaps another destination or any source
// extent, else 0.  Only enqueues on `s`; `workspace` (device, order_workspace_bytes() bytes, 256-byte
// aligned) is in use until the stream has passed this work.
hipError_t device_order_destinations(const tent_extent* dst_ext, uint64_t n_dst, const tent_extent* src_ext,
                                     uint64_t n_src, const uint64_t* seg_base, bool check, uint32_t* order_out,
                                     uint32_t* rank_out, uint32_t* overlap_dev, void* workspace, hipStream_t s)
{
    const uint64_t n = n_dst + (check ? n_src : 0);
    OrderWorkspace w;
    hipError_t e = layout(n, static_cast<uint8_t*>(workspace), &w);
    if (e != hipSuccess) return e;
    const uint32_t g = grid_for(n);
    hipLaunchKernelGGL(declare_keys_kernel, dim3(g), dim3(256), 0, s, dst_ext, n_dst, src_ext, check ? n_src : 0,
                       seg_base, w.keys_in, w.vals_in, overlap_dev);
    size_t bytes = w.sort_bytes;
    e = rocprim::radix_sort_pairs(w.sort_tmp, bytes, w.keys_in, w.keys, w.vals_in, w.vals, n, 0, 64, s);
    if (e != hipSuccess) return e;
    if (check) {
        e = exclusive_scan(EndAny{dst_ext, src_ext, n_dst, w.keys, w.vals}, n, w.far_any, w.partials, s, ScanMax{});
        if (e != hipSuccess) return e;
        e = exclusive_scan(EndDst{dst_ext, n_dst, w.keys, w.vals}, n, w.far_dst, w.partials, s, ScanMax{});
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(declare_check_kernel, dim3(g), dim3(256), 0, s, n_dst, n, w.keys, w.vals, w.far_any,
                           w.far_dst, overlap_dev);
    }
    e = exclusive_scan(IsDst{w.vals, n_dst}, n, w.pos, w.partials, s);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(declare_order_kernel, dim3(g), dim3(256), 0, s, n_dst, n, w.vals, w.pos, order_out, rank_out);
    return hipGetLastError();
}

}  // namespace tent
