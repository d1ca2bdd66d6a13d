// Device side of tent_declare: destination extents in ascending device address (the order in which
// the scatter kernel walks them) and the overlap check between extents.
//
// All extents get a 64-bit key (device address of their first byte) and are sorted with rocPRIM's
// radix sort (a library primitive: declaring a batch is not part of the per-step path).  Over the
// sorted order, "furthest end seen so far" is an exclusive max-scan; a destination extent overlaps
// something iff it starts before the furthest end of everything before it, a source extent overlaps
// a destination iff it starts before the furthest end of the destinations before it.
#include <cstring>

#include <rocprim/rocprim.hpp>

#include "tent_internal.h"

namespace tent {

namespace {

struct MaxOp {
    __device__ uint64_t operator()(uint64_t a, uint64_t b) const { return a > b ? a : b; }
};

// value = index into [destinations | sources]: v < n_dst is destination extent v
__global__ void __launch_bounds__(256) declare_keys_kernel(const tent_extent* dst_ext, uint64_t n_dst,
                                                           const tent_extent* src_ext, uint64_t n_src,
                                                           const uint64_t* seg_base, uint64_t* keys, uint32_t* vals)
{
    const uint64_t n = n_dst + n_src;
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t v = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; v < n; v += stride) {
        const tent_extent x = v < n_dst ? dst_ext[v] : src_ext[v - n_dst];
        keys[v] = seg_base[x.seg] + x.off;
        vals[v] = (uint32_t)v;
    }
}

// ends of all extents / of destinations only, in sorted order
__global__ void __launch_bounds__(256) declare_ends_kernel(const tent_extent* dst_ext, uint64_t n_dst,
                                                           const tent_extent* src_ext, uint64_t n,
                                                           const uint64_t* keys, const uint32_t* vals,
                                                           uint64_t* end_any, uint64_t* end_dst)
{
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t p = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; p < n; p += stride) {
        const uint32_t v = vals[p];
        const bool is_dst = v < n_dst;
        const uint64_t end = keys[p] + (is_dst ? dst_ext[v].len : src_ext[v - n_dst].len);
        end_any[p] = end;
        end_dst[p] = is_dst ? end : 0;
    }
}

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
__global__ void __launch_bounds__(256) declare_is_dst_kernel(uint64_t n_dst, uint64_t n, const uint32_t* vals, uint32_t* flag)
{
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t p = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; p < n; p += stride) flag[p] = vals[p] < n_dst;
}

__global__ void __launch_bounds__(256) declare_order_kernel(uint64_t n_dst, uint64_t n, const uint32_t* vals,
                                                            const uint32_t* pos, uint32_t* order, uint32_t* rank)
{
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t p = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; p < n; p += stride)
        if (vals[p] < n_dst) {
            order[pos[p]] = vals[p];
            if (rank) rank[vals[p]] = pos[p];              // the inverse: position of every extent in address order
        }
}

__global__ void declare_clear_kernel(uint32_t* overlap) { *overlap = 0; }

uint32_t grid_for(uint64_t n)
{
    uint64_t blocks = (n + 255) / 256;
    return (uint32_t)(blocks < 1 ? 1 : (blocks > 8192 ? 8192 : blocks));
}

}  // namespace

// Fills order_out[n_dst] with destination extent indices in ascending address, rank_out[n_dst] (if
// not null) with the inverse (position of every extent in that order) and, when `check` is set,
// *overlap_out (host) with 1 if a destination extent overlaps another destination or any source
// extent.  Synchronous; temporary device memory is allocated and freed inside.
hipError_t device_order_destinations(const tent_extent* dst_ext, uint64_t n_dst, const tent_extent* src_ext,
                                     uint64_t n_src, const uint64_t* seg_base, bool check, uint32_t* order_out,
                                     uint32_t* rank_out, uint32_t* overlap_out, hipStream_t s)
{
    const uint64_t n = n_dst + (check ? n_src : 0);
    *overlap_out = 0;
    uint8_t* tmp = nullptr;
    // layout: keys_in (later end_any), keys, far_any, far_dst, end_dst, vals_in, vals, flag, pos, overlap, library scratch
    const size_t n8 = (size_t)n * 8, n4 = ((size_t)n * 4 + 7) & ~(size_t)7;
    size_t sort_bytes = 0, scan64_bytes = 0, scan32_bytes = 0;
    hipError_t e = rocprim::radix_sort_pairs(nullptr, sort_bytes, (uint64_t*)nullptr, (uint64_t*)nullptr,
                                             (uint32_t*)nullptr, (uint32_t*)nullptr, n, 0, 64, s);
    if (e != hipSuccess) return e;
    e = rocprim::exclusive_scan(nullptr, scan64_bytes, (uint64_t*)nullptr, (uint64_t*)nullptr, (uint64_t)0, n, MaxOp{}, s);
    if (e != hipSuccess) return e;
    e = rocprim::exclusive_scan(nullptr, scan32_bytes, (uint32_t*)nullptr, (uint32_t*)nullptr, 0u, n,
                                rocprim::plus<uint32_t>(), s);
    if (e != hipSuccess) return e;
    size_t lib_bytes = sort_bytes > scan64_bytes ? sort_bytes : scan64_bytes;
    if (scan32_bytes > lib_bytes) lib_bytes = scan32_bytes;
    lib_bytes = (lib_bytes + 255) & ~(size_t)255;
    const size_t total = 5 * n8 + 4 * n4 + 256 + lib_bytes;
    e = hipMalloc((void**)&tmp, total);
    if (e != hipSuccess) return e;
    uint64_t* keys_in = (uint64_t*)tmp;
    uint64_t* keys = keys_in + n;
    uint64_t* far_any = keys + n;
    uint64_t* far_dst = far_any + n;
    uint64_t* end_dst = far_dst + n;
    uint32_t* vals_in = (uint32_t*)(tmp + 5 * n8);
    uint32_t* vals = (uint32_t*)(tmp + 5 * n8 + n4);
    uint32_t* flag = (uint32_t*)(tmp + 5 * n8 + 2 * n4);
    uint32_t* pos = (uint32_t*)(tmp + 5 * n8 + 3 * n4);
    uint32_t* overlap = (uint32_t*)(tmp + 5 * n8 + 4 * n4);
    void* lib_tmp = tmp + 5 * n8 + 4 * n4 + 256;

    const uint32_t g = grid_for(n);
    hipLaunchKernelGGL(declare_clear_kernel, dim3(1), dim3(1), 0, s, overlap);
    hipLaunchKernelGGL(declare_keys_kernel, dim3(g), dim3(256), 0, s, dst_ext, n_dst, src_ext, check ? n_src : 0,
                       seg_base, keys_in, vals_in);
    size_t bytes = lib_bytes;
    e = rocprim::radix_sort_pairs(lib_tmp, bytes, keys_in, keys, vals_in, vals, n, 0, 64, s);
    if (e == hipSuccess && check) {
        uint64_t* end_any = keys_in;                       // keys_in is free after the sort
        hipLaunchKernelGGL(declare_ends_kernel, dim3(g), dim3(256), 0, s, dst_ext, n_dst, src_ext, n, keys, vals,
                           end_any, end_dst);
        bytes = lib_bytes;
        e = rocprim::exclusive_scan(lib_tmp, bytes, end_any, far_any, (uint64_t)0, n, MaxOp{}, s);
        bytes = lib_bytes;
        if (e == hipSuccess) e = rocprim::exclusive_scan(lib_tmp, bytes, end_dst, far_dst, (uint64_t)0, n, MaxOp{}, s);
        if (e == hipSuccess)
            hipLaunchKernelGGL(declare_check_kernel, dim3(g), dim3(256), 0, s, n_dst, n, keys, vals, far_any, far_dst, overlap);
    }
    if (e == hipSuccess) {
        hipLaunchKernelGGL(declare_is_dst_kernel, dim3(g), dim3(256), 0, s, n_dst, n, vals, flag);
        bytes = lib_bytes;
        e = rocprim::exclusive_scan(lib_tmp, bytes, flag, pos, 0u, n, rocprim::plus<uint32_t>(), s);
        if (e == hipSuccess)
            hipLaunchKernelGGL(declare_order_kernel, dim3(g), dim3(256), 0, s, n_dst, n, vals, pos, order_out, rank_out);
    }
    if (e == hipSuccess) e = hipGetLastError();
    if (e == hipSuccess) e = hipMemcpyAsync(overlap_out, overlap, sizeof(uint32_t), hipMemcpyDeviceToHost, s);
    hipError_t e2 = hipStreamSynchronize(s);
    (void)hipFree(tmp);
    return e != hipSuccess ? e : e2;
}

}  // namespace tent
