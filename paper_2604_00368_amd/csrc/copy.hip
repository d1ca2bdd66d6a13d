// Gather / scatter of slice bytes between paged extents and per-rail staging regions.
//
// Gather: slice bytes are read from the transfer's source extents (the paged side) and written
// contiguously at arena + base[rail] + stage_off (the staging hop of Section 4.1 of the paper).
// Scatter: the same bytes are read back from staging and written to the destination extents at
// the slice's absolute offset inside the transfer (direct-to-offset writes, Section 4.4), so the
// result does not depend on the order in which slices are moved.
//
// Work decomposition: a work item is (slice, chunk) with chunk_bytes of the slice; one 256-lane
// workgroup walks the extents that intersect its chunk and copies each intersection ("piece")
// cooperatively.  When the two addresses and the length of a piece are multiples of 16 the piece
// moves as 16-byte-per-lane vectors, kUnroll loads in flight per lane before the first store;
// otherwise head/tail bytes are peeled when both sides share their alignment, and fully
// misaligned pieces move byte by byte.  All per-item bookkeeping is uniform across the workgroup.
#include "tent_internal.h"

namespace tent {

typedef uint32_t vec4u __attribute__((ext_vector_type(4)));

constexpr int kCopyBlock = 256;
constexpr int kUnroll = 8;

__device__ __forceinline__ void copy_vectors(vec4u* __restrict__ dst, const vec4u* __restrict__ src, uint64_t nvec)
{
    for (uint64_t base = 0; base < nvec; base += (uint64_t)kCopyBlock * kUnroll) {
        vec4u r[kUnroll];
#pragma unroll
        for (int k = 0; k < kUnroll; ++k) {
            const uint64_t idx = base + (uint64_t)k * kCopyBlock + threadIdx.x;
            if (idx < nvec) r[k] = __builtin_nontemporal_load(src + idx);
        }
#pragma unroll
        for (int k = 0; k < kUnroll; ++k) {
            const uint64_t idx = base + (uint64_t)k * kCopyBlock + threadIdx.x;
            if (idx < nvec) __builtin_nontemporal_store(r[k], dst + idx);
        }
    }
}

__device__ __forceinline__ void copy_bytes(uint8_t* __restrict__ dst, const uint8_t* __restrict__ src, uint64_t n)
{
    for (uint64_t x = threadIdx.x; x < n; x += kCopyBlock) dst[x] = src[x];
}

__device__ __forceinline__ void copy_piece(uint8_t* dst, const uint8_t* src, uint64_t n)
{
    const uint64_t d = (uint64_t)dst, s = (uint64_t)src;
    if (((d | s | n) & 15) == 0) {
        copy_vectors((vec4u*)dst, (const vec4u*)src, n >> 4);
    } else if (((d ^ s) & 15) == 0) {
        uint64_t head = (16 - (d & 15)) & 15;
        if (head > n) head = n;
        copy_bytes(dst, src, head);
        const uint64_t body = (n - head) & ~15ull;
        copy_vectors((vec4u*)(dst + head), (const vec4u*)(src + head), body >> 4);
        copy_bytes(dst + head + body, src + head + body, n - head - body);
    } else {
        copy_bytes(dst, src, n);
    }
}

__device__ __forceinline__ uint32_t last_not_above32(const uint64_t* a, uint32_t lo, uint32_t hi, uint64_t key)
{
    while (hi - lo > 1) {
        uint32_t mid = lo + ((hi - lo) >> 1);
        if (a[mid] <= key) lo = mid; else hi = mid;
    }
    return lo;
}

template <bool kGather>
__global__ void __launch_bounds__(kCopyBlock) copy_kernel(BatchDev b, uint8_t* arena, uint32_t chunk_bytes,
                                                          uint32_t chunks_per_slice)
{
    const uint64_t items = b.n_slices * chunks_per_slice;
    const uint32_t*    ptr = kGather ? b.src_ptr : b.dst_ptr;
    const tent_extent* ext = kGather ? b.src_ext : b.dst_ext;
    const uint64_t*    pre = kGather ? b.src_pre : b.dst_pre;
    const uint32_t*    e0s = kGather ? b.s_src_e0 : b.s_dst_e0;

    for (uint64_t item = blockIdx.x; item < items; item += gridDim.x) {
        const uint64_t i = item / chunks_per_slice;
        const uint32_t c = (uint32_t)(item - i * chunks_per_slice);
        if (b.s_state[i] != TENT_SLICE_BOUND) continue;
        const uint32_t len = b.s_len[i];
        const uint64_t lo = (uint64_t)c * chunk_bytes;
        if (lo >= len) continue;
        const uint64_t hi = lo + chunk_bytes < len ? lo + chunk_bytes : len;

        const uint32_t j = b.s_desc[i];
        const uint32_t e_lo = ptr[j], e_hi = ptr[j + 1];
        uint64_t pos = pre[e_lo] + b.s_off[i] + lo;          // position in the batch-wide extent prefix
        const uint64_t end = pos + (hi - lo);
        uint8_t* linear = arena + b.plan->base[b.s_rail[i]] + b.s_stage_off[i] + lo;
        uint32_t e = last_not_above32(pre, e0s[i], e_hi, pos);
        while (pos < end) {
            const uint64_t e_end = pre[e + 1];
            const uint64_t n = (e_end < end ? e_end : end) - pos;
            const tent_extent x = ext[e];
            uint8_t* paged = (uint8_t*)(b.seg_base[x.seg] + x.off + (pos - pre[e]));
            if (kGather) copy_piece(linear, paged, n); else copy_piece(paged, linear, n);
            linear += n;
            pos += n;
            ++e;
        }
    }
}

static void copy_geometry(const BatchDev& b, uint32_t chunk_bytes, uint32_t grid_cap,
                          uint32_t* chunk, uint32_t* cps, uint32_t* grid)
{
    uint64_t cb = chunk_bytes ? chunk_bytes : 64u * 1024u;
    if (cb > b.slice_bytes) cb = b.slice_bytes;
    if (cb > 0xFFFFFFFFull) cb = 0x80000000ull;
    uint64_t per = (b.slice_bytes + cb - 1) / cb;
    uint64_t items = b.n_slices * per;
    uint64_t cap = grid_cap ? grid_cap : 0x7FFFFFFFull;
    *chunk = (uint32_t)cb;
    *cps = (uint32_t)per;
    *grid = (uint32_t)(items < cap ? items : cap);
}

hipError_t launch_copy(const BatchDev& b, uint8_t* arena, bool gather, uint32_t chunk_bytes, uint32_t grid_cap,
                       hipStream_t s)
{
    uint32_t chunk, cps, grid;
    copy_geometry(b, chunk_bytes, grid_cap, &chunk, &cps, &grid);
    if (grid == 0) return hipSuccess;
    if (gather)
        hipLaunchKernelGGL(copy_kernel<true>, dim3(grid), dim3(kCopyBlock), 0, s, b, arena, chunk, cps);
    else
        hipLaunchKernelGGL(copy_kernel<false>, dim3(grid), dim3(kCopyBlock), 0, s, b, arena, chunk, cps);
    return hipGetLastError();
}

}  // namespace tent
