// Byte-exact movement of a range of one slice between its extents (the paged side) and a linear
// address, for geometry in which extent boundaries fall anywhere: used by the copy kernels where a
// tile crosses an extent boundary or a slice ends inside a lane's vector, and by the bounded
// staging path for lengths that are no multiple of the tile size.
#pragma once

#include "tent_internal.h"

namespace tent {

typedef uint32_t vec4u __attribute__((ext_vector_type(4)));
// 16-byte vector at any address: gfx950 global loads and stores need no alignment, and the compiler
// emits a single dwordx4 access for this type.
typedef vec4u vec4u_any __attribute__((aligned(1)));
// The same vector behind a pointer that is known to be device memory: addresses taken from tables are
// plain integers, and without the address space the compiler must emit generic (flat) accesses.
typedef __attribute__((address_space(1))) vec4u_any vec4u_dev;

// Wavefront-cooperative byte copy (64 lanes).
__device__ __forceinline__ void copy_bytes(uint8_t* __restrict__ dst, const uint8_t* __restrict__ src, uint64_t n)
{
    for (uint64_t x = threadIdx.x & 63; x < n; x += 64) dst[x] = src[x];
}

// Wavefront-cooperative copy of n bytes, any alignment: bytes up to the first 16-byte boundary of
// the destination, then aligned 16-byte stores fed by 16-byte loads at whatever alignment the
// source has (gfx950 global loads need no alignment), then the remaining bytes.
__device__ __forceinline__ void copy_piece(uint8_t* dst, const uint8_t* src, uint64_t n)
{
    uint64_t head = (16 - ((uint64_t)dst & 15)) & 15;
    if (head > n) head = n;
    copy_bytes(dst, src, head);
    const uint64_t nvec = (n - head) >> 4;
    vec4u* dv = (vec4u*)(dst + head);
    const uint8_t* sb = src + head;
    for (uint64_t v = threadIdx.x & 63; v < nvec; v += 64) {
        vec4u x;
        __builtin_memcpy(&x, sb + (v << 4), 16);
        dv[v] = x;
    }
    const uint64_t done = head + (nvec << 4);
    copy_bytes(dst + done, src + done, n - done);
}

__device__ __forceinline__ uint32_t last_not_above32(const uint64_t* a, uint32_t lo, uint32_t hi, uint64_t key)
{
    while (hi - lo > 1) {
        uint32_t mid = lo + ((hi - lo) >> 1);
        if (a[mid] <= key) lo = mid; else hi = mid;
    }
    return lo;
}

// Generic path for one wavefront: bytes [lo, hi) of slice i, walking the extents that intersect the range.
template <bool kGather>
__device__ __forceinline__ void copy_range_generic(const BatchDev& b, uint64_t i, uint64_t lo, uint64_t hi, uint8_t* linear)
{
    const uint32_t*    ptr = kGather ? b.src_ptr : b.dst_ptr;
    const tent_extent* ext = kGather ? b.src_ext : b.dst_ext;
    const uint64_t*    pre = kGather ? b.src_pre : b.dst_pre;
    const uint32_t     e0  = kGather ? b.s_src_e0[i] : b.s_dst_e0[i];
    const uint32_t j = b.s_desc[i];
    const uint32_t e_lo = ptr[j], e_hi = ptr[j + 1];
    uint64_t pos = pre[e_lo] + b.s_off[i] + lo;              // position in the batch-wide extent prefix
    const uint64_t end = pos + (hi - lo);
    uint32_t e = last_not_above32(pre, e0, e_hi, pos);
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

}  // namespace tent
