// Device-wide exclusive prefix scan over 64-bit integers for gfx950.
//
// Three launches: (1) every workgroup reduces its tile, (2) one workgroup scans the
// per-tile results, (3) every workgroup scans its tile again and combines with its tile's prefix.
// Inside a workgroup each lane owns kScanItems consecutive elements; lane totals are
// combined with a 64-wide wavefront scan and the wavefront totals are carried through LDS.
// The operator is any associative, commutative integer operation with identity 0 (sum by default,
// maximum for "furthest end seen so far").  The result does not depend on scheduling (a fixed
// tree of integer operations), and no workgroup ever waits on another one.
#pragma once

#include "tent_internal.h"

namespace tent {

struct ScanSum { __device__ __forceinline__ uint64_t operator()(uint64_t a, uint64_t b) const { return a + b; } };
struct ScanMax { __device__ __forceinline__ uint64_t operator()(uint64_t a, uint64_t b) const { return a > b ? a : b; } };

template <class Op>
__device__ __forceinline__ uint64_t wave_inclusive_scan(uint64_t v, Op op)
{
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        uint64_t up = __shfl_up((unsigned long long)v, d, 64);
        if (lane >= d) v = op(up, v);
    }
    return v;
}
__device__ __forceinline__ uint64_t wave_inclusive_scan(uint64_t v) { return wave_inclusive_scan(v, ScanSum{}); }

// Exclusive scan of one value per lane across a workgroup of kScanBlock lanes.
// Returns the lane's exclusive prefix; *block_total receives the result over the workgroup.
template <class Op>
__device__ __forceinline__ uint64_t block_exclusive_scan(uint64_t v, uint64_t* block_total, Op op)
{
    constexpr int kWaves = kScanBlock / 64;
    __shared__ uint64_t wave_sum[kWaves];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint64_t inc = wave_inclusive_scan(v, op);
    if (lane == 63) wave_sum[wave] = inc;
    __syncthreads();
    uint64_t carry = 0, total = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        uint64_t s = wave_sum[w];
        if (w < wave) carry = op(carry, s);
        total = op(total, s);
    }
    __syncthreads();
    *block_total = total;
    const uint64_t before = __shfl_up((unsigned long long)inc, 1, 64);   // inclusive result of the lane below
    return lane == 0 ? carry : op(carry, before);
}

template <class F, class Op>
__global__ void __launch_bounds__(kScanBlock) scan_reduce_kernel(F f, Op op, uint64_t n, uint64_t* partials)
{
    const uint64_t base = (uint64_t)blockIdx.x * kScanTile + (uint64_t)threadIdx.x * kScanItems;
    uint64_t sum = 0;
#pragma unroll
    for (int k = 0; k < (int)kScanItems; ++k)
        if (base + k < n) sum = op(sum, f(base + k));
    uint64_t total;
    block_exclusive_scan(sum, &total, op);
    if (threadIdx.x == 0) partials[blockIdx.x] = total;
}

// One workgroup: partials[0..nb) -> exclusive prefix in place, partials[nb] = grand total.
// (internal linkage: the same instantiation exists in several translation units, each with its own code object)
template <class Op>
static __global__ void __launch_bounds__(kScanBlock) scan_spine_kernel(Op op, uint64_t* partials, uint64_t nb)
{
    uint64_t carry = 0;
    for (uint64_t lo = 0; lo < nb; lo += kScanBlock) {
        uint64_t i = lo + threadIdx.x;
        uint64_t v = i < nb ? partials[i] : 0;
        uint64_t total;
        uint64_t ex = block_exclusive_scan(v, &total, op);
        if (i < nb) partials[i] = op(carry, ex);
        carry = op(carry, total);
    }
    if (threadIdx.x == 0) partials[nb] = carry;
}

template <class F, class Op>
__global__ void __launch_bounds__(kScanBlock) scan_down_kernel(F f, Op op, uint64_t n, const uint64_t* partials,
                                                              uint64_t* out)
{
    const uint64_t base = (uint64_t)blockIdx.x * kScanTile + (uint64_t)threadIdx.x * kScanItems;
    uint64_t v[kScanItems];
    uint64_t sum = 0;
#pragma unroll
    for (int k = 0; k < (int)kScanItems; ++k) {
        v[k] = base + k < n ? f(base + k) : 0;
        sum = op(sum, v[k]);
    }
    uint64_t total;
    uint64_t run = op(partials[blockIdx.x], block_exclusive_scan(sum, &total, op));
#pragma unroll
    for (int k = 0; k < (int)kScanItems; ++k) {
        if (base + k < n) out[base + k] = run;
        run = op(run, v[k]);
    }
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == kScanBlock - 1) out[n] = run;   // grand total
}

// out[i] = op over f(0..i-1) for i in [0, n] (out has n + 1 entries); partials needs
// scan_partials_capacity(n) entries.
template <class F, class Op = ScanSum>
hipError_t exclusive_scan(F f, uint64_t n, uint64_t* out, uint64_t* partials, hipStream_t s, Op op = Op{})
{
    if (n == 0) return hipErrorInvalidValue;
    const uint64_t nb = (n + kScanTile - 1) / kScanTile;
    if (nb > 0x7FFFFFFFull) return hipErrorInvalidValue;
    hipLaunchKernelGGL((scan_reduce_kernel<F, Op>), dim3((uint32_t)nb), dim3(kScanBlock), 0, s, f, op, n, partials);
    hipLaunchKernelGGL((scan_spine_kernel<Op>), dim3(1), dim3(kScanBlock), 0, s, op, partials, nb);
    hipLaunchKernelGGL((scan_down_kernel<F, Op>), dim3((uint32_t)nb), dim3(kScanBlock), 0, s, f, op, n, partials, out);
    return hipGetLastError();
}

}  // namespace tent
