// Device-wide exclusive prefix sum over 64-bit integers for gfx950.
//
// Three launches: (1) every workgroup reduces its tile, (2) one workgroup scans the
// per-tile sums, (3) every workgroup scans its tile again and adds its tile's offset.
// Inside a workgroup each lane owns kScanItems consecutive elements; lane totals are
// combined with a 64-wide wavefront scan and the wavefront totals are carried through LDS.
// The result does not depend on scheduling (integer adds in a fixed tree), and no
// workgroup ever waits on another one.
#pragma once

#include "tent_internal.h"

namespace tent {

__device__ __forceinline__ uint64_t wave_inclusive_scan(uint64_t v)
{
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        uint64_t up = __shfl_up((unsigned long long)v, d, 64);
        if (lane >= d) v += up;
    }
    return v;
}

// Exclusive scan of one value per lane across a workgroup of kScanBlock lanes.
// Returns the lane's exclusive prefix; *block_total receives the sum over the workgroup.
__device__ __forceinline__ uint64_t block_exclusive_scan(uint64_t v, uint64_t* block_total)
{
    constexpr int kWaves = kScanBlock / 64;
    __shared__ uint64_t wave_sum[kWaves];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint64_t inc = wave_inclusive_scan(v);
    if (lane == 63) wave_sum[wave] = inc;
    __syncthreads();
    uint64_t carry = 0, total = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        uint64_t s = wave_sum[w];
        if (w < wave) carry += s;
        total += s;
    }
    __syncthreads();
    *block_total = total;
    return carry + inc - v;
}

template <class F>
__global__ void __launch_bounds__(kScanBlock) scan_reduce_kernel(F f, uint64_t n, uint64_t* partials)
{
    const uint64_t base = (uint64_t)blockIdx.x * kScanTile + (uint64_t)threadIdx.x * kScanItems;
    uint64_t sum = 0;
#pragma unroll
    for (int k = 0; k < (int)kScanItems; ++k)
        if (base + k < n) sum += f(base + k);
    uint64_t total;
    block_exclusive_scan(sum, &total);
    if (threadIdx.x == 0) partials[blockIdx.x] = total;
}

// One workgroup: partials[0..nb) -> exclusive prefix in place, partials[nb] = grand total.
static __global__ void __launch_bounds__(kScanBlock) scan_spine_kernel(uint64_t* partials, uint64_t nb)
{
    uint64_t carry = 0;
    for (uint64_t lo = 0; lo < nb; lo += kScanBlock) {
        uint64_t i = lo + threadIdx.x;
        uint64_t v = i < nb ? partials[i] : 0;
        uint64_t total;
        uint64_t ex = block_exclusive_scan(v, &total);
        if (i < nb) partials[i] = carry + ex;
        carry += total;
    }
    if (threadIdx.x == 0) partials[nb] = carry;
}

template <class F>
__global__ void __launch_bounds__(kScanBlock) scan_down_kernel(F f, uint64_t n, const uint64_t* partials,
                                                              uint64_t* out)
{
    const uint64_t base = (uint64_t)blockIdx.x * kScanTile + (uint64_t)threadIdx.x * kScanItems;
    uint64_t v[kScanItems];
    uint64_t sum = 0;
#pragma unroll
    for (int k = 0; k < (int)kScanItems; ++k) {
        v[k] = base + k < n ? f(base + k) : 0;
        sum += v[k];
    }
    uint64_t total;
    uint64_t run = partials[blockIdx.x] + block_exclusive_scan(sum, &total);
#pragma unroll
    for (int k = 0; k < (int)kScanItems; ++k) {
        if (base + k < n) out[base + k] = run;
        run += v[k];
    }
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == kScanBlock - 1) out[n] = run;   // grand total
}

// out[i] = sum of f(0..i-1) for i in [0, n]; partials needs scan_partials_capacity(n) entries.
template <class F>
hipError_t exclusive_scan(F f, uint64_t n, uint64_t* out, uint64_t* partials, hipStream_t s)
{
    if (n == 0) return hipErrorInvalidValue;
    const uint64_t nb = (n + kScanTile - 1) / kScanTile;
    hipLaunchKernelGGL(scan_reduce_kernel<F>, dim3((uint32_t)nb), dim3(kScanBlock), 0, s, f, n, partials);
    hipLaunchKernelGGL(scan_spine_kernel, dim3(1), dim3(kScanBlock), 0, s, partials, nb);
    hipLaunchKernelGGL(scan_down_kernel<F>, dim3((uint32_t)nb), dim3(kScanBlock), 0, s, f, n, partials, out);
    return hipGetLastError();
}

}  // namespace tent
