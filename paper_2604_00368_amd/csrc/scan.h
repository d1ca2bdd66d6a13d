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

// Two independent sum scans in the same three launches (a launch of a small kernel costs more than its
// work): out1[i] = sum f1(0..i-1) for i in [0, n1], out2 likewise over n2; partials1 and partials2 each
// need scan_partials_capacity(max(n1, n2)) entries.
template <class F1, class F2>
__global__ void __launch_bounds__(kScanBlock) scan_reduce2_kernel(F1 f1, F2 f2, uint64_t n1, uint64_t n2,
                                                                 uint64_t* partials1, uint64_t* partials2)
{
    const uint64_t base = (uint64_t)blockIdx.x * kScanTile + (uint64_t)threadIdx.x * kScanItems;
    uint64_t sum1 = 0, sum2 = 0;
#pragma unroll
    for (int k = 0; k < (int)kScanItems; ++k) {
        if (base + k < n1) sum1 += f1(base + k);
        if (base + k < n2) sum2 += f2(base + k);
    }
    uint64_t total1, total2;
    block_exclusive_scan(sum1, &total1, ScanSum{});
    block_exclusive_scan(sum2, &total2, ScanSum{});
    if (threadIdx.x == 0) { partials1[blockIdx.x] = total1; partials2[blockIdx.x] = total2; }
}

// (a template for the same reason as scan_spine_kernel: internal linkage without an unused-function warning)
template <class Op>
static __global__ void __launch_bounds__(kScanBlock) scan_spine2_kernel(Op, uint64_t* partials1, uint64_t* partials2, uint64_t nb)
{
    uint64_t carry1 = 0, carry2 = 0;
    for (uint64_t lo = 0; lo < nb; lo += kScanBlock) {
        const uint64_t i = lo + threadIdx.x;
        uint64_t total1, total2;
        const uint64_t ex1 = block_exclusive_scan(i < nb ? partials1[i] : 0, &total1, ScanSum{});
        const uint64_t ex2 = block_exclusive_scan(i < nb ? partials2[i] : 0, &total2, ScanSum{});
        if (i < nb) { partials1[i] = carry1 + ex1; partials2[i] = carry2 + ex2; }
        carry1 += total1;
        carry2 += total2;
    }
    if (threadIdx.x == 0) { partials1[nb] = carry1; partials2[nb] = carry2; }
}

template <class F1, class F2>
__global__ void __launch_bounds__(kScanBlock) scan_down2_kernel(F1 f1, F2 f2, uint64_t n1, uint64_t n2,
                                                               const uint64_t* partials1, const uint64_t* partials2,
                                                               uint64_t* out1, uint64_t* out2)
{
    const uint64_t base = (uint64_t)blockIdx.x * kScanTile + (uint64_t)threadIdx.x * kScanItems;
    uint64_t v1[kScanItems], v2[kScanItems];
    uint64_t sum1 = 0, sum2 = 0;
#pragma unroll
    for (int k = 0; k < (int)kScanItems; ++k) {
        v1[k] = base + k < n1 ? f1(base + k) : 0;
        v2[k] = base + k < n2 ? f2(base + k) : 0;
        sum1 += v1[k];
        sum2 += v2[k];
    }
    uint64_t total1, total2;
    uint64_t run1 = partials1[blockIdx.x] + block_exclusive_scan(sum1, &total1, ScanSum{});
    uint64_t run2 = partials2[blockIdx.x] + block_exclusive_scan(sum2, &total2, ScanSum{});
    // entry n of either output is its grand total: it is written by the lane that reaches index n
#pragma unroll
    for (int k = 0; k < (int)kScanItems; ++k) {
        if (base + k <= n1) out1[base + k] = run1;
        if (base + k <= n2) out2[base + k] = run2;
        run1 += v1[k];
        run2 += v2[k];
    }
    if (base + kScanItems == n1) out1[n1] = run1;
    if (base + kScanItems == n2) out2[n2] = run2;
}

template <class F1, class F2>
hipError_t exclusive_scan2(F1 f1, F2 f2, uint64_t n1, uint64_t n2, uint64_t* out1, uint64_t* out2, uint64_t* partials1,
                           uint64_t* partials2, hipStream_t s)
{
    if (n1 == 0 || n2 == 0) return hipErrorInvalidValue;
    const uint64_t n = n1 > n2 ? n1 : n2;
    const uint64_t nb = (n + kScanTile - 1) / kScanTile;
    if (nb > 0x7FFFFFFFull) return hipErrorInvalidValue;
    hipLaunchKernelGGL((scan_reduce2_kernel<F1, F2>), dim3((uint32_t)nb), dim3(kScanBlock), 0, s, f1, f2, n1, n2, partials1, partials2);
    hipLaunchKernelGGL((scan_spine2_kernel<ScanSum>), dim3(1), dim3(kScanBlock), 0, s, ScanSum{}, partials1, partials2, nb);
    hipLaunchKernelGGL((scan_down2_kernel<F1, F2>), dim3((uint32_t)nb), dim3(kScanBlock), 0, s, f1, f2, n1, n2, partials1, partials2,
                       out1, out2);
    return hipGetLastError();
}

}  // namespace tent
