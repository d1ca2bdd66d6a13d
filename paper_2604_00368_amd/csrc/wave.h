// Cross-lane helpers for the one-wavefront chain kernels (lane = rail): all-reduces built from DPP
// row operations, and argmin / argmax over (cost, lane) pairs.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tent {

template <int kCtrl>
__device__ __forceinline__ uint32_t dpp32(uint32_t v)
{
    // every control used below gives each lane a valid source lane, so no fill value is needed
    return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, kCtrl, 0xF, 0xF, true);
}
template <int kCtrl>
__device__ __forceinline__ uint64_t dpp64(uint64_t v)
{
    return ((uint64_t)dpp32<kCtrl>((uint32_t)(v >> 32)) << 32) | dpp32<kCtrl>((uint32_t)v);
}
__device__ __forceinline__ uint64_t xor64(uint64_t v, int mask)
{
    return (uint64_t)__shfl_xor((unsigned long long)v, mask, 64);
}

// All-reduce over the wavefront with a symmetric butterfly (quad swaps, half-row mirror, row mirror,
// then rows), so every lane ends with the same value.  `wide` > 16 / > 32 enables the row steps.
template <class Op>
__device__ __forceinline__ uint64_t wave_reduce64(uint64_t v, int wide, Op op)
{
    v = op(v, dpp64<0xB1>(v));
    v = op(v, dpp64<0x4E>(v));
    v = op(v, dpp64<0x141>(v));
    v = op(v, dpp64<0x140>(v));
    if (wide > 16) v = op(v, xor64(v, 16));
    if (wide > 32) v = op(v, xor64(v, 32));
    return v;
}
struct OpMin { __device__ uint64_t operator()(uint64_t a, uint64_t b) const { return a < b ? a : b; } };
struct OpMax { __device__ uint64_t operator()(uint64_t a, uint64_t b) const { return a > b ? a : b; } };
struct OpAdd { __device__ uint64_t operator()(uint64_t a, uint64_t b) const { return a + b; } };
struct OpAddF {
    __device__ uint64_t operator()(uint64_t a, uint64_t b) const
    {
        return (uint64_t)__double_as_longlong(__longlong_as_double((long long)a) + __longlong_as_double((long long)b));
    }
};
__device__ __forceinline__ double wave_sum_f64(double x, int wide)
{
    return __longlong_as_double((long long)wave_reduce64((uint64_t)__double_as_longlong(x), wide, OpAddF{}));
}
__device__ __forceinline__ uint64_t uniform64(uint64_t v)
{
    uint32_t lo = __builtin_amdgcn_readfirstlane((int)(uint32_t)v);
    uint32_t hi = __builtin_amdgcn_readfirstlane((int)(uint32_t)(v >> 32));
    return ((uint64_t)hi << 32) | lo;
}
__device__ __forceinline__ uint64_t read_lane64(uint64_t v, int lane)
{
    uint32_t lo = __builtin_amdgcn_readlane((int)(uint32_t)v, lane);
    uint32_t hi = __builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), lane);
    return ((uint64_t)hi << 32) | lo;
}


// 32-bit all-reduce over the wavefront; the DPP moves fold into the min/max/add instructions.
template <class Op>
__device__ __forceinline__ uint32_t wave_reduce32(uint32_t v, int wide, Op op)
{
    v = op(v, dpp32<0xB1>(v));
    v = op(v, dpp32<0x4E>(v));
    v = op(v, dpp32<0x141>(v));
    v = op(v, dpp32<0x140>(v));
    if (wide > 16) v = op(v, (uint32_t)__shfl_xor((int)v, 16, 64));
    if (wide > 32) v = op(v, (uint32_t)__shfl_xor((int)v, 32, 64));
    return v;
}
struct Min32 { __device__ uint32_t operator()(uint32_t a, uint32_t b) const { return a < b ? a : b; } };
struct Max32 { __device__ uint32_t operator()(uint32_t a, uint32_t b) const { return a > b ? a : b; } };
struct Add32 { __device__ uint32_t operator()(uint32_t a, uint32_t b) const { return a + b; } };

// Lane holding the smallest (cost, lane) pair among the lanes with valid = true (ties to the lowest
// lane), as a uniform value.  The 64-bit key (cost << 6) | lane is reduced as two 32-bit halves:
// first the high half, then the low half among the lanes that match the winning high half.
__device__ __forceinline__ int argmin_cost(uint64_t cost, bool valid, int lane, int wide)
{
    const uint32_t hi = valid ? (uint32_t)(cost >> 26) : 0xFFFFFFFFu;
    const uint32_t lo = ((uint32_t)cost << 6) | (uint32_t)lane;
    const uint32_t hi_min = wave_reduce32(hi, wide, Min32{});
    const uint32_t lo_min = wave_reduce32(hi == hi_min && valid ? lo : 0xFFFFFFFFu, wide, Min32{});
    return (int)(__builtin_amdgcn_readfirstlane((int)lo_min) & 63);
}
// Same for the largest (cost, lane) pair (ties to the highest lane).
__device__ __forceinline__ int argmax_cost(uint64_t cost, bool valid, int lane, int wide)
{
    const uint32_t hi = valid ? (uint32_t)(cost >> 26) : 0u;
    const uint32_t lo = ((uint32_t)cost << 6) | (uint32_t)lane;
    const uint32_t hi_max = wave_reduce32(hi, wide, Max32{});
    const uint32_t lo_max = wave_reduce32(hi == hi_max && valid ? lo : 0u, wide, Max32{});
    return (int)(__builtin_amdgcn_readfirstlane((int)lo_max) & 63);
}

}  // namespace tent
