// Retry rotation (Section 4.3, "Link-Level Resilience") and failure marking of the rail simulator.
//
// A slice that failed on a rail is not bound by predicted cost again: slice i on its k-th retry
// takes candidate number (i + k) mod |candidates| of the rotation order the host derived from the
// rails' health, the retried slices are issued ahead of everything else in ascending slice index,
// and their bytes count in the queue statistics the cost model then starts from.  The rail of a
// retried slice is therefore a pure function of (i, k); what needs work is its staging offset, the
// bytes of the earlier retried slices on the same rail -- one prefix sum per rail over the retry
// list.  Three launches: per-chunk byte and slice counts per rail, an exclusive scan of those
// over the chunks (one lane per rail), and the in-order walk of every chunk by one wavefront.
#include "tent_internal.h"

namespace tent {
namespace {

__device__ __forceinline__ uint64_t lane_read64(uint64_t v, int lane)
{
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, lane);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), lane);
    return ((uint64_t)hi << 32) | lo;
}

__device__ __forceinline__ uint32_t rotation_rail(const RotateParams& rot, uint32_t id, uint32_t retry)
{
    return rot.cand[((uint64_t)id + retry) % rot.n_cand];
}

// Step 1: bytes and slices per (chunk, rail).  Integer sums: the order of the atomics is immaterial.
__global__ void __launch_bounds__(64) rotate_count_kernel(BatchDev b, RotateParams rot)
{
    __shared__ unsigned long long bytes[TENT_MAX_RAILS];
    __shared__ uint32_t cnt[TENT_MAX_RAILS];
    const uint64_t n = b.plan->n_retry;
    const uint64_t begin = (uint64_t)blockIdx.x * kRotChunk;
    if (begin >= n) return;
    bytes[threadIdx.x] = 0;
    cnt[threadIdx.x] = 0;
    __syncthreads();
    const uint64_t end = begin + kRotChunk < n ? begin + kRotChunk : n;
    for (uint64_t q = begin + threadIdx.x; q < end; q += 64) {
        const uint32_t id = b.retry_ids[q];
        const uint32_t d = rotation_rail(rot, id, b.s_retry[id]);
        atomicAdd(&bytes[d], (unsigned long long)b.s_len[id]);
        atomicAdd(&cnt[d], 1u);
    }
    __syncthreads();
    b.rot_bytes[(uint64_t)blockIdx.x * TENT_MAX_RAILS + threadIdx.x] = bytes[threadIdx.x];
    b.rot_cnt[(uint64_t)blockIdx.x * TENT_MAX_RAILS + threadIdx.x] = cnt[threadIdx.x];
}

// Step 2: lane d turns rail d's per-chunk byte counts into their exclusive prefix and publishes
// the totals of the rotation pass.
__global__ void __launch_bounds__(64) rotate_spine_kernel(BatchDev b)
{
    const uint64_t n = b.plan->n_retry;
    const uint64_t chunks = (n + kRotChunk - 1) / kRotChunk;
    uint64_t run = 0, slices = 0;
    for (uint64_t c = 0; c < chunks; ++c) {
        const uint64_t at = c * TENT_MAX_RAILS + threadIdx.x;
        const uint64_t t = b.rot_bytes[at];
        b.rot_bytes[at] = run;
        run += t;
        slices += b.rot_cnt[at];
    }
    b.plan->Tr[threadIdx.x] = run;
    b.plan->cr[threadIdx.x] = slices;
}

// Step 3: one wavefront walks its chunk in order, 64 retried slices at a time.  Lane d keeps the
// running byte count of rail d; for every rail present among the 64 slices a wave-wide inclusive
// scan over the lengths of that rail's slices gives each its offset.
__global__ void __launch_bounds__(64) rotate_emit_kernel(BatchDev b, RotateParams rot)
{
    const uint64_t n = b.plan->n_retry;
    const uint64_t begin = (uint64_t)blockIdx.x * kRotChunk;
    if (begin >= n) return;
    const int lane = threadIdx.x;
    uint64_t my_base = b.rot_bytes[(uint64_t)blockIdx.x * TENT_MAX_RAILS + lane];
    const uint64_t end = begin + kRotChunk < n ? begin + kRotChunk : n;
    for (uint64_t blk = begin; blk < end; blk += 64) {
        const uint64_t q = blk + lane;
        const bool valid = q < end;
        uint32_t id = 0, len = 0, d = 0;
        if (valid) {
            id = b.retry_ids[q];
            len = b.s_len[id];
            d = rotation_rail(rot, id, b.s_retry[id]);
        }
        uint64_t off = 0;
        uint64_t todo = __ballot(valid);
        while (todo) {                                           // one round per rail present in the block
            const int leader = __ffsll((long long)todo) - 1;
            const uint32_t r = (uint32_t)__builtin_amdgcn_readlane((int)d, leader);
            const bool mine = valid && d == r;
            uint64_t incl = mine ? len : 0;
#pragma unroll
            for (int step = 1; step < 64; step <<= 1) {
                const uint64_t up = (uint64_t)__shfl_up((unsigned long long)incl, step, 64);
                if (lane >= step) incl += up;
            }
            const uint64_t base_r = lane_read64(my_base, (int)r);
            if (mine) off = base_r + incl - len;
            const uint64_t total = lane_read64(incl, 63);
            if (lane == (int)r) my_base += total;
            todo &= ~__ballot(mine);
        }
        if (valid) {
            b.s_rail[id] = d;
            b.s_stage_off[id] = off;
            b.s_state[id] = TENT_SLICE_BOUND;
        }
    }
}

// Rail simulator: every BOUND slice on a failed rail returns to the pending set with one more retry.
__global__ void __launch_bounds__(256) fail_kernel(BatchDev b, FailParams fp)
{
    __shared__ uint32_t cnt[TENT_MAX_RAILS];
    if (threadIdx.x < TENT_MAX_RAILS) cnt[threadIdx.x] = 0;
    __syncthreads();
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < b.n_slices; i += stride) {
        if (b.s_state[i] != TENT_SLICE_BOUND) continue;
        const uint32_t d = b.s_rail[i];
        if (d >= TENT_MAX_RAILS || !fp.failed[d]) continue;
        b.s_state[i] = TENT_SLICE_PENDING;
        const uint8_t k = b.s_retry[i];
        if (k < 255) b.s_retry[i] = (uint8_t)(k + 1);
        atomicAdd(&cnt[d], 1u);
    }
    __syncthreads();
    if (threadIdx.x < TENT_MAX_RAILS && cnt[threadIdx.x])
        atomicAdd((unsigned long long*)&b.plan->fail_cnt[threadIdx.x], (unsigned long long)cnt[threadIdx.x]);
}

__global__ void __launch_bounds__(64) fail_clear_kernel(BatchDev b) { b.plan->fail_cnt[threadIdx.x] = 0; }

}  // namespace

hipError_t launch_rotate(const BatchDev& b, const RotateParams& rot, hipStream_t s)
{
    if (rot.n_cand == 0 || rot.n_cand > TENT_MAX_RAILS) return hipErrorInvalidValue;
    const uint64_t chunks = (b.n_slices + kRotChunk - 1) / kRotChunk;          // upper bound; idle chunks exit at once
    if (chunks == 0 || chunks > 0x7FFFFFFFull) return hipErrorInvalidValue;
    hipLaunchKernelGGL(rotate_count_kernel, dim3((uint32_t)chunks), dim3(64), 0, s, b, rot);
    hipLaunchKernelGGL(rotate_spine_kernel, dim3(1), dim3(64), 0, s, b);
    hipLaunchKernelGGL(rotate_emit_kernel, dim3((uint32_t)chunks), dim3(64), 0, s, b, rot);
    return hipGetLastError();
}

hipError_t launch_fail(const BatchDev& b, const FailParams& fp, hipStream_t s)
{
    hipLaunchKernelGGL(fail_clear_kernel, dim3(1), dim3(64), 0, s, b);
    uint64_t blocks = (b.n_slices + 255) / 256;
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(fail_kernel, dim3((uint32_t)blocks), dim3(256), 0, s, b, fp);
    return hipGetLastError();
}

}  // namespace tent
