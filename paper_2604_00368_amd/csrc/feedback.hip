// Telemetry feedback: the bandwidth probe of Section 4.2 of the paper (Eq. 2, "peak picking") and
// the smoothed update of the rail bandwidth estimates, plus the rail simulator's slice latencies.
//
//   B_probe_d = min{ B_hw_d, max_i alpha * L_i / (tau_i - delta) }      over the window's slices on d
//   B_d      <- EWMA of the probes
//
// The window is the set of BOUND slices.  Per-rail maxima are integer, so the reduction order does
// not matter: every workgroup keeps 64 maxima in LDS (atomic max), then merges them into the
// batch's result block with one global atomic max per rail.
#include "tent_internal.h"

namespace tent {

// ceil(x * 1000 / bw) without overflow for x < 2^53: whole thousands first, then the remainder.
__device__ __forceinline__ uint64_t drain_ns(uint64_t x, uint32_t bw)
{
    const uint64_t whole = x / bw, rest = x - whole * bw;
    return whole * 1000 + (rest * 1000 + bw - 1) / bw;
}

__global__ void __launch_bounds__(256) sim_latency_kernel(BatchDev b, LatencyParams lp)
{
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < b.n_slices; i += stride) {
        if (b.s_state[i] != TENT_SLICE_BOUND) continue;
        const uint32_t d = b.s_rail[i];
        const uint64_t x = lp.queued[d] + b.s_stage_off[i] + b.s_len[i];
        b.s_tau[i] = lp.lat_ns[d] + drain_ns(x, lp.bw_MBps[d]);
    }
}

hipError_t launch_sim_latency(const BatchDev& b, const LatencyParams& lp, hipStream_t s)
{
    uint64_t blocks = (b.n_slices + 255) / 256;
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(sim_latency_kernel, dim3((uint32_t)blocks), dim3(256), 0, s, b, lp);
    return hipGetLastError();
}

__global__ void __launch_bounds__(64) probe_clear_kernel(BatchDev b)
{
    b.plan->peak[threadIdx.x] = 0;
}

__global__ void __launch_bounds__(256) probe_peak_kernel(BatchDev b, ProbeParams pp)
{
    __shared__ unsigned long long peak[TENT_MAX_RAILS];
    if (threadIdx.x < TENT_MAX_RAILS) peak[threadIdx.x] = 0;
    __syncthreads();
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < b.n_slices; i += stride) {
        if (b.s_state[i] != TENT_SLICE_BOUND) continue;
        const uint32_t d = b.s_rail[i];
        const tent_probe_params cal = pp.cal[d];
        const uint64_t tau = b.s_tau[i];
        uint64_t sample = cal.hw_MBps;                       // tau <= delta: no rate information
        if (tau > cal.delta_ns)
            sample = ((uint64_t)cal.alpha_q8 * b.s_len[i] * 1000ull) / (256ull * (tau - cal.delta_ns));
        atomicMax(&peak[d], (unsigned long long)sample + 1);  // stored +1 so that 0 means "no sample"
    }
    __syncthreads();
    if (threadIdx.x < TENT_MAX_RAILS && peak[threadIdx.x])
        atomicMax((unsigned long long*)&b.plan->peak[threadIdx.x], peak[threadIdx.x]);
}

// Cap by the hardware bandwidth and fold the probe into the estimate.
__global__ void __launch_bounds__(64) probe_update_kernel(BatchDev b, ProbeParams pp)
{
    const uint32_t d = threadIdx.x;
    uint32_t probe = 0, next = pp.bw_MBps[d];
    const uint64_t pk = b.plan->peak[d];
    if (d < pp.n_rails && pk) {
        const tent_probe_params cal = pp.cal[d];
        const uint64_t best = pk - 1;
        probe = (uint32_t)(best < cal.hw_MBps ? best : cal.hw_MBps);
        const uint64_t mixed = ((uint64_t)cal.ewma_q8 * probe + (uint64_t)(256 - cal.ewma_q8) * next) >> 8;
        next = (uint32_t)(mixed ? mixed : 1);
    }
    b.plan->probe[d] = probe;
    b.plan->bw_next[d] = next;
}

hipError_t launch_probe(const BatchDev& b, const ProbeParams& pp, hipStream_t s)
{
    hipLaunchKernelGGL(probe_clear_kernel, dim3(1), dim3(64), 0, s, b);
    uint64_t blocks = (b.n_slices + 255) / 256;
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(probe_peak_kernel, dim3((uint32_t)blocks), dim3(256), 0, s, b, pp);
    hipLaunchKernelGGL(probe_update_kernel, dim3(1), dim3(64), 0, s, b, pp);
    return hipGetLastError();
}

}  // namespace tent
