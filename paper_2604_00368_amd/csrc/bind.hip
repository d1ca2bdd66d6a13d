// Rail assignment, slice by slice (Algorithm 1, Stage 2 of the paper with the per-slice
// earliest-completion rule of Section 4.2): for every pending slice in ascending index the
// admitted rail with the smallest predicted completion cost
//     c0_d + (((A_d + len) * c1_d) >> 16)          (Eq. 1 scaled by the topology penalty)
// wins, ties going to the lowest rail index; the winner's in-flight bytes A_d grow by len, and
// the slice's staging offset is the number of bytes bound to that rail before it.
//
// The binding of slice i depends on all earlier bindings, so this kernel is a dependency chain:
// one wavefront, lane d holds rail d's state in registers, and every slice costs one multiply-add,
// a cross-lane minimum over 64-bit keys and a predicated update.  Slice lengths are fetched 64 at a
// time (one per lane, next block prefetched) and results leave in coalesced 64-wide stores.
#include "tent_internal.h"

namespace tent {

template <int kCtrl>
__device__ __forceinline__ uint64_t dpp_move64(uint64_t v)
{
    // every control used below gives each lane a valid source lane, so no fill value is needed
    int lo = __builtin_amdgcn_mov_dpp((int)(uint32_t)v, kCtrl, 0xF, 0xF, true);
    int hi = __builtin_amdgcn_mov_dpp((int)(uint32_t)(v >> 32), kCtrl, 0xF, 0xF, true);
    return ((uint64_t)(uint32_t)hi << 32) | (uint32_t)lo;
}

__device__ __forceinline__ uint64_t min64(uint64_t a, uint64_t b) { return a < b ? a : b; }

// Minimum of a 64-bit key over the wavefront, returned in every lane.  Rows of 16 lanes are
// reduced with DPP butterflies (quad swaps, half-row mirror, row mirror); rows are only combined
// when more than 16 / 32 lanes can hold a live key.
__device__ __forceinline__ uint64_t wave_min64(uint64_t k, uint32_t live_lanes)
{
    k = min64(k, dpp_move64<0xB1>(k));      // quad_perm [1,0,3,2]
    k = min64(k, dpp_move64<0x4E>(k));      // quad_perm [2,3,0,1]
    k = min64(k, dpp_move64<0x141>(k));     // row_half_mirror
    k = min64(k, dpp_move64<0x140>(k));     // row_mirror
    if (live_lanes > 16) k = min64(k, (uint64_t)__shfl_xor((unsigned long long)k, 16, 64));
    if (live_lanes > 32) k = min64(k, (uint64_t)__shfl_xor((unsigned long long)k, 32, 64));
    return k;
}

__device__ __forceinline__ uint64_t read_lane64(uint64_t v, int lane)
{
    uint32_t lo = __builtin_amdgcn_readlane((int)(uint32_t)v, lane);
    uint32_t hi = __builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), lane);
    return ((uint64_t)hi << 32) | lo;
}

__global__ void __launch_bounds__(64) bind_serial_kernel(BatchDev b, RailParams rp, int mode)
{
    const bool use_pending = (mode & kBindUsePending) != 0;
    const int lane = threadIdx.x;
    const uint64_t n = use_pending ? b.plan->n_pending : b.n_slices;
    const bool live = lane < (int)rp.n_rails && ((rp.admitted >> lane) & 1);
    const uint64_t c0 = rp.c0[lane];
    const uint32_t c1 = (uint32_t)rp.c1[lane];
    uint64_t A = rp.A[lane], T = 0, cnt = 0;
    uint64_t n_before = 0;
    if (mode & kBindAfterRotation) {          // the rotation pass went first: its bytes are queued and staged ahead
        T = b.plan->Tr[lane];
        cnt = b.plan->cr[lane];
        A += T;
        n_before = b.plan->n_retry;
    }

    uint32_t id_next = 0, len_next = 0;
    if ((uint64_t)lane < n) {
        id_next = use_pending ? b.pending[lane] : (uint32_t)lane;
        len_next = b.s_len[id_next];
    }
    for (uint64_t blk = 0; blk < n; blk += 64) {
        const uint32_t id = id_next, len = len_next;
        const uint64_t q_next = blk + 64 + lane;
        if (q_next < n) {                                   // prefetch the next block of lengths
            id_next = use_pending ? b.pending[q_next] : (uint32_t)q_next;
            len_next = b.s_len[id_next];
        }
        const int m = (int)(n - blk < 64 ? n - blk : 64);
        uint32_t out_rail = 0;
        uint64_t out_off = 0;
        for (int t = 0; t < m; ++t) {
            const uint32_t L = __builtin_amdgcn_readlane((int)len, t);
            const uint64_t cost = c0 + (((A + L) * (uint64_t)c1) >> 16);
            uint64_t key = live ? ((cost << 6) | (uint32_t)lane) : ~0ull;
            key = wave_min64(key, rp.n_rails);
            const int win = (int)(__builtin_amdgcn_readfirstlane((int)(uint32_t)key) & 63);
            const uint64_t T_win = read_lane64(T, win);
            if (lane == t) { out_rail = (uint32_t)win; out_off = T_win; }
            if (lane == win) { A += L; T += L; ++cnt; }
        }
        if (lane < m) {
            b.s_rail[id] = out_rail;
            b.s_stage_off[id] = out_off;
            b.s_state[id] = TENT_SLICE_BOUND;
        }
    }

    // per-rail totals and staging region bases (exclusive sum of 256-byte-rounded totals)
    uint64_t rounded = (T + 255) & ~255ull;
    uint64_t inc = rounded;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        uint64_t up = __shfl_up((unsigned long long)inc, d, 64);
        if (lane >= d) inc += up;
    }
    PlanState* ps = b.plan;
    ps->T[lane] = T;
    ps->cnt[lane] = cnt;
    ps->A_after[lane] = A;
    ps->base[lane] = inc - rounded;
    if (lane == 0) {
        ps->n_bound = n + n_before;
        if (!use_pending) ps->n_pending = n;
    }
}

hipError_t launch_bind_serial(const BatchDev& b, const RailParams& rp, int mode, hipStream_t s)
{
    hipLaunchKernelGGL(bind_serial_kernel, dim3(1), dim3(64), 0, s, b, rp, mode);
    return hipGetLastError();
}

}  // namespace tent
