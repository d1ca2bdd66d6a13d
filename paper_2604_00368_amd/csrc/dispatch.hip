// Request-level dispatch (Algorithm 1 of the paper, Stages 1-3; Section 4.2 "Slice Dispatching" and
// "Quality of Service").  The algorithm runs once per request -- here per declared transfer, in
// declaration order:
//   Stage 1  admitted rails = non-excluded rails whose priority slot accepts the request
//            (the host passes one mask per priority level for the current window);
//   Stage 2  s_d = c0_d + (((A_d + L) * c1_d) >> 16) with the queue state at the start of the request;
//   Stage 3  mice (request shorter than theta): the whole request goes to one rail, picked round robin
//            among the admitted rails with s_d <= s_min + floor(gamma * s_min / 256);
//            elephants: weighted proportional spraying with weights 1 / s_d -- the request's pending
//            slices are dealt in order, each to the rail with the smallest (m_d + 1) * s_d (m_d = slices
//            of the request already on d, ties to the lowest rail).
//
// Requests depend on each other through A_d, so the per-request decisions form a chain: one
// wavefront, lane d = rail d.  Inside an elephant request nothing depends on A_d any more: dealing by
// smallest (m_d + 1) * s_d is the merge of the rails' arithmetic sequences s_d, 2 s_d, 3 s_d, ..., so the
// chain only needs the number of slots K_d each rail takes among the first n merged elements (a
// floating-point estimate of the cut level, repaired with exact integer comparisons), and a second,
// fully parallel kernel gives every slot its rank in the merge in closed form (R integer divisions).
#include "scan.h"
#include "tile_tables.h"
#include "wave.h"

namespace tent {
namespace {

constexpr uint64_t kNoKey = ~0ull;

// ---- the chain over requests -------------------------------------------------------------------
// kWide = 16, 32 or 64: smallest of these that covers the rails; lanes beyond the rails only tag along
// (uniform decisions are read from lane 0's row).
// Runs in the first wavefront of a workgroup (lane = threadIdx.x < 64).
template <int kWide>
__device__ __forceinline__ void dispatch_chain(const BatchDev& b, const RailParams& rp, const DispatchParams& dp)
{
    const int lane = threadIdx.x;
    const uint64_t S = b.slice_bytes;
    const uint32_t D = b.n_desc;
    const uint32_t stride = b.run_stride;
    const uint64_t c0 = rp.c0[lane];
    const uint64_t c1 = rp.c1[lane];
    uint64_t A = rp.A[lane], T = 0, cnt = 0;
    uint64_t rr = dp.rr_start, n_mice = 0, n_elephant = 0, n_deferred = 0, n_bound = 0, n_pending = 0;
    const uint64_t lanes_below = (1ull << lane) - 1;

    for (uint32_t blk = 0; blk < D; blk += 64) {
        // lane t fetches the description of request blk + t
        const uint32_t jl = blk + lane;
        uint32_t my_n = 0, my_short = 0, my_prio = 2;
        uint64_t my_len = 0;
        if (jl < D) {
            const uint64_t f0 = b.first[jl], f1 = b.first[jl + 1];
            my_n = (uint32_t)(b.scan_tmp[f1] - b.scan_tmp[f0]);              // slices of the request not DONE
            my_len = b.src_pre[b.src_ptr[jl + 1]] - b.src_pre[b.src_ptr[jl]];
            const uint64_t last_len = my_len - (f1 - f0 - 1) * S;
            if (b.s_state[f1 - 1] != TENT_SLICE_DONE) my_short = (uint32_t)(S - last_len);
            if (!dp.all_high) my_prio = b.priority[jl];
        }
        const int m = (int)(D - blk < 64 ? D - blk : 64);
        uint32_t my_mode = 0;
        for (int t = 0; t < m; ++t) {
            const uint32_t n = (uint32_t)__builtin_amdgcn_readlane((int)my_n, t);
            if (n == 0) continue;
            n_pending += n;
            const uint32_t prio = (uint32_t)__builtin_amdgcn_readlane((int)my_prio, t);
            const uint64_t adm = dp.adm[prio > 2 ? 2 : prio];
            if (adm == 0) {                                                  // Stage 1: nothing admitted
                if (lane == t) my_mode = 3;
                ++n_deferred;
                continue;
            }
            const uint64_t L_req = read_lane64(my_len, t);
            const uint32_t short_by = (uint32_t)__builtin_amdgcn_readlane((int)my_short, t);
            const bool live = (adm >> lane) & 1;
            const bool mice = L_req < dp.theta;
            const uint64_t L = mice ? L_req : (L_req < S ? L_req : S);
            uint64_t s = c0 + (((A + L) * c1) >> 16);                        // Stage 2
            uint64_t K = 0, bytes = 0;
            if (mice) {
                const uint64_t s_min = wave_reduce64(live ? s : kNoKey, kWide, OpMin{});
                const uint64_t limit = s_min + ((s_min * dp.gamma_q8) >> 8);
                const uint64_t cand = __ballot(live && s <= limit);
                const uint32_t idx = (uint32_t)(rr % (uint64_t)__popcll(cand));
                ++rr;
                const bool me = ((cand >> lane) & 1) && (uint32_t)__popcll(cand & lanes_below) == idx;
                if (me) { K = n; bytes = (uint64_t)n * S - short_by; }
                if (lane == t) my_mode = 1;
                ++n_mice;
            } else {
                if (s == 0) s = 1;
                // cut level of the merge: x with sum_d floor(x / s_d) ~ n
                const double inv = live ? 1.0 / (double)s : 0.0;
                const double sum_inv = wave_sum_f64(inv, kWide);
                const double n_live = (double)__popcll(adm);
                const double x = ((double)n + 0.5 * n_live) / sum_inv;
                if (live) {
                    const double kf = x * inv;
                    K = kf >= (double)n ? n : (uint64_t)kf;
                }
                uint64_t total = uniform64(wave_reduce64(K, kWide, OpAdd{}));
                // exact repair: grow by the cheapest free slot / shrink by the dearest held slot
#pragma clang loop unroll(disable)
                while (total < n) {
                    const int win = argmin_cost((K + 1) * s, live, lane, kWide);
                    if (lane == win) ++K;
                    ++total;
                }
#pragma clang loop unroll(disable)
                while (total > n) {
                    const int win = argmax_cost(K * s, live && K, lane, kWide);
                    if (lane == win) --K;
                    --total;
                }
                // the held slots must be exactly the first n of the merge: the dearest held slot
                // (ties: highest rail last) precedes the cheapest free slot (ties: lowest rail first)
                int last = 0;
#pragma clang loop unroll(disable)
                for (int guard = 0; guard < 4096; ++guard) {
                    last = argmax_cost(K * s, live && K, lane, kWide);
                    const int next = argmin_cost((K + 1) * s, live, lane, kWide);
                    const uint64_t held = read_lane64(K * s, last);
                    const uint64_t free_ = read_lane64((K + 1) * s, next);
                    if (held < free_ || (held == free_ && last < next)) break;
                    if (lane == last) --K;
                    if (lane == next) ++K;
                }
                // the request's last pending slice is the last element of the merge
                bytes = K * S - (lane == last ? short_by : 0);
                if (lane == t) my_mode = 2;
                ++n_elephant;
            }
            if (lane < (int)stride) {
                const uint64_t row = (uint64_t)(blk + t) * stride + lane;
                b.run_K[row] = (uint32_t)K;
                b.run_T[row] = T;
            }
            A += bytes;
            T += bytes;
            cnt += K;
            n_bound += n;
        }
        if (jl < D) b.req_mode[jl] = (uint8_t)my_mode;
    }

    const uint64_t rounded = (T + 255) & ~255ull;
    uint64_t inc = rounded;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint64_t up = (uint64_t)__shfl_up((unsigned long long)inc, d, 64);
        if (lane >= d) inc += up;
    }
    PlanState* ps = b.plan;
    ps->T[lane] = T;
    ps->cnt[lane] = cnt;
    ps->A_after[lane] = A;
    ps->base[lane] = inc - rounded;
    if (lane == 0) {
        ps->n_bound = n_bound;
        ps->n_pending = n_pending;
        ps->n_mice = n_mice;
        ps->n_elephant = n_elephant;
        ps->n_deferred = n_deferred;
        ps->rr_next = rr;
    }
}

template <int kWide>
__global__ void __launch_bounds__(64) dispatch_chain_kernel(BatchDev b, RailParams rp, DispatchParams dp)
{
    dispatch_chain<kWide>(b, rp, dp);
}

// First plan of a batch: the tile tables of the copy kernels are built by the other workgroups of the
// chain's launch (they depend on the slice table only).
template <int kWide>
__global__ void __launch_bounds__(256) dispatch_chain_tables_kernel(BatchDev b, RailParams rp, DispatchParams dp)
{
    if (blockIdx.x == 0) {
        if (threadIdx.x < 64) dispatch_chain<kWide>(b, rp, dp);
        return;
    }
    build_tile_tables(b, blockIdx.x - 1, gridDim.x - 1);
}

// ---- emit: one lane per pending position ---------------------------------------------------------
// Position q of the pending list belongs to request j; inside the request the lane takes slot
// number t = q - (first pending position of j) in rail-major order, i.e. slot k of rail d, computes
// the slot's rank in the merge and hands it to the request's rank-th pending slice.
__global__ void __launch_bounds__(256) dispatch_emit_kernel(BatchDev b, RailParams rp, DispatchParams dp)
{
    const uint32_t R = rp.n_rails;
    const uint32_t stride = b.run_stride;
    const uint64_t S = b.slice_bytes;
    const uint64_t n = b.scan_tmp[b.n_slices];                       // slices not DONE
    const uint64_t gstride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t q = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; q < n; q += gstride) {
        const uint32_t i_q = b.pending[q];
        const uint32_t j = b.s_desc[i_q];
        const uint32_t mode = b.req_mode[j];
        if (mode != 1 && mode != 2) continue;                        // deferred
        const uint64_t q0 = b.scan_tmp[b.first[j]];                  // first pending position of the request
        const uint64_t row = (uint64_t)j * stride;
        uint32_t t = (uint32_t)(q - q0), d = 0;
        for (; d < R; ++d) {
            const uint32_t kd = b.run_K[row + d];
            if (t < kd) break;
            t -= kd;
        }
        if (d >= R) continue;
        const uint32_t k = t;
        uint64_t rank = k;
        if (mode == 2) {
            const uint64_t req_len = b.src_pre[b.src_ptr[j + 1]] - b.src_pre[b.src_ptr[j]];
            const uint64_t L = req_len < S ? req_len : S;
            uint64_t s_d = rp.c0[d] + (((rp.A[d] + b.run_T[row + d] + L) * rp.c1[d]) >> 16);
            if (s_d == 0) s_d = 1;
            const uint64_t key = (uint64_t)(k + 1) * s_d;
            for (uint32_t o = 0; o < R; ++o) {
                const uint32_t ko = b.run_K[row + o];
                if (o == d || ko == 0) continue;
                uint64_t s_o = rp.c0[o] + (((rp.A[o] + b.run_T[row + o] + L) * rp.c1[o]) >> 16);
                if (s_o == 0) s_o = 1;
                // slots of a lower rail win ties, slots of a higher rail lose them
                const uint64_t before = (o < d ? key : key - 1) / s_o;
                rank += before < ko ? before : ko;
            }
        }
        const uint32_t id = b.pending[q0 + rank];
        b.s_rail[id] = d;
        b.s_stage_off[id] = b.run_T[row + d] + (uint64_t)k * S;
        b.s_state[id] = TENT_SLICE_BOUND;
    }
}

struct NotDone {
    const uint8_t* state;
    __device__ uint64_t operator()(uint64_t i) const { return state[i] != TENT_SLICE_DONE; }
};

__global__ void __launch_bounds__(256) pending_list_kernel(BatchDev b)
{
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < b.n_slices; i += stride)
        if (b.s_state[i] != TENT_SLICE_DONE) {
            b.pending[b.scan_tmp[i]] = (uint32_t)i;
            b.s_state[i] = TENT_SLICE_PENDING;                       // a slice bound earlier and never moved is dealt again
        }
}

}  // namespace

hipError_t launch_dispatch(const BatchDev& b, const RailParams& rp, const DispatchParams& dp, bool build_tables,
                           hipStream_t s)
{
    hipError_t e = exclusive_scan(NotDone{b.s_state}, b.n_slices, b.scan_tmp, b.scan_partials, s);
    if (e != hipSuccess) return e;
    uint64_t blocks = (b.n_slices + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(pending_list_kernel, dim3((uint32_t)blocks), dim3(256), 0, s, b);
    if (build_tables) {
        const dim3 grid(1 + tile_table_blocks(b)), block(256);
        if (rp.n_rails <= 16)      hipLaunchKernelGGL(dispatch_chain_tables_kernel<16>, grid, block, 0, s, b, rp, dp);
        else if (rp.n_rails <= 32) hipLaunchKernelGGL(dispatch_chain_tables_kernel<32>, grid, block, 0, s, b, rp, dp);
        else                       hipLaunchKernelGGL(dispatch_chain_tables_kernel<64>, grid, block, 0, s, b, rp, dp);
    } else {
        if (rp.n_rails <= 16)      hipLaunchKernelGGL(dispatch_chain_kernel<16>, dim3(1), dim3(64), 0, s, b, rp, dp);
        else if (rp.n_rails <= 32) hipLaunchKernelGGL(dispatch_chain_kernel<32>, dim3(1), dim3(64), 0, s, b, rp, dp);
        else                       hipLaunchKernelGGL(dispatch_chain_kernel<64>, dim3(1), dim3(64), 0, s, b, rp, dp);
    }
    hipLaunchKernelGGL(dispatch_emit_kernel, dim3((uint32_t)blocks), dim3(256), 0, s, b, rp, dp);
    return hipGetLastError();
}

}  // namespace tent
