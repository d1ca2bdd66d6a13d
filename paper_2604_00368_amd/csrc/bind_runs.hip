// Run-parallel rail assignment.  Produces exactly the binding of the slice-by-slice rule
// (Algorithm 1 Stage 2 of the paper with per-slice earliest completion, Section 4.2; ties to the
// lowest rail; in-flight bytes A_d grow with every bound slice), but only the chain over *runs* of
// equal-length slices is sequential.
//
// Why this is exact.  Inside a run of m slices of equal length l, rail d's successive candidate costs
//     f_d(k) = c0_d + (((A_d + (k+1) l) c1_d) >> 16),   k = 0, 1, ...
// are nondecreasing in k, so picking the cheapest rail m times is a merge of R sorted sequences: the
// run takes the m smallest triples (f_d(k), d, k) in lexicographic order, and the slice at position
// p of the run gets the triple of rank p.  Three steps follow from that:
//   1. run table     maximal runs of equal-length pending slices (flag heads, exclusive scan);
//   2. chain         one wavefront, lane = rail, walks the runs in order and finds, per run, how many
//                    slots k_d each rail takes.  The split is found by evaluating
//                    count_d(v) = #{k : f_d(k) <= v} (closed form, two integer divisions) at a cost
//                    level v guessed from a floating-point water-filling model, then repaired one
//                    slot at a time (add the cheapest free slot / drop the dearest taken slot) until
//                    exactly m slots are taken.  Floating point only steers the guess; the counts
//                    and repairs are integer and exact.  Runs of one slice (tails) are a plain argmin.
//   3. emit          one lane per slot (d, k): its rank in the run is
//                    k + sum_{d' < d} count_d'(f) + sum_{d' > d} count_d'(f - 1),  f = f_d(k),
//                    which gives the slice it belongs to; staging offset = T_d at run start + k l.
#include "scan.h"
#include "tile_tables.h"
#include "wave.h"

namespace tent {

namespace {

constexpr int kTol = 4;                    // repair at most this many slots one by one
constexpr uint64_t kCostCap = 1ull << 47;  // every feasible (X * c1) >> 16 is below this (host precondition)

// floor(a / b) for 1 <= b < 2^32 with inv = 1.0 / b.  The floating-point quotient is only an
// estimate; the remainder check makes the result exact for every a.
__device__ __forceinline__ uint64_t div_exact(uint64_t a, uint32_t b, double inv)
{
    if (a >> 50) return a / b;
    uint64_t q = (uint64_t)((double)a * inv);
    int64_t r = (int64_t)(a - q * b);
#pragma clang loop unroll(disable)
    while (r < 0) { --q; r += b; }
#pragma clang loop unroll(disable)
    while (r >= (int64_t)b) { ++q; r -= b; }
    return q;
}

// Per-rail constants of one plan.
struct Rail {
    uint64_t c0;
    uint32_t c1;        // >= 1
    double inv_c1;
};

// Cost of the rail's slot k (0-based) of a run of l-byte slices when A bytes are already queued.
// k + 1 <= 2^32 - 1 because a batch holds fewer than 2^32 - 1 slices.
__device__ __forceinline__ uint64_t slot_cost(const Rail& r, uint64_t A, uint32_t l, uint32_t k)
{
    const uint64_t x = A + (uint64_t)(k + 1u) * l;
    return r.c0 + ((x * (uint64_t)r.c1) >> 16);
}

// #{k >= 0 : slot_cost(k) <= v}, clamped to m.  v may be negative.
__device__ __forceinline__ uint32_t slots_upto(const Rail& r, uint64_t A, uint32_t l, double inv_l, int64_t v, uint32_t m)
{
    if (v < 0 || (uint64_t)v < r.c0) return 0;
    uint64_t w1 = (uint64_t)v - r.c0 + 1;
    if (w1 > kCostCap) w1 = kCostCap;
    // largest X with (X * c1) >> 16 <= w1 - 1, i.e. floor((w1 * 65536 - 1) / c1), without overflow
    const uint64_t q1 = div_exact(w1, r.c1, r.inv_c1);
    const uint64_t r1 = w1 - q1 * r.c1;
    const uint64_t xmax = r1 == 0 ? (q1 << 16) - 1 : (q1 << 16) + div_exact((r1 << 16) - 1, r.c1, r.inv_c1);
    if (xmax < A + l) return 0;
    uint64_t room = xmax - A;
    const uint64_t want = (uint64_t)m * l;
    if (room > want) room = want;
    const uint64_t k = div_exact(room, l, inv_l);
    return (uint32_t)(k < m ? k : m);
}

// ---- step 1: run table ------------------------------------------------------------------------
struct RunHead {
    const uint32_t* s_len;
    const uint32_t* pending;      // nullptr: position = slice index
    const uint64_t* n_pending;    // device-resident count of positions
    __device__ uint64_t operator()(uint64_t q) const
    {
        if (q >= *n_pending) return 0;
        if (q == 0) return 1;
        const uint32_t a = pending ? pending[q] : (uint32_t)q;
        const uint32_t p = pending ? pending[q - 1] : (uint32_t)(q - 1);
        return s_len[a] != s_len[p];
    }
};

__global__ void __launch_bounds__(256) run_table_kernel(BatchDev b, int use_pending)
{
    const uint64_t n = b.plan->n_pending;
    RunHead head{b.s_len, use_pending ? b.pending : nullptr, &b.plan->n_pending};
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t q = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; q < n; q += stride)
        if (head(q) && b.scan_tmp[q] < b.run_capacity) b.run_start[b.scan_tmp[q]] = (uint32_t)q;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        // a transfer contributes at most two runs, so the capacity of 2 * n_desc always suffices
        uint64_t n_runs = b.scan_tmp[b.n_slices];
        if (n_runs > b.run_capacity) n_runs = b.run_capacity;
        b.plan->n_runs = n_runs;
        b.run_start[n_runs] = (uint32_t)n;
    }
}

__global__ void set_pending_all_kernel(BatchDev b) { b.plan->n_pending = b.n_slices; }

// ---- step 2: chain over runs ------------------------------------------------------------------
// Same value as slots_upto, reached from a floating-point estimate that is then checked against
// the integer cost of the neighbouring slots; falls back to the closed form when the estimate
// cannot be trusted to be within a few slots.
__device__ __forceinline__ uint32_t slots_upto_fast(const Rail& r, uint64_t A, uint32_t l, double inv_l, int64_t v, uint32_t m)
{
    if (v < 0 || (uint64_t)v < r.c0) return 0;
    const uint64_t w1 = (uint64_t)v - r.c0 + 1;
    if ((w1 >> 36) || (A >> 52)) return slots_upto(r, A, l, inv_l, v, m);
    const double x = (double)(w1 << 16) * r.inv_c1;            // bytes the rail may hold at cost v
    double kf = (x - (double)A) * inv_l;
    kf = kf < 0.0 ? 0.0 : (kf > (double)m ? (double)m : kf);
    uint32_t k = (uint32_t)kf;
    // the estimate is almost always exact: two cost evaluations confirm it
    const bool low = k < m && slot_cost(r, A, l, k) <= (uint64_t)v;
    const bool high = k > 0 && slot_cost(r, A, l, k - 1) > (uint64_t)v;
    if (low) {
        ++k;
#pragma clang loop unroll(disable)
        while (k < m && slot_cost(r, A, l, k) <= (uint64_t)v) ++k;
    } else if (high) {
        --k;
#pragma clang loop unroll(disable)
        while (k > 0 && slot_cost(r, A, l, k - 1) > (uint64_t)v) --k;
    }
    return k;
}

// kWide = 16, 32 or 64: lanes that can hold a rail; with 16 every reduction stays inside one DPP row.
// Runs in the first wavefront of a workgroup (lane = threadIdx.x < 64).
template <int kWide>
__device__ __forceinline__ void bind_chain(const BatchDev& b, const RailParams& rp, int mode)
{
    const bool use_pending = (mode & kBindUsePending) != 0;
    const int lane = threadIdx.x;
    constexpr int R = kWide;                                  // reduction width
    const int n_rails = (int)rp.n_rails;
    const bool live = lane < n_rails && ((rp.admitted >> lane) & 1);
    const uint64_t live_mask = __ballot(live);
    const double n_live = (double)__popcll(live_mask);
    Rail rail;
    rail.c0 = rp.c0[lane];
    rail.c1 = live ? (uint32_t)rp.c1[lane] : 1u;
    rail.inv_c1 = 1.0 / (double)rail.c1;
    const double G = live ? 65536.0 * rail.inv_c1 : 0.0;      // bytes the rail absorbs per picosecond
    const double g = (double)rail.c0 * G;                     // its fixed latency expressed in bytes
    const double c0d1 = 1.0 - (double)rail.c0;               // 1 - c0 as a double (c0 < 2^53)
    uint64_t A = rp.A[lane], T = 0, cnt = 0;
    uint64_t n_before = 0;
    if (mode & kBindAfterRotation) {          // the rotation pass went first: its bytes are queued and staged ahead
        T = b.plan->Tr[lane];
        cnt = b.plan->cr[lane];
        A += T;
        n_before = b.plan->n_retry;
    }
    double Ad = (double)A;                                    // floating-point shadow of A, estimates only
    const uint64_t n_runs = b.plan->n_runs;
    const uint32_t stride = b.run_stride;

    // Water-filling model: once every admitted rail has received a slot, all of them sit at the
    // common cost level, and level(bytes) = (bytes + sum_d(g_d + A_d)) / sum_d G_d needs no
    // cross-lane work: the second sum grows by exactly the bytes bound.
    bool all_proven = false;
    double pool_G = 0.0, pool_B = 0.0, inv_pool_G = 0.0;

    // run descriptors are fetched 64 at a time, one per lane, the next block prefetched
    uint32_t nx_start = 0, nx_m = 0, nx_len = 1, nx_id = 0;
    auto fetch = [&](uint64_t r) {
        if (r < n_runs) {
            nx_start = b.run_start[r];
            nx_m = b.run_start[r + 1] - nx_start;
            nx_id = use_pending ? b.pending[nx_start] : nx_start;
            nx_len = b.s_len[nx_id];
        }
    };
    fetch(lane);
    for (uint64_t blk = 0; blk < n_runs; blk += 64) {
        const uint32_t my_m = nx_m, my_len = nx_len, my_id = nx_id;
        const double my_inv_len = 1.0 / (double)my_len;       // one division per lane serves 64 runs
        fetch(blk + 64 + lane);
        const int in_blk = (int)(n_runs - blk < 64 ? n_runs - blk : 64);
        // results of single-slice runs wait in the lane that fetched the run and leave after the block
        uint32_t single_rail = 0xFFFFFFFFu;
        uint64_t single_off = 0;
        for (int t = 0; t < in_blk; ++t) {
            const uint32_t l = __builtin_amdgcn_readlane((int)my_len, t);
            const uint32_t m = __builtin_amdgcn_readlane((int)my_m, t);
            const uint64_t row = (blk + t) * stride;
            uint32_t k = 0;

            const double ld = (double)l;
            if (m == 1) {
                // a single slice: plain argmin
                const int win = argmin_cost(slot_cost(rail, A, l, 0), live, lane, R);
                const uint64_t T_win = read_lane64(T, win);
                if (lane == t) { single_rail = (uint32_t)win; single_off = T_win; }
                k = lane == win;
            } else {
                if (lane < n_rails) b.run_T[row + lane] = T;
                const double inv_l = __longlong_as_double((long long)read_lane64(
                    (uint64_t)__double_as_longlong(my_inv_len), t));
                uint32_t taken = 0;
                bool solved = false;
                if (__builtin_expect(all_proven && m > (uint32_t)kTol, 1)) {
                    // Steady state, lean path: level from the incremental water-filling sums, slot
                    // counts from a floating-point estimate confirmed by the integer cost of the
                    // slot below and the slot above, repair with incrementally updated costs.
                    const double v = (((double)m + 0.5 * n_live) * ld + pool_B) * inv_pool_G;
                    if (__builtin_expect(v >= 0.0 && v < 1.0e15, 1)) {
                        const double vfl = floor(v);
                        const uint64_t vi = (uint64_t)vfl;
                        double kf = ((vfl + c0d1) * G - Ad) * inv_l;
                        kf = kf > 0.0 ? kf : 0.0;
                        kf = kf < (double)m ? kf : (double)m;
                        uint32_t kk = (uint32_t)kf;
                        const uint64_t lc1 = (uint64_t)l * rail.c1;
                        uint64_t p_prev = (A + (uint64_t)kk * l) * (uint64_t)rail.c1;   // slot kk-1 ends here
                        uint64_t p_next = p_prev + lc1;                                  // slot kk ends here
                        uint64_t c_prev = rail.c0 + (p_prev >> 16);
                        uint64_t c_next = rail.c0 + (p_next >> 16);
                        const bool off = live && ((kk < m && c_next <= vi) || (kk > 0 && c_prev > vi));
                        if (__builtin_expect(__ballot(off) == 0, 1)) {
                            const uint32_t tt = __builtin_amdgcn_readfirstlane((int)wave_reduce32(kk, R, Add32{}));
                            int miss = (int)m - (int)tt;
                            if (__builtin_expect(miss <= kTol && miss >= -kTol, 1)) {
                                while (miss > 0) {            // add the cheapest free slot
                                    const int win = argmin_cost(c_next, live && kk < m, lane, R);
                                    if (lane == win) {
                                        ++kk;
                                        p_prev = p_next; c_prev = c_next;
                                        p_next += lc1;   c_next = rail.c0 + (p_next >> 16);
                                    }
                                    --miss;
                                }
                                while (miss < 0) {            // drop the dearest taken slot
                                    const int win = argmax_cost(c_prev, live && kk > 0, lane, R);
                                    if (lane == win) {
                                        --kk;
                                        p_next = p_prev; c_next = c_prev;
                                        p_prev -= lc1;   c_prev = rail.c0 + (p_prev >> 16);
                                    }
                                    ++miss;
                                }
                                k = kk;
                                taken = m;
                                solved = true;
                            }
                        }
                    }
                }
                if (__builtin_expect(!solved && m > (uint32_t)kTol, 0)) {
                    double v;
                    if (all_proven) {
                        v = (((double)m + 0.5 * n_live) * (double)l + pool_B) * inv_pool_G;
                    } else {
                        // rails whose next slot already costs more than the level stay out of the pool
                        const uint64_t head = live ? slot_cost(rail, A, l, 0) : ~0ull;
                        bool wet = live;
                        v = 0.0;
                        for (int pass = 0; pass < 64; ++pass) {
                            const uint64_t wet_mask = __ballot(wet);
                            const double sumG = wave_sum_f64(wet ? G : 0.0, R);
                            const double sumB = wave_sum_f64(wet ? g + (double)A : 0.0, R);
                            const double need = ((double)m + 0.5 * (double)__popcll(wet_mask)) * (double)l;
                            v = __longlong_as_double((long long)uniform64((uint64_t)__double_as_longlong((need + sumB) / sumG)));
                            const bool still = wet && (cnt > 0 || (double)head <= v);
                            const uint64_t still_mask = __ballot(still);
                            if (still_mask == wet_mask || still_mask == 0) break;
                            wet = still;
                        }
                    }
                    // bracket (computed only if the first guess misses):
                    // slots summed over rails stay below m at `lo` and reach at least m at `hi`
                    bool bracketed = false;
                    int64_t lo = 0, hi = 0;
                    for (int iter = 0;; ++iter) {
                        int64_t vi = (v >= 0.0 && v < 9.0e18) ? (int64_t)v : -1;
                        if (!bracketed && vi < 0) {
                            const uint64_t head = live ? slot_cost(rail, A, l, 0) : ~0ull;
                            const uint64_t alone = live ? slot_cost(rail, A, l, m - 1) : ~0ull;
                            lo = (int64_t)uniform64(wave_reduce64(head, R, OpMin{})) - 1;
                            hi = (int64_t)uniform64(wave_reduce64(alone, R, OpMin{}));
                            bracketed = true;
                        }
                        if (bracketed && (iter >= 8 || vi <= lo || vi >= hi)) {   // guess unusable: bisect
                            vi = lo + (hi - lo) / 2;
                            if (vi <= lo) vi = hi;
                        }
                        const uint32_t kk = live ? slots_upto_fast(rail, A, l, inv_l, vi, m) : 0;
                        const uint64_t tt = uniform64(wave_reduce64(kk, R, OpAdd{}));
                        const int64_t miss = (int64_t)m - (int64_t)tt;
                        if (miss <= kTol && miss >= -kTol) { k = kk; taken = (uint32_t)tt; break; }
                        if (!bracketed) {
                            const uint64_t head = live ? slot_cost(rail, A, l, 0) : ~0ull;
                            const uint64_t alone = live ? slot_cost(rail, A, l, m - 1) : ~0ull;
                            lo = (int64_t)uniform64(wave_reduce64(head, R, OpMin{})) - 1;
                            hi = (int64_t)uniform64(wave_reduce64(alone, R, OpMin{}));
                            bracketed = true;
                        }
                        if (miss > 0) { if (vi > lo) lo = vi; } else { if (vi < hi) hi = vi; }
                        if (hi - lo == 1) {
                            // the whole deficit sits at cost `hi`: hand it out in rail order
                            const uint32_t k_lo = live ? slots_upto(rail, A, l, inv_l, lo, m) : 0;
                            const uint32_t k_hi = live ? slots_upto(rail, A, l, inv_l, hi, m) : 0;
                            const uint64_t below = uniform64(wave_reduce64(k_lo, R, OpAdd{}));
                            uint64_t tie = k_hi - k_lo, inc = tie;
#pragma unroll
                            for (int d = 1; d < 64; d <<= 1) {
                                uint64_t up = (uint64_t)__shfl_up((unsigned long long)inc, d, 64);
                                if (lane >= d) inc += up;
                            }
                            const uint64_t before = inc - tie;                 // ties on lower rails
                            const uint64_t rem = (uint64_t)m - below;
                            const uint64_t take = before >= rem ? 0 : (rem - before < tie ? rem - before : tie);
                            k = k_lo + (uint32_t)take;
                            taken = m;
                            break;
                        }
                        const bool near = live && (kk > 0 || slot_cost(rail, A, l, 0) <= (uint64_t)(vi < 0 ? 0 : vi) + 1);
                        double rate = wave_sum_f64(near ? G : 0.0, R);
                        if (!(rate > 0.0)) rate = wave_sum_f64(G, R);
                        v = __longlong_as_double((long long)uniform64(
                            (uint64_t)__double_as_longlong((double)vi + (double)miss * (double)l / rate)));
                    }
                }
                // repair: add the cheapest free slot / drop the dearest taken slot
                while (taken < m) {
                    const int win = argmin_cost(slot_cost(rail, A, l, k), live && k < m, lane, R);
                    k += lane == win;
                    ++taken;
                }
                while (taken > m) {
                    const int win = argmax_cost(slot_cost(rail, A, l, k > 0 ? k - 1 : 0), live && k > 0, lane, R);
                    k -= lane == win;
                    --taken;
                }
                if (lane < n_rails) b.run_K[row + lane] = k;
            }
            const uint64_t bytes = (uint64_t)k * l;
            A += bytes;
            T += bytes;
            cnt += k;
            Ad = fma((double)k, ld, Ad);
            if (all_proven) {
                pool_B += (double)m * ld;
            } else if (__ballot(live && cnt > 0) == live_mask) {
                all_proven = true;
                pool_G = wave_sum_f64(G, R);
                pool_B = wave_sum_f64(live ? g + (double)A : 0.0, R);
                pool_G = __longlong_as_double((long long)uniform64((uint64_t)__double_as_longlong(pool_G)));
                pool_B = __longlong_as_double((long long)uniform64((uint64_t)__double_as_longlong(pool_B)));
                inv_pool_G = 1.0 / pool_G;
            }
        }
        if (single_rail != 0xFFFFFFFFu) {
            b.s_rail[my_id] = single_rail;
            b.s_stage_off[my_id] = single_off;
            b.s_state[my_id] = TENT_SLICE_BOUND;
        }
    }

    // per-rail totals and staging region bases (exclusive sum of 256-byte-rounded totals)
    const uint64_t rounded = (T + 255) & ~255ull;
    uint64_t inc = rounded;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        uint64_t up = (uint64_t)__shfl_up((unsigned long long)inc, d, 64);
        if (lane >= d) inc += up;
    }
    PlanState* ps = b.plan;
    ps->T[lane] = T;
    ps->cnt[lane] = cnt;
    ps->A_after[lane] = A;
    ps->base[lane] = inc - rounded;
    if (lane == 0) ps->n_bound = ps->n_pending + n_before;
}

template <int kWide>
__global__ void __launch_bounds__(64) bind_chain_kernel(BatchDev b, RailParams rp, int mode)
{
    bind_chain<kWide>(b, rp, mode);
}

// The chain is one wavefront; the tile tables of the copy kernels depend on the slice table only, not
// on the binding.  On a first plan both go into one launch: workgroup 0 walks the chain, the others
// build the tables, so the tables cost no time of their own.
template <int kWide>
__global__ void __launch_bounds__(256) bind_chain_tables_kernel(BatchDev b, RailParams rp, int mode)
{
    if (blockIdx.x == 0) {
        if (threadIdx.x < 64) bind_chain<kWide>(b, rp, mode);
        return;
    }
    build_tile_tables(b, blockIdx.x - 1, gridDim.x - 1);
}

// ---- step 3: emit -----------------------------------------------------------------------------
// One lane per position q of the pending sequence; inside its run the lane enumerates slot
// t = q - run_start as (rail d, index k) in rail-major order and computes the slot's rank.
__global__ void __launch_bounds__(256) bind_emit_kernel(BatchDev b, RailParams rp, int use_pending)
{
    __shared__ uint64_t sh_c0[TENT_MAX_RAILS];
    __shared__ uint32_t sh_c1[TENT_MAX_RAILS];
    __shared__ double sh_inv[TENT_MAX_RAILS];
    const uint32_t R = rp.n_rails;
    if (threadIdx.x < TENT_MAX_RAILS) {
        const uint32_t c1 = (uint32_t)rp.c1[threadIdx.x];
        sh_c0[threadIdx.x] = rp.c0[threadIdx.x];
        sh_c1[threadIdx.x] = c1 ? c1 : 1u;
        sh_inv[threadIdx.x] = 1.0 / (double)(c1 ? c1 : 1u);
    }
    __syncthreads();
    const uint64_t n = b.plan->n_pending;
    const uint32_t stride = b.run_stride;
    const uint64_t gstride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t q = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; q < n; q += gstride) {
        // run of this position: number of heads at or before q, minus one
        const uint32_t id_q = use_pending ? b.pending[q] : (uint32_t)q;
        uint64_t r = b.scan_tmp[q];
        {
            const bool head = q == 0 || b.s_len[id_q] != b.s_len[use_pending ? b.pending[q - 1] : (uint32_t)(q - 1)];
            if (!head) r -= 1;
        }
        const uint32_t start = b.run_start[r];
        const uint32_t m = b.run_start[r + 1] - start;
        if (m == 1) continue;                                   // bound by the chain kernel
        const uint32_t l = b.s_len[id_q];
        const double inv_l = 1.0 / (double)l;
        const uint64_t row = r * stride;
        // slot t -> (d, k)
        uint32_t t = (uint32_t)(q - start), d = 0;
        for (; d < R; ++d) {
            const uint32_t kd = ((rp.admitted >> d) & 1) ? b.run_K[row + d] : 0;
            if (t < kd) break;
            t -= kd;
        }
        if (d >= R) continue;
        const uint32_t k = t;
        const uint64_t T_d = b.run_T[row + d];
        Rail me{sh_c0[d], sh_c1[d], sh_inv[d]};
        const uint64_t f = slot_cost(me, rp.A[d] + T_d, l, k);
        uint64_t rank = k;
        for (uint32_t o = 0; o < R; ++o) {
            if (o == d || !((rp.admitted >> o) & 1)) continue;
            const uint32_t ko = b.run_K[row + o];
            if (ko == 0) continue;
            Rail other{sh_c0[o], sh_c1[o], sh_inv[o]};
            const uint64_t A_o = rp.A[o] + b.run_T[row + o];
            // slots of a lower rail win ties, slots of a higher rail lose them
            const uint32_t c = slots_upto(other, A_o, l, inv_l, o < d ? (int64_t)f : (int64_t)f - 1, ko);
            rank += c;
        }
        const uint64_t pos = (uint64_t)start + rank;
        const uint32_t id = use_pending ? b.pending[pos] : (uint32_t)pos;
        b.s_rail[id] = d;
        b.s_stage_off[id] = T_d + (uint64_t)k * l;
        b.s_state[id] = TENT_SLICE_BOUND;
    }
}

}  // namespace

hipError_t launch_bind_runs(const BatchDev& b, const RailParams& rp, int mode, hipStream_t s)
{
    const bool use_pending = (mode & kBindUsePending) != 0;
    const int up = use_pending ? 1 : 0;
    if (!use_pending) hipLaunchKernelGGL(set_pending_all_kernel, dim3(1), dim3(1), 0, s, b);
    RunHead head{b.s_len, use_pending ? b.pending : nullptr, &b.plan->n_pending};
    hipError_t e = exclusive_scan(head, b.n_slices, b.scan_tmp, b.scan_partials, s);
    if (e != hipSuccess) return e;
    uint64_t blocks = (b.n_slices + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(run_table_kernel, dim3((uint32_t)blocks), dim3(256), 0, s, b, up);
    if (mode & kBindBuildTables) {
        const dim3 grid(1 + tile_table_blocks(b)), block(256);
        if (rp.n_rails <= 16)      hipLaunchKernelGGL(bind_chain_tables_kernel<16>, grid, block, 0, s, b, rp, mode);
        else if (rp.n_rails <= 32) hipLaunchKernelGGL(bind_chain_tables_kernel<32>, grid, block, 0, s, b, rp, mode);
        else                       hipLaunchKernelGGL(bind_chain_tables_kernel<64>, grid, block, 0, s, b, rp, mode);
    } else {
        if (rp.n_rails <= 16)      hipLaunchKernelGGL(bind_chain_kernel<16>, dim3(1), dim3(64), 0, s, b, rp, mode);
        else if (rp.n_rails <= 32) hipLaunchKernelGGL(bind_chain_kernel<32>, dim3(1), dim3(64), 0, s, b, rp, mode);
        else                       hipLaunchKernelGGL(bind_chain_kernel<64>, dim3(1), dim3(64), 0, s, b, rp, mode);
    }
    hipLaunchKernelGGL(bind_emit_kernel, dim3((uint32_t)blocks), dim3(256), 0, s, b, rp, up);
    return hipGetLastError();
}

}  // namespace tent
