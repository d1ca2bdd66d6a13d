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
//   1. run table     maximal runs of equal-length pending slices (flag heads, exclusive scan), and one record
//                    per run with everything that does not depend on the rails' state, among it the cost level
//                    at which the run will end according to a floating-point water-filling model;
//   2. chain         one wavefront, lane = rail, walks the runs in order and finds, per run, how many
//                    slots k_d each rail takes.  The split is found from the record's level (slot count per
//                    rail from a floating-point estimate, confirmed against the integer costs of the two
//                    neighbouring slots) and repaired one slot at a time (add the cheapest free slot / drop
//                    the dearest taken slot) until exactly m slots are taken; where the estimate does not
//                    hold, count_d(v) = #{k : f_d(k) <= v} (closed form, two integer divisions) is evaluated
//                    at bracketed levels instead.  Floating point only steers the guess; the counts and
//                    repairs are integer and exact.  Runs of one slice (tails) are a plain argmin.  A second
//                    wavefront feeds the run records to the chain through a ring in LDS.
//   3. emit          one lane per slot (d, k): its rank in the run is
//                    k + sum_{d' < d} count_d'(f) + sum_{d' > d} count_d'(f - 1),  f = f_d(k),
//                    which gives the slice it belongs to; staging offset = T_d at run start + k l.
#include <type_traits>

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

// Smallest 32-bit key over the wavefront (keys carry a lane in their low 6 bits), as a uniform value.
template <int R>
__device__ __forceinline__ uint32_t wave_min_key(uint32_t key)
{
    return (uint32_t)__builtin_amdgcn_readfirstlane((int)wave_reduce32(key, R, Min32{}));
}

// Costs within 2^25 ps of the level are compared as 32-bit keys (offset << 6 | lane, below 2^31); a cost farther
// on the harmless side (a free slot far above the level, a taken slot far below it) gets the key kFarKey | lane,
// which loses against every near key; a winner at or above kFarKey means "no near candidate" and is never used.
constexpr uint32_t kRelBits = 25;
constexpr uint64_t kRelSpan = 1ull << kRelBits;
constexpr uint32_t kFarKey = 0x80000000u;
constexpr uint32_t kNoKey = 0xFFFFFFFFu;
constexpr uint64_t kNoLevel = ~0ull;
// The lean path sums slot counts in 32 bits: runs stay below 2^24 slices and a lane whose estimate cannot be
// used adds 2^25 instead of its count, so that with up to 64 lanes the sum neither wraps nor comes near m.
constexpr uint32_t kLeanRunMax = 1u << 24;
constexpr uint32_t kOffMark = 1u << 25;

// ---- step 1b: one record per run ---------------------------------------------------------------
// Everything the chain needs to know about a run that does not depend on the rails' state, computed
// in parallel before the chain starts; the chain fetches the records a block at a time.  The cost
// level comes from the water-filling model: the rails that take part end a run at a common cost level,
// level(bytes) = (bytes + sum_d h_d G_d) / sum_d G_d over those rails, with G_d = 65536 / c1_d bytes per
// picosecond and h_d the rail's head cost; a rail takes part once the level has passed its head cost.  The
// bytes bound before a run are known in advance (a prefix sum of the pending lengths), so the level after
// every run is too.  It is an estimate: the chain verifies what it derives from it in integers.
struct PendingLen {
    const uint32_t* s_len;
    const uint32_t* pending;      // nullptr: position = slice index
    const uint64_t* n_pending;
    __device__ uint64_t operator()(uint64_t q) const
    {
        if (q >= *n_pending) return 0;
        return s_len[pending ? pending[q] : (uint32_t)q];
    }
};

__global__ void __launch_bounds__(256) run_records_kernel(BatchDev b, RailParams rp, int mode)
{
    // Admitted rails in ascending order of their head cost h_d = c0_d + A_d c1_d / 65536 (what the rail's next byte
    // would cost): sh_h[j] the j-th smallest, sh_G[j] and sh_hG[j] the sums of G_d and of h_d G_d over the first j + 1.
    // At cost level v the rails with h_d < v hold sum (v - h_d) G_d bytes, so the level that holds B bytes is
    // (B + sh_hG[j]) / sh_G[j] for the first j at which it does not reach the next rail's head cost.
    __shared__ double sh_h[TENT_MAX_RAILS], sh_G[TENT_MAX_RAILS], sh_hG[TENT_MAX_RAILS];
    __shared__ uint32_t sh_live;
    const uint32_t t = threadIdx.x;
    if (t < TENT_MAX_RAILS) {
        auto head = [&](uint32_t d, double* G) -> double {
            const double c1 = (double)(uint32_t)rp.c1[d];                       // c1 >= 1 on this path
            const uint64_t A = rp.A[d] + ((mode & kBindAfterRotation) ? b.plan->Tr[d] : 0);
            *G = 65536.0 / c1;
            return (double)rp.c0[d] + (double)A * c1 * (1.0 / 65536.0);
        };
        const bool live = t < rp.n_rails && ((rp.admitted >> t) & 1);
        double G = 0.0;
        const double h = live ? head(t, &G) : 0.0;
        uint32_t rank = 0, n_live = 0;
        for (uint32_t d = 0; d < rp.n_rails; ++d) {
            if (!((rp.admitted >> d) & 1)) continue;
            ++n_live;
            double Gd;
            const double hd = head(d, &Gd);
            rank += (hd < h || (hd == h && d < t)) ? 1u : 0u;
        }
        if (live) { sh_h[rank] = h; sh_G[rank] = G; sh_hG[rank] = h * G; }
        if (t == 0) sh_live = n_live;
    }
    __syncthreads();
    if (t == 0) {
        for (uint32_t j = 1; j < sh_live; ++j) { sh_G[j] += sh_G[j - 1]; sh_hG[j] += sh_hG[j - 1]; }
    }
    __syncthreads();
    const uint64_t n_runs = b.plan->n_runs;
    const uint64_t r = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (r > n_runs) return;
    RunRec rec{0, 0, kNoLevel, 0.0, 0.0};
    if (r < n_runs) {
        const uint32_t start = b.run_start[r];
        const uint32_t id = (mode & kBindUsePending) ? b.pending[start] : start;
        rec.len = b.s_len[id];
        rec.m = b.run_start[r + 1] - start;
        rec.inv_len = 1.0 / (double)rec.len;
        const double bytes = (double)rec.m * (double)rec.len + (double)b.len_pre[start];
        const uint32_t n_live = sh_live;
        double v = -1.0;
        for (uint32_t j = 0; j < n_live; ++j) {
            // half a slice per participating rail on top: the slot counts are rounded down
            v = (bytes + 0.5 * (double)(j + 1) * (double)rec.len + sh_hG[j]) / sh_G[j];
            if (j + 1 == n_live || v <= sh_h[j + 1]) break;
        }
        // no level (the chain then takes its general path) for runs too short to gain from one or too long for
        // the short path's 32-bit slot sums
        if (v >= 0.0 && v < 1.0e14 && rec.m > (uint32_t)kTol && rec.m < kLeanRunMax) {
            rec.level = (uint64_t)v;
            rec.level_f = (double)rec.level;
        }
    }
    b.run_rec[r] = rec;
}

// ---- step 2: chain over runs ------------------------------------------------------------------
// kWide = 16, 32 or 64: lanes that can hold a rail; with 16 every reduction stays inside one DPP row.
// Runs in lanes 0 .. kWide-1 of the first wavefront of a workgroup; the other lanes leave at once.
//
// Per rail the chain keeps the exact product P = A * c1 of the bytes in flight (so that a slot's cost
// is c0 + ((P + j * l * c1) >> 16) with additions only), the bytes bound T, and a floating-point
// shadow of A for the estimates.  The loop is a chain of dependent instructions on one wavefront,
// so what counts is how few it issues per run and that it never waits for memory: run records come
// kWide at a time, one per lane, out of a ring in LDS that a second wavefront fills ahead of their use,
// and are handed out with readlane; results leave as one row of K and one of T per run.  The general path sits in a function of
// its own: inlined, its code and registers made the loop's short paths measurably slower.

// State of one lane of the chain that a run may change, and the slots the lane takes in the run.
struct ChainVars {
    uint64_t P, T;
    double Bd;
    uint64_t ref_level;
    uint32_t cnt, all_proven, k;
};

// A run of m slices of l bytes from any state and with any (or no) level estimate: the level is searched
// with exact slot counts (bracket, interpolation, bisection) and the split repaired slot by slot.  Kept
// out of line: the chain's loop calls it only where its short path does not apply.
template <int kWide>
__device__ __attribute__((noinline)) uint64_t bind_run_general(ChainVars cv, Rail rail, double G, double g, bool live,
                                                               uint64_t live_mask, uint64_t A_less_T, int lane, uint32_t l,
                                                               uint32_t m, uint64_t vi, double level_f, double inv_l)
{
    constexpr int R = kWide;
    const uint64_t T = cv.T;
    const uint32_t cnt = cv.cnt;
    bool all_proven = cv.all_proven != 0;
    uint32_t k = 0, taken = 0;
    const uint64_t A = A_less_T + T;
    if (!all_proven) all_proven = __ballot(live && cnt > 0) == live_mask;
    if (m > (uint32_t)kTol) {
        double v;
        if (vi != kNoLevel && all_proven) {
            v = level_f;
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
            int64_t vg = (v >= 0.0 && v < 9.0e18) ? (int64_t)v : -1;
            if (!bracketed && vg < 0) {
                const uint64_t head = live ? slot_cost(rail, A, l, 0) : ~0ull;
                const uint64_t alone = live ? slot_cost(rail, A, l, m - 1) : ~0ull;
                lo = (int64_t)uniform64(wave_reduce64(head, R, OpMin{})) - 1;
                hi = (int64_t)uniform64(wave_reduce64(alone, R, OpMin{}));
                bracketed = true;
            }
            if (bracketed && (iter >= 8 || vg <= lo || vg >= hi)) {   // guess unusable: bisect
                vg = lo + (hi - lo) / 2;
                if (vg <= lo) vg = hi;
            }
            const uint32_t kk = live ? slots_upto_fast(rail, A, l, inv_l, vg, m) : 0;
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
            if (miss > 0) { if (vg > lo) lo = vg; } else { if (vg < hi) hi = vg; }
            if (hi - lo == 1) {
                // the whole deficit sits at cost `hi`: hand it out in rail order
                const uint32_t k_lo = live ? slots_upto(rail, A, l, inv_l, lo, m) : 0;
                const uint32_t k_hi = live ? slots_upto(rail, A, l, inv_l, hi, m) : 0;
                const uint64_t below = uniform64(wave_reduce64(k_lo, R, OpAdd{}));
                uint64_t tie = k_hi - k_lo, inc = tie;
#pragma unroll
                for (int d = 1; d < kWide; d <<= 1) {
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
            const bool near = live && (kk > 0 || slot_cost(rail, A, l, 0) <= (uint64_t)(vg < 0 ? 0 : vg) + 1);
            double rate = wave_sum_f64(near ? G : 0.0, R);
            if (!(rate > 0.0)) rate = wave_sum_f64(G, R);
            v = __longlong_as_double((long long)uniform64(
                (uint64_t)__double_as_longlong((double)vg + (double)miss * (double)l / rate)));
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
    // only the slot count (low half) and the "every rail has a slot" flag (bit 32) go back: the caller derives its
    // state from the count, so that the loop's registers are not tied to those of the calling convention
    return (uint64_t)k | ((uint64_t)(all_proven ? 1u : 0u) << 32);
}

// Run records reach the chain through a ring of blocks in LDS, kWide records a block, one per lane, each as
// two 16-byte halves {len, m, level} and {level_f, inv_len}.  A second wavefront of the workgroup, the feeder,
// copies them there from global memory several blocks ahead.  A load that the chain issued itself would have to
// be awaited through the counter its row stores also use, that is, at once and at full memory latency per block,
// which is long while another batch's copies saturate the memory.  `filled` counts the blocks the feeder has
// written, `taken` those the chain has read; the feeder stays at most kRingBlocks ahead, the chain waits only
// for a block that is not there yet.  Neither wait depends on the waiting wavefront itself, and both loops end
// with the run table.
typedef uint32_t Quad __attribute__((ext_vector_type(4)));
constexpr int kRingBlocks = 8;
static_assert(sizeof(RunRec) == 32, "a run record is two 16-byte halves");

template <int kWide>
struct RecordRing {
    Quad lo[kRingBlocks][kWide];
    Quad hi[kRingBlocks][kWide];
    uint32_t filled;
    uint32_t taken;
};

// First instruction of both roles, before the workgroup's barrier.
template <int kWide>
__device__ __forceinline__ void ring_reset(RecordRing<kWide>& ring)
{
    if (threadIdx.x == 0) { ring.filled = 0; ring.taken = 0; }
}

template <int kWide>
__device__ __forceinline__ void feed_records(const BatchDev& b, const RunRec* __restrict__ recs, RecordRing<kWide>& ring, int lane)
{
    if (lane >= kWide) return;
    const uint64_t n_runs = b.plan->n_runs;
    const Quad* src = reinterpret_cast<const Quad*>(recs);
    for (uint64_t j = 0; j * kWide < n_runs; ++j) {
        while (__hip_atomic_load(&ring.taken, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) + (uint32_t)kRingBlocks <= (uint32_t)j)
            __builtin_amdgcn_s_sleep(4);
        const uint64_t r = j * kWide + lane < n_runs ? j * kWide + lane : n_runs;      // the table ends with a spare record
        const Quad lo = src[2 * r], hi = src[2 * r + 1];
        ring.lo[j % kRingBlocks][lane] = lo;
        ring.hi[j % kRingBlocks][lane] = hi;
        __hip_atomic_store(&ring.filled, (uint32_t)j + 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
    }
}

template <int kWide, bool kFar>
__device__ __forceinline__ void bind_chain(const BatchDev& b, const RailParams& rp, int mode, RecordRing<kWide>& ring)
{
    const int lane = threadIdx.x;
    if (lane >= kWide) return;
    constexpr int R = kWide;                                  // reduction width
    const int n_rails = (int)rp.n_rails;
    const bool live = lane < n_rails && ((rp.admitted >> lane) & 1);
    const uint64_t live_mask = __ballot(live);
    Rail rail;
    rail.c0 = rp.c0[lane];
    rail.c1 = live ? (uint32_t)rp.c1[lane] : 1u;
    rail.inv_c1 = 1.0 / (double)rail.c1;
    const double G = live ? 65536.0 * rail.inv_c1 : 0.0;      // bytes the rail absorbs per picosecond
    const double g = (double)rail.c0 * G;                     // its fixed latency expressed in bytes
    uint64_t T = 0;
    uint32_t cnt = 0;                                         // a batch holds fewer than 2^32 - 1 slices
    uint64_t n_before = 0;
    if (mode & kBindAfterRotation) {          // the rotation pass went first: its bytes are queued and staged ahead
        T = b.plan->Tr[lane];
        cnt = (uint32_t)b.plan->cr[lane];
        n_before = b.plan->n_retry;
    }
    const uint64_t A_less_T = rp.A[lane];                     // A = A_less_T + T at any time
    uint64_t P = (A_less_T + T) * (uint64_t)rail.c1;          // exact: (max A + pending bytes) * max c1 < 2^63
    // xmax(v) - A, the bytes the rail may still take up to cost level v, is estimated as v * G + Bd
    double Bd = (1.0 - (double)rail.c0) * G - (double)(A_less_T + T);
    const uint64_t n_runs = b.plan->n_runs;
    const uint32_t stride = b.run_stride;
    uint64_t* row_T = b.run_T + lane;
    uint32_t* row_K = b.run_K + lane;

    bool all_proven = false;                                  // every admitted rail has received a slot
    // cost level of the last run that went down the lean path: single slices that follow are compared
    // relative to it with 32-bit keys
    uint64_t ref_level = kNoLevel;
    const uint32_t lane_rev = 63u - (uint32_t)lane;

    // One slice of l bytes: plain argmin.  Near a known level the costs are compared as 32-bit keys
    // (cost - level + 2^24) << 6 | lane; a rail far above the window gets a far key, a rail below it key 0, and a
    // winning key below 64 or a far one sends the slice to the 64-bit compare, as does an unknown level.
    // Returns 1 in the winning lane.
    auto bind_single = [&](uint32_t l) -> uint32_t {
        const uint64_t p_one = P + (uint64_t)l * rail.c1;
        const uint64_t cost = rail.c0 + (p_one >> 16);
        int win = 0;
        bool keyed = ref_level != kNoLevel;
        if (__builtin_expect(keyed, 1)) {
            const uint64_t rel = cost - ref_level + (kRelSpan >> 1);
            uint32_t key;
            if constexpr (kFar) {
                const uint32_t near_key = rel < kRelSpan ? (((uint32_t)rel << 6) | (uint32_t)lane) : kFarKey | (uint32_t)lane;
                key = live ? ((int64_t)rel < 0 ? 0u : near_key) : kNoKey;
            } else {
                key = live ? (rel < kRelSpan ? (((uint32_t)rel << 6) | (uint32_t)lane) : 0u) : kNoKey;
            }
            const uint32_t best = wave_min_key<R>(key);
            win = (int)(best & 63u);
            keyed = best - 64u < kFarKey - 64u;
        }
        if (__builtin_expect(!keyed, 0)) win = argmin_cost(cost, live, lane, R);
        const bool mine = lane == win;
        if (mine) {
            P = p_one;
            T += l;
            cnt += 1u;
            Bd -= (double)l;
        }
        return mine ? 1u : 0u;
    };

    // A run of m >= 2 slices of l bytes with estimated end level vi: slots per rail.
    auto bind_run = [&](uint32_t l, uint32_t m, uint64_t vi, double level_f, double inv_l) -> uint32_t {
        const uint64_t lc1 = (uint64_t)l * rail.c1;           // cost numerator of one slice on this rail
        if (__builtin_expect(vi != kNoLevel, 1)) {          // a record carries a level only for kTol < m < kLeanRunMax
            // Lean path.  Slots at or below the level, per rail: slot j is iff j + 1 < kf, so the count is
            // ceil(kf) - 1, taken as trunc(kf - 1e-6) (an exactly integer kf, common when all lengths are
            // multiples of a power of two, must not count, hence the small bias against rounding noise).  The
            // estimate is confirmed by the integer cost of the slot below (last one taken), which must not exceed
            // the level, and of the slot above (first one free), which must; a count beyond the run's length
            // fails the same test.  A rail whose first slot lies far above the level (a long queue) takes no
            // slot and stays out of the repair through its far key.
            const double kf = fma(fma(level_f, G, Bd), inv_l, -1.0e-6);
            uint32_t kk;                                                          // trunc(kf); below zero gives 0, above 2^32 - 1 saturates
            asm("v_cvt_u32_f64_e32 %0, %1" : "=v"(kk) : "v"(kf));
            // kk * lc1 from a 32 x 32 -> 64 product and one 32-bit product for the high half (sums are modulo 2^64,
            // as the exact value fits by the plan's precondition whenever kk is a count that the test below accepts)
            uint64_t p_prev = P + (uint64_t)kk * (uint32_t)lc1;                  // slot kk-1 ends here
            p_prev += (uint64_t)((uint32_t)(lc1 >> 32) * kk) << 32;
            uint64_t p_next = p_prev + lc1;                                       // slot kk ends here
            // costs relative to the level, signed: the first free slot must lie above it (up >= 1), the last taken
            // slot not above it (below <= 0)
            const int64_t cv = (int64_t)(rail.c0 - vi);
            int64_t up = (int64_t)(p_next >> 16) + cv;
            int64_t below = (int64_t)(p_prev >> 16) + cv;
            // kFar: a rail may lie far on the harmless side of the level (far keys); otherwise every rail must
            // lie within the window, which saves the two selects per run where all rails stay close to the level
            const bool off = kFar ? live & ((kk > m) | ((kk < m) & (up < 1)) | ((kk > 0) & (below > 0)))
                                  : live & ((kk > m) | ((kk < m) & ((uint64_t)(up - 1) >= kRelSpan - 1)) |
                                            ((kk > 0) & ((uint64_t)(below + (int64_t)(kRelSpan - 1)) >= kRelSpan)));
            auto up_key = [&]() -> uint32_t {
                return up < (int64_t)kRelSpan ? (((uint32_t)up << 6) | (uint32_t)lane) : kFarKey | (uint32_t)lane;
            };
            auto down_key = [&]() -> uint32_t {
                return below > -(int64_t)kRelSpan ? (((0u - (uint32_t)below) << 6) | lane_rev) : kFarKey | lane_rev;
            };
            {   // a lane that is off adds kOffMark to the slot sum, which then misses m by more than any repair covers
                // three reductions side by side: slots taken, cheapest free slot, dearest taken slot
                // (ties: the free slot of the lowest rail is next, the taken slot of the highest rail is last)
                uint32_t key_up = (live & (kk < m)) ? (kFar ? up_key() : (((uint32_t)up << 6) | (uint32_t)lane)) : kNoKey;
                uint32_t key_down = (live & (kk > 0)) ? (kFar ? down_key() : (((0u - (uint32_t)below) << 6) | lane_rev)) : kNoKey;
                const uint32_t sum_r = wave_reduce32(off ? kOffMark : kk, R, Add32{});
                uint32_t up_r = wave_reduce32(key_up, R, Min32{});
                uint32_t down_r = wave_reduce32(key_down, R, Min32{});
                int miss = (int)m - (int)(uint32_t)__builtin_amdgcn_readfirstlane((int)sum_r);
                if (__builtin_expect(miss >= -kTol && miss <= kTol, 1)) {
                    // repair one slot at a time: add the cheapest free slot / drop the dearest taken slot; the
                    // first step's winners are already known, further steps redo one reduction each
                    // (true: done; false: no near candidate, start over in the general path)
                    auto repair = [&]() -> bool {
                        if (miss > 0) {
                            for (int need = miss;;) {
                                const uint32_t best = (uint32_t)__builtin_amdgcn_readfirstlane((int)up_r);
                                if (best >= kFarKey) return false;
                                if (lane == (int)(best & 63u)) {
                                    ++kk;
                                    p_prev = p_next;
                                    p_next += lc1;
                                    up = (int64_t)(p_next >> 16) + cv;
                                    key_up = kk < m ? up_key() : kNoKey;
                                }
                                if (--need == 0) return true;
                                up_r = wave_reduce32(key_up, R, Min32{});
                            }
                        }
                        for (int drop = -miss;;) {
                            const uint32_t best = (uint32_t)__builtin_amdgcn_readfirstlane((int)down_r);
                            if (best >= kFarKey) return false;
                            if (lane == 63 - (int)(best & 63u)) {
                                --kk;
                                p_next = p_prev;
                                p_prev -= lc1;
                                below = (int64_t)(p_prev >> 16) + cv;
                                key_down = kk > 0 ? down_key() : kNoKey;
                            }
                            if (--drop == 0) return true;
                            down_r = wave_reduce32(key_down, R, Min32{});
                        }
                    };
                    const bool exact = miss == 0 || repair();
                    if (__builtin_expect(exact, 1)) {
                        P = p_prev;
                        T += (uint64_t)kk * l;
                        cnt += kk;
                        Bd = fma(-(double)kk, (double)l, Bd);
                        ref_level = vi;
                        return kk;
                    }
                }
            }
        }
        // General path (any state, any level), kept out of line so that the loop stays short.
        const uint64_t res = bind_run_general<kWide>(ChainVars{P, T, Bd, ref_level, cnt, all_proven ? 1u : 0u, 0u}, rail, G, g, live,
                                                     live_mask, A_less_T, lane, l, m, vi, level_f, inv_l);
        const uint32_t k = (uint32_t)res;
        all_proven = (res >> 32) != 0;
        T += (uint64_t)k * l;
        cnt += k;
        Bd = fma(-(double)k, (double)l, Bd);
        P = (A_less_T + T) * (uint64_t)rail.c1;
        ref_level = kNoLevel;
        return k;
    };

    auto put_row = [&](uint64_t T_before, uint32_t k) {
        *row_T = T_before;
        *row_K = k;
        row_T += stride;
        row_K += stride;
    };

    auto pair64 = [](uint32_t lo, uint32_t hi, int t) -> uint64_t {
        return ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)hi, t) << 32) | (uint32_t)__builtin_amdgcn_readlane((int)lo, t);
    };

    // Block j of kWide records, one per lane, from the ring the feeder wavefront keeps filled.
    auto take_block = [&](uint64_t j, Quad& lo, Quad& hi) {
        while (__hip_atomic_load(&ring.filled, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) <= (uint32_t)j)
            __builtin_amdgcn_s_sleep(1);
        lo = ring.lo[j % kRingBlocks][lane];
        hi = ring.hi[j % kRingBlocks][lane];
        if (lane == 0) __hip_atomic_store(&ring.taken, (uint32_t)j + 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
    };
    Quad mine_lo = {0, 0, 0, 0}, mine_hi = {0, 0, 0, 0};
    for (uint64_t blk = 0; blk < n_runs; blk += kWide) {
        take_block(blk / kWide, mine_lo, mine_hi);
        const int in_blk = (int)(n_runs - blk < (uint64_t)kWide ? n_runs - blk : (uint64_t)kWide);
        for (int t = 0; t < in_blk; ++t) {
            const uint32_t l = (uint32_t)__builtin_amdgcn_readlane((int)mine_lo.x, t);
            const uint32_t m = (uint32_t)__builtin_amdgcn_readlane((int)mine_lo.y, t);
            const uint64_t T_before = T;
            if (m == 1) {
                put_row(T_before, bind_single(l));
                continue;
            }
            put_row(T_before, bind_run(l, m, pair64(mine_lo.z, mine_lo.w, t), __longlong_as_double((long long)pair64(mine_hi.x, mine_hi.y, t)),
                                       __longlong_as_double((long long)pair64(mine_hi.z, mine_hi.w, t))));
            // the single slice that usually follows a run (a transfer's tail) is bound in the same round
            if (t + 1 < in_blk && (uint32_t)__builtin_amdgcn_readlane((int)mine_lo.y, t + 1) == 1u) {
                ++t;
                const uint32_t l_tail = (uint32_t)__builtin_amdgcn_readlane((int)mine_lo.x, t);
                const uint64_t T_mid = T;
                put_row(T_mid, bind_single(l_tail));
            }
        }
    }

    // per-rail totals and staging region bases (exclusive sum of 256-byte-rounded totals)
    const uint64_t rounded = (T + 255) & ~255ull;
    uint64_t inc = rounded;
#pragma unroll
    for (int d = 1; d < kWide; d <<= 1) {
        uint64_t up = (uint64_t)__shfl_up((unsigned long long)inc, d, 64);
        if (lane >= d) inc += up;
    }
    PlanState* ps = b.plan;
    ps->T[lane] = T;
    ps->cnt[lane] = cnt;
    ps->A_after[lane] = A_less_T + T;
    ps->base[lane] = inc - rounded;
    if (lane == 0) ps->n_bound = ps->n_pending + n_before;
}

// Wavefront 0 walks the chain, wavefront 1 feeds it the run records.
template <int kWide, bool kFar>
__global__ void __launch_bounds__(128) bind_chain_kernel(BatchDev b, RailParams rp, int mode,
                                                         const RunRec* __restrict__ recs)
{
    __shared__ RecordRing<kWide> ring;
    ring_reset(ring);
    __syncthreads();
    if (threadIdx.x < 64) bind_chain<kWide, kFar>(b, rp, mode, ring);
    else feed_records<kWide>(b, recs, ring, (int)threadIdx.x - 64);
}

// The chain is one wavefront; the tile tables of the copy kernels depend on the slice table only, not
// on the binding.  On a first plan both go into one launch: workgroup 0 walks the chain, the others
// build the tables, so the tables cost no time of their own.
template <int kWide, bool kFar>
__global__ void __launch_bounds__(256) bind_chain_tables_kernel(BatchDev b, RailParams rp, int mode,
                                                                const RunRec* __restrict__ recs)
{
    __shared__ RecordRing<kWide> ring;
    if (blockIdx.x == 0) {
        ring_reset(ring);
        __syncthreads();
        if (threadIdx.x < 64) bind_chain<kWide, kFar>(b, rp, mode, ring);
        else if (threadIdx.x < 128) feed_records<kWide>(b, recs, ring, (int)threadIdx.x - 64);
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
    // run ids (a scan of the run heads) and the bytes bound before every pending position, in the same launches
    RunHead head{b.s_len, use_pending ? b.pending : nullptr, &b.plan->n_pending};
    PendingLen plen{b.s_len, use_pending ? b.pending : nullptr, &b.plan->n_pending};
    hipError_t e = exclusive_scan2(head, plen, b.n_slices, b.n_slices, b.scan_tmp, b.len_pre, b.scan_partials, b.scan_partials2, s);
    if (e != hipSuccess) return e;
    uint64_t blocks = (b.n_slices + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(run_table_kernel, dim3((uint32_t)blocks), dim3(256), 0, s, b, up);
    // one record per run for the chain
    hipLaunchKernelGGL(run_records_kernel, dim3((b.run_capacity + 1 + 255) / 256), dim3(256), 0, s, b, rp, mode);
    // Which variant of the chain: when the rails' head costs lie close together at the start (idle rails, short
    // queues) and no rail's slots are far apart, all rails stay close to the common level throughout and the
    // variant without far keys is a few percent faster; otherwise (long queues, bytes of a rotation pass ahead,
    // large slices on a slow rail) rails may sit far from the level.  Either variant is exact for any input.
    bool far_keys = (mode & kBindAfterRotation) != 0;
    {
        uint64_t lo = ~0ull, hi = 0;
        for (uint32_t d = 0; d < rp.n_rails; ++d) {
            if (!((rp.admitted >> d) & 1)) continue;
            const uint64_t h = rp.c0[d] + ((rp.A[d] * rp.c1[d]) >> 16);       // in range by the plan's precondition
            lo = h < lo ? h : lo;
            hi = h > hi ? h : hi;
            // a rail whose slots are a large part of the window apart often has its next slot outside it
            if (((b.slice_bytes * rp.c1[d]) >> 16) >= (kRelSpan >> 2)) far_keys = true;
        }
        if (hi >= lo && hi - lo >= (kRelSpan >> 1)) far_keys = true;
    }
    auto launch_chain = [&](auto wide, auto far) {
        constexpr int kW = decltype(wide)::value;
        constexpr bool kF = decltype(far)::value;
        if (mode & kBindBuildTables)
            hipLaunchKernelGGL((bind_chain_tables_kernel<kW, kF>), dim3(1 + tile_table_blocks(b)), dim3(256), 0, s, b, rp, mode, b.run_rec);
        else
            hipLaunchKernelGGL((bind_chain_kernel<kW, kF>), dim3(1), dim3(128), 0, s, b, rp, mode, b.run_rec);
    };
    auto launch_width = [&](auto far) {
        if (rp.n_rails <= 16)      launch_chain(std::integral_constant<int, 16>{}, far);
        else if (rp.n_rails <= 32) launch_chain(std::integral_constant<int, 32>{}, far);
        else                       launch_chain(std::integral_constant<int, 64>{}, far);
    };
    if (far_keys) launch_width(std::true_type{});
    else          launch_width(std::false_type{});
    hipLaunchKernelGGL(bind_emit_kernel, dim3((uint32_t)blocks), dim3(256), 0, s, b, rp, up);
    return hipGetLastError();
}

}  // namespace tent
