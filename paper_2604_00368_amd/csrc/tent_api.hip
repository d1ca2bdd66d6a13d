// Host runtime behind the C ABI: argument validation, device tables, rail-state conversion and
// kernel sequencing.  Every step of the hot path itself runs in the HIP kernels of this library.
#include <algorithm>
#include <cstring>
#include <mutex>
#include <thread>
#include <new>
#include <utility>
#include <vector>

#include "tent_internal.h"

using namespace tent;

// Static workspace of tent_declare_static: callers that must not allocate get their batch's tables
// here.  One copy per GPU, held until the process ends.  In host code the array's name is only a
// stand-in: its address on a GPU is looked up once, with that GPU current, and host code uses the
// looked-up pointer and nothing else.
static __device__ __align__(256) unsigned char scratch[TENT_STATIC_WORKSPACE_BYTES];

namespace {

struct Segment { uint8_t* base; uint64_t len; };

// A stream on which work of a batch was enqueued, with an event recorded after the latest such work.
struct StreamMark {
    hipStream_t stream = nullptr;
    hipEvent_t event = nullptr;
    bool used = false;
};
constexpr int kMarks = 4;

struct Batch {
    bool alive = false;
    bool planned = false;        // a plan has been enqueued since declare / reset
    bool has_done = false;       // execute ran since declare / reset: DONE slices may exist
    bool has_retry = false;      // a rail failed since declare / reset: slices with a retry count may exist
    bool broken = false;         // an execute failed after its slices were marked DONE: only reset or release help
    uint64_t bound_hint = 0;     // upper bound on the number of BOUND slices, as far as the host knows
    uint64_t tile_hint = ~0ull;  // upper bound on the copy tiles of the BOUND slices, as far as the host knows
    uint32_t generation = 0;
    uint64_t payload = 0;
    uint64_t max_req_slices = 0; // most slices any one transfer has
    RailParams last_rails{};     // telemetry of the last plan (for the rail simulator)
    uint32_t last_lat_ns[TENT_MAX_RAILS] = {};
    // The last execute's bookkeeping (staging addresses, tile lists, DONE marks) ends at prep_event on
    // exec_stream; its copies, which follow, read none of what a re-plan writes, and end at done_event.
    hipStream_t exec_stream = nullptr;
    bool prep_recorded = false;
    bool done_recorded = false;
    // The declaration's device work (descriptor upload, address sort, overlap check) runs on the
    // context's own stream and ends at decl_event; `verdict` (pinned host memory) then holds the
    // overlap check's result.
    bool decl_pending = false;
    uint32_t* overlap_dev = nullptr;
    // Device memory of the tables: an allocation of the batch's own, or the library's static workspace.
    void* block = nullptr;
    uint64_t block_bytes = 0;
    bool in_static = false;
    uint64_t static_generation = 0;
    bool marks_lost = false;     // work was enqueued that no mark covers: waiting for the batch means waiting for the device
    BatchDev dev{};

    // Created once per slot and kept across the batches that use it.
    hipEvent_t prep_event = nullptr, done_event = nullptr, decl_event = nullptr;
    uint32_t* verdict = nullptr;
    StreamMark marks[kMarks];
};

// Event pairs recorded around the launches of one stage since the last tent_get_timings.
struct Timing {
    std::vector<std::pair<hipEvent_t, hipEvent_t>> pool;   // every pair ever created for the stage
    size_t used = 0;                                        // pairs recorded since the last read-out
};

struct Block { void* ptr; uint64_t bytes; };

}  // namespace

struct tent_ctx {
    int device = 0;
    tent_config cfg{};
    uint32_t max_rails = TENT_MAX_RAILS;
    std::vector<Segment> segments;
    uint64_t* seg_base_dev = nullptr;       // device table of segment base addresses
    uint32_t seg_capacity = 0;
    std::vector<Batch> batches;
    Batch static_batch;                     // the one batch whose tables live in the static workspace
    PlanState* host_plan = nullptr;         // pinned read-back buffer
    hipStream_t aux_stream = nullptr;       // second stream of the pipelined bounded execute (default priority)
    std::vector<hipEvent_t> sync_events;    // ordering events of the pipelined bounded execute, reused
    // tent_declare: its device work runs on a stream of the library's own, so that it neither waits for
    // nor holds up the caller's streams; host arrays travel through two pinned buffers used in turn.
    hipStream_t decl_stream = nullptr;
    uint8_t* stage[2] = {nullptr, nullptr};
    uint64_t stage_bytes[2] = {0, 0};
    hipEvent_t stage_event[2] = {nullptr, nullptr};
    bool stage_busy[2] = {false, false};
    uint32_t stage_turn = 0;
    void* order_ws = nullptr;               // workspace of the address sort, grown when a declaration needs more
    uint64_t order_ws_bytes = 0;
    std::vector<Block> spare;               // table allocations of released batches, handed to later declarations
    Timing timing[TENT_T_COUNT];
};

namespace {

constexpr uint32_t kMaxSegments = 4096;
constexpr size_t kMaxTimedIntervals = 1u << 16;   // per stage, between two tent_get_timings calls
constexpr size_t kSpareBlocks = 4;                // released table allocations kept for reuse
constexpr uint64_t kStageInitial = 1ull << 20;    // pinned bytes per staging buffer at tent_create
constexpr uint32_t kStaticSlot = 0xFFFFFFFFu;     // slot field of a handle whose tables live in the static workspace

constexpr uint64_t kStaticBytes = TENT_STATIC_WORKSPACE_BYTES;
struct StaticArea {
    void* ptr = nullptr;         // device address of `scratch` on this GPU
    uint64_t generation = 0;     // goes up with every tent_declare_static on this GPU: older static batches are dead
};
constexpr int kMaxDevices = 64;
StaticArea g_static[kMaxDevices];
std::mutex g_static_mutex;

#define HIP_TRY(expr) do { if ((expr) != hipSuccess) return TENT_ERR_HIP; } while (0)

struct DeviceGuard {
    int prev = -1;
    bool ok = true;
    explicit DeviceGuard(int dev) {
        if (hipGetDevice(&prev) != hipSuccess) { ok = false; return; }
        if (prev != dev && hipSetDevice(dev) != hipSuccess) ok = false;
        target = dev;
    }
    ~DeviceGuard() { if (prev >= 0 && prev != target) (void)hipSetDevice(prev); }
    int target = -1;
};

bool capturing(hipStream_t s)
{
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(s, &cap) != hipSuccess) { (void)hipGetLastError(); return false; }
    return cap != hipStreamCaptureStatusNone;
}

// Remember that work of the batch was just enqueued on `s` (nothing is recorded into a stream that is
// being captured into a graph: such work is only known to be over when the device is idle).
void note_stream(Batch& b, hipStream_t s)
{
    if (capturing(s)) { b.marks_lost = true; return; }
    StreamMark* slot = nullptr;
    for (StreamMark& m : b.marks) {
        if (m.used && m.stream == s) { slot = &m; break; }
        if (!m.used && !slot) slot = &m;
    }
    if (!slot || !slot->event || hipEventRecord(slot->event, s) != hipSuccess) {
        (void)hipGetLastError();
        b.marks_lost = true;
        return;
    }
    slot->stream = s;
    slot->used = true;
}

// Records the batch's stream use when an entry point returns, whichever way it returns.
struct StreamNote {
    Batch& b;
    hipStream_t s;
    StreamNote(Batch& batch, hipStream_t stream) : b(batch), s(stream) {}
    ~StreamNote() { note_stream(b, s); }
};

// Host-side wait for everything that was enqueued for the batch.
void wait_batch_idle(Batch& b)
{
    if (b.decl_pending) (void)hipEventSynchronize(b.decl_event);
    for (StreamMark& m : b.marks)
        if (m.used) (void)hipEventSynchronize(m.event);
    if (b.marks_lost) (void)hipDeviceSynchronize();
    (void)hipGetLastError();
}

bool init_slot(Batch& b)
{
    bool ok = hipEventCreateWithFlags(&b.prep_event, hipEventDisableTiming) == hipSuccess &&
              hipEventCreateWithFlags(&b.done_event, hipEventDisableTiming) == hipSuccess &&
              hipEventCreateWithFlags(&b.decl_event, hipEventDisableTiming) == hipSuccess &&
              hipHostMalloc((void**)&b.verdict, 64, hipHostMallocDefault) == hipSuccess;
    for (StreamMark& m : b.marks)
        ok = ok && hipEventCreateWithFlags(&m.event, hipEventDisableTiming) == hipSuccess;
    if (!ok) (void)hipGetLastError();
    return ok;
}

void destroy_slot(Batch& b)
{
    if (b.prep_event) (void)hipEventDestroy(b.prep_event);
    if (b.done_event) (void)hipEventDestroy(b.done_event);
    if (b.decl_event) (void)hipEventDestroy(b.decl_event);
    if (b.verdict) (void)hipHostFree(b.verdict);
    for (StreamMark& m : b.marks)
        if (m.event) (void)hipEventDestroy(m.event);
    b.prep_event = b.done_event = b.decl_event = nullptr;
    b.verdict = nullptr;
    for (StreamMark& m : b.marks) m = StreamMark{};
}

// Start a new batch in a slot: everything but the slot's events, its pinned word and its generation starts afresh.
void renew_slot(Batch& b)
{
    Batch fresh;
    fresh.generation = b.generation + 1;
    fresh.prep_event = b.prep_event;
    fresh.done_event = b.done_event;
    fresh.decl_event = b.decl_event;
    fresh.verdict = b.verdict;
    for (int k = 0; k < kMarks; ++k) fresh.marks[k].event = b.marks[k].event;
    b = fresh;
}

// The batch's tables go back to the context (an allocation is kept for a later declaration of
// similar size; what the context cannot keep is freed).  The caller has waited for the batch.
void free_batch(tent_ctx* ctx, Batch& b)
{
    if (b.block && !b.in_static) {
        bool kept = false;
        if (ctx->spare.size() < kSpareBlocks) {
            try { ctx->spare.push_back({b.block, b.block_bytes}); kept = true; } catch (const std::bad_alloc&) {}
        } else {
            // keep the larger allocations: replace the smallest spare one if this one is larger
            size_t least = 0;
            for (size_t k = 1; k < ctx->spare.size(); ++k)
                if (ctx->spare[k].bytes < ctx->spare[least].bytes) least = k;
            if (ctx->spare[least].bytes < b.block_bytes) {
                (void)hipFree(ctx->spare[least].ptr);
                ctx->spare[least] = {b.block, b.block_bytes};
                kept = true;
            }
        }
        if (!kept) (void)hipFree(b.block);
    }
    b.block = nullptr;
    b.block_bytes = 0;
    b.alive = false;
    b.decl_pending = false;
    b.prep_recorded = b.done_recorded = false;
    b.marks_lost = false;
    for (StreamMark& m : b.marks) { m.used = false; m.stream = nullptr; }
    b.dev = BatchDev{};
}

Batch* find_batch(tent_ctx* ctx, tent_batch_t h)
{
    const uint64_t idx = (h & 0xFFFFFFFFull);
    const uint32_t gen = (uint32_t)(h >> 32);
    if (idx == kStaticSlot) {
        Batch* b = &ctx->static_batch;
        if (!b->alive || b->generation != gen) return nullptr;
        // a later tent_declare_static on this GPU (from any context) has taken the workspace over
        uint64_t now = 0;
        {
            std::lock_guard<std::mutex> lk(g_static_mutex);
            now = ctx->device < kMaxDevices ? g_static[ctx->device].generation : 0;
        }
        if (now != b->static_generation) { b->alive = false; return nullptr; }
        return b;
    }
    if (idx == 0 || idx > ctx->batches.size()) return nullptr;
    Batch* b = &ctx->batches[idx - 1];
    return (b->alive && b->generation == gen) ? b : nullptr;
}

// Every per-batch table is carved from ONE range of device memory: a declaration asks for about fifty
// arrays, and fifty allocator calls cost more than everything else a declaration does.  The requests
// are collected first and then laid out at 256-byte aligned offsets.
struct Carver {
    struct Want { void** slot; uint64_t bytes; };
    static constexpr int kMost = 80;
    Want wants[kMost];
    int n = 0;
    bool overflow = false;
    template <class T>
    void want(T** out, uint64_t count)
    {
        if (n == kMost) { overflow = true; return; }
        wants[n++] = {reinterpret_cast<void**>(out), std::max<uint64_t>(count, 1) * sizeof(T)};
    }
    uint64_t total() const
    {
        uint64_t t = 0;
        for (int k = 0; k < n; ++k) t += (wants[k].bytes + 255) & ~255ull;
        return t;
    }
    void place(void* base) const
    {
        uint64_t at = 0;
        for (int k = 0; k < n; ++k) {
            *wants[k].slot = static_cast<char*>(base) + at;
            at += (wants[k].bytes + 255) & ~255ull;
        }
    }
};

// Device memory for a batch's tables: a spare allocation of a released batch when one is large enough
// (and not absurdly larger), else a new one.
int acquire_block(tent_ctx* ctx, uint64_t need, void** out, uint64_t* out_bytes)
{
    size_t best = ctx->spare.size();
    for (size_t k = 0; k < ctx->spare.size(); ++k) {
        const uint64_t have = ctx->spare[k].bytes;
        if (have >= need && have <= 4 * need + (1ull << 20) &&
            (best == ctx->spare.size() || have < ctx->spare[best].bytes))
            best = k;
    }
    if (best != ctx->spare.size()) {
        *out = ctx->spare[best].ptr;
        *out_bytes = ctx->spare[best].bytes;
        ctx->spare.erase(ctx->spare.begin() + (long)best);
        return TENT_OK;
    }
    void* p = nullptr;
    if (hipMalloc(&p, need) != hipSuccess) {
        (void)hipGetLastError();
        return TENT_ERR_NOMEM;
    }
    *out = p;
    *out_bytes = need;
    return TENT_OK;
}

// Pinned buffer for the host arrays of one declaration: the two buffers are used in turn, so a
// declaration seldom has to wait for the upload of the one before.  With `may_grow` unset a buffer
// that is too small is reported (nullptr) instead of being replaced.
uint8_t* acquire_stage(tent_ctx* ctx, uint64_t need, bool may_grow, int* which)
{
    const int k = (int)(ctx->stage_turn & 1);
    if (ctx->stage_busy[k]) {
        (void)hipEventSynchronize(ctx->stage_event[k]);
        ctx->stage_busy[k] = false;
    }
    if (ctx->stage_bytes[k] < need) {
        if (!may_grow) return nullptr;
        uint8_t* p = nullptr;
        const uint64_t want = need + need / 4;
        if (hipHostMalloc((void**)&p, want, hipHostMallocDefault) != hipSuccess) { (void)hipGetLastError(); return nullptr; }
        if (ctx->stage[k]) (void)hipHostFree(ctx->stage[k]);
        ctx->stage[k] = p;
        ctx->stage_bytes[k] = want;
    }
    ++ctx->stage_turn;
    *which = k;
    return ctx->stage[k];
}

// Host array -> device through the pinned buffer whose turn it is, one buffer-full at a time, waiting
// for each piece (used when the buffer cannot hold a declaration's arrays and must not be replaced).
bool upload_in_pieces(tent_ctx* ctx, void* dev, const void* host, uint64_t bytes)
{
    const int k = (int)(ctx->stage_turn & 1);
    if (ctx->stage_busy[k]) {
        if (hipEventSynchronize(ctx->stage_event[k]) != hipSuccess) return false;
        ctx->stage_busy[k] = false;
    }
    const uint64_t cap = ctx->stage_bytes[k];
    if (cap == 0) return false;
    for (uint64_t at = 0; at < bytes; at += cap) {
        const uint64_t n = std::min(cap, bytes - at);
        std::memcpy(ctx->stage[k], static_cast<const uint8_t*>(host) + at, n);
        if (hipMemcpyAsync(static_cast<uint8_t*>(dev) + at, ctx->stage[k], n, hipMemcpyHostToDevice, ctx->decl_stream) != hipSuccess ||
            hipStreamSynchronize(ctx->decl_stream) != hipSuccess)
            return false;
    }
    return true;
}

// CSR pointer arrays: start at 0, strictly increasing (no empty transfer).
bool pointers_ok(uint32_t n_desc, const uint32_t* p)
{
    if (p[0] != 0) return false;
    for (uint32_t j = 0; j < n_desc; ++j)
        if (p[j + 1] <= p[j]) return false;
    return true;
}

// Walk both extent lists of the transfers [j0, j1): structure, bounds, equal lengths; every extent is
// copied to `se_out` / `de_out` (if not null) on the way.
struct WalkResult {
    int rc = TENT_OK;
    uint64_t total = 0, slices = 0, bits = 0, most = 0;
};

void validate_range(const tent_ctx* ctx, uint32_t j0, uint32_t j1, const uint32_t* sp, const tent_extent* se,
                    const uint32_t* dp, const tent_extent* de, tent_extent* se_out, tent_extent* de_out, WalkResult* out)
{
    const uint64_t S = ctx->cfg.slice_bytes;
    const size_t n_seg = ctx->segments.size();
    const Segment* seg = ctx->segments.data();
    WalkResult r;
    for (uint32_t j = j0; j < j1; ++j) {
        uint64_t ls = 0, ld = 0;
        for (uint32_t e = sp[j]; e < sp[j + 1]; ++e) {
            const tent_extent x = se[e];
            if (x.len == 0 || x.seg >= n_seg) { r.rc = TENT_ERR_INVALID; *out = r; return; }
            const uint64_t seg_len = seg[x.seg].len;
            if (x.off > seg_len || x.len > seg_len - x.off) { r.rc = TENT_ERR_INVALID; *out = r; return; }
            if (se_out) se_out[e] = x;
            ls += x.len;
            r.bits |= x.len;
        }
        for (uint32_t e = dp[j]; e < dp[j + 1]; ++e) {
            const tent_extent x = de[e];
            if (x.len == 0 || x.seg >= n_seg) { r.rc = TENT_ERR_INVALID; *out = r; return; }
            const uint64_t seg_len = seg[x.seg].len;
            if (x.off > seg_len || x.len > seg_len - x.off) { r.rc = TENT_ERR_INVALID; *out = r; return; }
            if (de_out) de_out[e] = x;
            ld += x.len;
            r.bits |= x.len;
        }
        if (ls != ld) { r.rc = TENT_ERR_INVALID; *out = r; return; }
        r.total += ls;
        const uint64_t cnt = (ls + S - 1) / S;
        r.slices += cnt;
        r.most = std::max(r.most, cnt);
    }
    *out = r;
}

// The whole batch; also returns the payload and the number of slices the device splitter will produce.
// Large batches are walked by a few threads, each over a range of transfers with about the same number of
// extents: the walk streams some tens of megabytes and is the longest part of a declaration.
int validate(const tent_ctx* ctx, uint32_t n_desc, const uint32_t* sp, const tent_extent* se,
             const uint32_t* dp, const tent_extent* de, tent_extent* se_out, tent_extent* de_out,
             uint64_t* payload, uint64_t* n_slices, uint64_t* len_bits, uint64_t* max_req_slices, bool may_spawn)
{
    constexpr uint32_t kMaxWalkers = 4;
    constexpr uint64_t kExtentsPerWalker = 1ull << 16;
    const uint64_t n_ext = (uint64_t)sp[n_desc] + dp[n_desc];
    uint32_t walkers = (uint32_t)std::min<uint64_t>(kMaxWalkers, n_ext / kExtentsPerWalker);
    walkers = std::min(walkers, std::max(1u, std::thread::hardware_concurrency()));
    if (!may_spawn) walkers = 1;                       // a thread's stack is an allocation: not for callers that forbid them
    WalkResult part[kMaxWalkers];
    uint32_t used = 1;
    if (walkers >= 2) {
        // cut points: transfers at which the running count of extents passes k / walkers of the total
        uint32_t cut[kMaxWalkers + 1];
        cut[0] = 0;
        for (uint32_t k = 1; k < walkers; ++k) {
            const uint64_t want = n_ext * k / walkers;
            uint32_t lo = cut[k - 1], hi = n_desc;
            while (lo < hi) {
                const uint32_t mid = lo + (hi - lo) / 2;
                if ((uint64_t)sp[mid] + dp[mid] < want) lo = mid + 1; else hi = mid;
            }
            cut[k] = lo;
        }
        cut[walkers] = n_desc;
        std::thread th[kMaxWalkers];
        uint32_t started = 0;
        try {
            for (uint32_t k = 1; k < walkers; ++k) {
                th[k] = std::thread(validate_range, ctx, cut[k], cut[k + 1], sp, se, dp, de, se_out, de_out, &part[k]);
                ++started;
            }
        } catch (...) {
            // no more threads to be had: the ranges not handed out are walked here
        }
        validate_range(ctx, cut[0], cut[1], sp, se, dp, de, se_out, de_out, &part[0]);
        for (uint32_t k = 1; k <= started; ++k) th[k].join();
        for (uint32_t k = started + 1; k < walkers; ++k)
            validate_range(ctx, cut[k], cut[k + 1], sp, se, dp, de, se_out, de_out, &part[k]);
        used = walkers;
    } else {
        validate_range(ctx, 0, n_desc, sp, se, dp, de, se_out, de_out, &part[0]);
    }
    uint64_t total = 0, slices = 0, bits = 0, most = 0;
    for (uint32_t k = 0; k < used; ++k) {
        if (part[k].rc != TENT_OK) return part[k].rc;
        total += part[k].total;
        slices += part[k].slices;
        bits |= part[k].bits;
        most = std::max(most, part[k].most);
    }
    *payload = total;
    *n_slices = slices;
    *len_bits = bits;
    *max_req_slices = most;
    return TENT_OK;
}

// Brackets the launches of one stage with a pair of HIP events on the caller's stream.
struct StageTimer {
    hipEvent_t stop = nullptr;
    hipStream_t s;
    StageTimer(tent_ctx* c, int stage, hipStream_t stream) : s(stream)
    {
        if (!(c->cfg.flags & TENT_FLAG_PROFILE)) return;
        Timing& t = c->timing[stage];
        if (t.used >= kMaxTimedIntervals) return;          // nobody reads the timings: stop collecting
        if (t.used == t.pool.size()) {
            hipEvent_t a = nullptr, b = nullptr;
            if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) {
                if (a) (void)hipEventDestroy(a);
                return;
            }
            try { t.pool.emplace_back(a, b); } catch (const std::bad_alloc&) {
                (void)hipEventDestroy(a); (void)hipEventDestroy(b);
                return;
            }
        }
        (void)hipEventRecord(t.pool[t.used].first, s);
        stop = t.pool[t.used].second;
        ++t.used;
    }
    ~StageTimer() { if (stop) (void)hipEventRecord(stop, s); }
};

// A re-plan enqueued on another stream than the last execute's may overlap that execute's copies: it
// only has to come after the execute's bookkeeping.
hipError_t order_after_execute_bookkeeping(const Batch& b, hipStream_t s)
{
    if (!b.prep_recorded || s == b.exec_stream) return hipSuccess;
    return hipStreamWaitEvent(s, b.prep_event, 0);
}

// Marks the end of an execute's bookkeeping on its stream.  Nothing is recorded into a stream that is
// being captured into a graph; a graph holds its launches in stream order anyway.
hipError_t record_execute_bookkeeping(Batch& b, hipStream_t s)
{
    b.prep_recorded = false;
    b.done_recorded = false;
    if (capturing(s)) return hipSuccess;
    hipError_t e = hipEventRecord(b.prep_event, s);
    if (e != hipSuccess) return e;
    b.exec_stream = s;
    b.prep_recorded = true;
    return hipSuccess;
}

// Marks the end of an execute's copies on its stream: what batch-level completion waits for.
hipError_t record_execute_done(Batch& b, hipStream_t s)
{
    b.done_recorded = false;
    if (capturing(s)) return hipSuccess;
    hipError_t e = hipEventRecord(b.done_event, s);
    if (e != hipSuccess) return e;
    b.exec_stream = s;
    b.done_recorded = true;
    return hipSuccess;
}

// The first call that needs the batch's tables waits (on the host) for the declaration's device work
// and learns the verdict of the overlap check.  A batch that fails it is released.
int finish_declare(tent_ctx* ctx, Batch& b)
{
    if (!b.decl_pending) return TENT_OK;
    HIP_TRY(hipEventSynchronize(b.decl_event));
    b.decl_pending = false;
    if (*b.verdict != 0) {
        wait_batch_idle(b);
        free_batch(ctx, b);
        return TENT_ERR_INVALID;
    }
    return TENT_OK;
}

// Telemetry -> integer coefficients (Eq. 1 with the topology penalty folded in).
int convert_rails(const tent_rail_state* rails, uint32_t n_rails, uint64_t pending_bytes, RailParams* rp)
{
    std::memset(rp, 0, sizeof(*rp));
    rp->n_rails = n_rails;
    uint64_t max_c1 = 0, max_A = 0;
    for (uint32_t d = 0; d < n_rails; ++d) {
        const tent_rail_state& r = rails[d];
        if (r.health > 2) return TENT_ERR_INVALID;
        if (r.bw_MBps == 0) return TENT_ERR_RANGE;
        const uint64_t bp = (uint64_t)r.beta1_q8 * r.penalty_q8;
        // a degraded rail keeps half its weight: its predicted cost counts twice (Section 4.3)
        const uint64_t weight = r.health == 1 ? 2 : 1;
        const uint64_t c1 = weight * ((1000000ull * bp) / r.bw_MBps);
        if (c1 >= (1ull << 32)) return TENT_ERR_RANGE;
        rp->c1[d] = c1;
        rp->c0[d] = weight * (((uint64_t)r.lat_ns * 1000ull * r.penalty_q8) >> 8);
        rp->A[d] = r.queued_bytes;
        if (r.health != 2) {
            rp->admitted |= 1ull << d;
            max_c1 = std::max(max_c1, c1);
            max_A = std::max(max_A, r.queued_bytes);
        }
    }
    // (max A + pending bytes) * max c1 must stay below 2^63 so that no cost wraps
    const unsigned __int128 worst = ((unsigned __int128)max_A + pending_bytes) * max_c1;
    if (worst >= ((unsigned __int128)1 << 63)) return TENT_ERR_RANGE;
    return TENT_OK;
}

// tent_declare and tent_declare_static.  With `use_static` the tables and the sort's workspace are
// carved from the static workspace of the context's GPU and nothing is allocated, on the device or
// on the host.
int declare_impl(tent_ctx* ctx, uint32_t n_desc, const uint32_t* src_ptr, const tent_extent* src_ext,
                 const uint32_t* dst_ptr, const tent_extent* dst_ext, tent_batch_t* out, bool use_static)
{
    if (!ctx || !src_ptr || !src_ext || !dst_ptr || !dst_ext || !out || n_desc == 0) return TENT_ERR_INVALID;
    *out = 0;
    if (n_desc >= 0x7FFFFFFFu) return TENT_ERR_RANGE;
    if (!pointers_ok(n_desc, src_ptr) || !pointers_ok(n_desc, dst_ptr)) return TENT_ERR_INVALID;
    const uint64_t ns = src_ptr[n_desc], nd = dst_ptr[n_desc];
    if (ns + nd >= 0xFFFFFFFFull) return TENT_ERR_RANGE;
    DeviceGuard g(ctx->device);
    if (!g.ok) return TENT_ERR_HIP;

    // Host arrays -> pinned buffer (laid out as they will lie in the upload): both pointer arrays,
    // both extent lists, then the device view of the batch.
    const uint64_t ptr_bytes = ((uint64_t)n_desc + 1) * sizeof(uint32_t);
    const uint64_t o_sp = 0, o_dp = (o_sp + ptr_bytes + 15) & ~15ull, o_se = (o_dp + ptr_bytes + 15) & ~15ull;
    const uint64_t o_de = o_se + ns * sizeof(tent_extent), o_self = o_de + nd * sizeof(tent_extent);
    const uint64_t stage_need = o_self + sizeof(BatchDev);
    int which = -1;
    uint8_t* st = acquire_stage(ctx, stage_need, !use_static, &which);
    if (!st && !use_static) return TENT_ERR_NOMEM;

    uint64_t payload = 0, n_slices = 0, len_bits = 0, max_req_slices = 0;
    int rc = validate(ctx, n_desc, src_ptr, src_ext, dst_ptr, dst_ext, st ? (tent_extent*)(st + o_se) : nullptr,
                      st ? (tent_extent*)(st + o_de) : nullptr, &payload, &n_slices, &len_bits, &max_req_slices, !use_static);
    if (rc != TENT_OK) return rc;
    if (n_slices >= 0xFFFFFFFEull) return TENT_ERR_RANGE;

    Batch* slot_b = nullptr;
    size_t slot = 0;
    if (use_static) {
        slot_b = &ctx->static_batch;
        if (slot_b->alive) {                              // the context's earlier static batch gives way
            wait_batch_idle(*slot_b);
            free_batch(ctx, *slot_b);
        }
    } else {
        // reuse a dead slot or append
        slot = ctx->batches.size();
        for (size_t k = 0; k < ctx->batches.size(); ++k) if (!ctx->batches[k].alive) { slot = k; break; }
        if (slot == ctx->batches.size()) {
            if (slot + 1 >= kStaticSlot) return TENT_ERR_RANGE;
            try { ctx->batches.emplace_back(); } catch (const std::bad_alloc&) { return TENT_ERR_NOMEM; }
            if (!init_slot(ctx->batches[slot])) {
                destroy_slot(ctx->batches[slot]);
                ctx->batches.pop_back();
                return TENT_ERR_NOMEM;
            }
        }
        slot_b = &ctx->batches[slot];
    }
    Batch& b = *slot_b;
    renew_slot(b);
    b.payload = payload;
    b.max_req_slices = max_req_slices;
    BatchDev& d = b.dev;
    d.n_desc = n_desc;
    d.n_src_ext = ns;
    d.n_dst_ext = nd;
    d.n_slices = n_slices;
    d.slice_bytes = ctx->cfg.slice_bytes;
    d.seg_base = ctx->seg_base_dev;
    // Tile size: the largest power of two in [1 KiB, 4 KiB] that divides the slice size and every
    // extent length, so that no tile crosses an extent boundary; geometry that allows no such size
    // gets 1 KiB tiles, and the tiles that do cross a boundary take the generic copy path.
    {
        const uint64_t bits = len_bits | d.slice_bytes | kCopyBlockBytes;
        uint32_t tile = (uint32_t)(bits & (~bits + 1));
        d.tile_bytes = tile < 1024 ? 1024 : tile;
        d.tiles_per_slice = (uint32_t)((d.slice_bytes + d.tile_bytes - 1) / d.tile_bytes);
    }
    const uint64_t n_tiles = n_slices * d.tiles_per_slice;
    // Destination-ordered scatter needs every boundary on a tile boundary (addresses may have any
    // alignment); other geometry keeps the slice-ordered scatter.
    {
        const uint64_t bits = len_bits | d.slice_bytes;
        d.n_sc_tiles = (bits & (d.tile_bytes - 1)) == 0 ? payload / d.tile_bytes : 0;
    }

    uint32_t *sp = nullptr, *dp = nullptr;
    tent_extent *se = nullptr, *de = nullptr;
    const uint64_t scan_n = std::max<uint64_t>(std::max(ns, nd), std::max<uint64_t>(n_slices, n_desc));
    BatchDev* self_dev = nullptr;
    uint32_t* order_dev = nullptr;
    uint32_t* rank_dev = nullptr;
    Carver cv;
    cv.want(&sp, (uint64_t)n_desc + 1);
    cv.want(&dp, (uint64_t)n_desc + 1);
    cv.want(&se, ns);
    cv.want(&de, nd);
    cv.want(&d.src_pre, ns + 1);
    cv.want(&d.dst_pre, nd + 1);
    cv.want(&d.first, (uint64_t)n_desc + 1);
    cv.want(&d.s_desc, n_slices);
    cv.want(&d.s_off, n_slices);
    cv.want(&d.s_len, n_slices);
    cv.want(&d.s_src_e0, n_slices);
    cv.want(&d.s_dst_e0, n_slices);
    cv.want(&d.s_rail, n_slices);
    cv.want(&d.s_stage_off, n_slices);
    cv.want(&d.s_state, n_slices);
    cv.want(&d.s_tau, n_slices);
    cv.want(&d.s_rec, n_slices);
    cv.want(&d.s_retry, n_slices);
    cv.want(&d.priority, (uint64_t)n_desc);
    cv.want(&d.req_mode, (uint64_t)n_desc);
    cv.want(&self_dev, 1);
    cv.want(&b.overlap_dev, 1);
    if (d.n_sc_tiles == 0) {                              // per-slice tile tables only for untiled geometry
        cv.want(&d.src_tile, n_tiles);
        cv.want(&d.dst_tile, n_tiles);
    }
    d.run_capacity = 2u * n_desc;
    d.run_stride = ctx->max_rails <= 16 ? 16u : ctx->max_rails <= 32 ? 32u : 64u;   // a row per run, one entry per lane of the chain
    cv.want(&d.run_start, (uint64_t)d.run_capacity + 1);
    cv.want(&d.run_T, (uint64_t)d.run_capacity * d.run_stride);
    cv.want(&d.run_K, (uint64_t)d.run_capacity * d.run_stride);
    cv.want(&d.run_rec, (uint64_t)d.run_capacity + 1);
    cv.want(&d.len_pre, n_slices + 1);
    cv.want(&order_dev, nd);
    cv.want(&rank_dev, nd);
    if (d.n_sc_tiles) {
        cv.want(&d.ord_pre, nd + 1);
        cv.want(&d.ga_src, d.n_sc_tiles);
        cv.want(&d.ga_lin, d.n_sc_tiles);
        cv.want(&d.ga_slice, d.n_sc_tiles);
        cv.want(&d.ga_x, d.n_sc_tiles);
        if (ctx->cfg.flags & TENT_FLAG_BOUNDED_STAGING) cv.want(&d.ga_dst, d.n_sc_tiles);
        // an execute goes over a list of tiles only when at most half of the batch's tiles can move
        d.act_capacity = d.n_sc_tiles / 2 + 1;
        cv.want(&d.tile_scan, n_slices + 1);
        cv.want(&d.tile_partials, scan_partials_capacity(n_slices));
        cv.want(&d.act_src, d.act_capacity);
        cv.want(&d.act_lin, d.act_capacity);
        cv.want(&d.act_dst, d.act_capacity);
        cv.want(&d.sc_dst, d.n_sc_tiles);
        cv.want(&d.sc_lin, d.n_sc_tiles);
        cv.want(&d.sc_slice, d.n_sc_tiles);
        cv.want(&d.sc_x, d.n_sc_tiles);
    }
    if (ctx->cfg.flags & TENT_FLAG_BOUNDED_STAGING) {
        cv.want(&d.ch_lo, (uint64_t)kMaxChunks * TENT_MAX_RAILS);
        cv.want(&d.ch_hi, (uint64_t)kMaxChunks * TENT_MAX_RAILS);
        cv.want(&d.ch_base, (uint64_t)kMaxChunks * TENT_MAX_RAILS);
    }
    cv.want(&d.pending, n_slices);
    cv.want(&d.retry_ids, n_slices);
    const uint64_t rot_chunks = (n_slices + kRotChunk - 1) / kRotChunk;
    cv.want(&d.rot_bytes, rot_chunks * TENT_MAX_RAILS);
    cv.want(&d.rot_cnt, rot_chunks * TENT_MAX_RAILS);
    cv.want(&d.scan_tmp, scan_n + 1);
    cv.want(&d.scan_partials, scan_partials_capacity(scan_n));
    cv.want(&d.scan_partials2, scan_partials_capacity(scan_n));
    cv.want(&d.plan, 1);
    if (cv.overflow) return TENT_ERR_NOMEM;

    // destination extents in address order (for the scatter) and the overlap check run on the device
    const bool check = !(ctx->cfg.flags & TENT_FLAG_SKIP_OVERLAP_CHECK);
    const bool order = check || d.n_sc_tiles != 0;
    uint64_t ws_need = 0;
    if (order && order_workspace_bytes(nd, ns, check, &ws_need) != hipSuccess) { (void)hipGetLastError(); return TENT_ERR_HIP; }
    const uint64_t table_bytes = cv.total();
    void* workspace = nullptr;
    if (use_static) {
        // both the tables and the sort's workspace must fit the static workspace
        if (table_bytes + ws_need > kStaticBytes) return TENT_ERR_RANGE;
        uint8_t* area = nullptr;
        {
            std::lock_guard<std::mutex> lk(g_static_mutex);
            if (ctx->device >= kMaxDevices || !g_static[ctx->device].ptr) return TENT_ERR_STATE;
            area = static_cast<uint8_t*>(g_static[ctx->device].ptr);
            b.static_generation = ++g_static[ctx->device].generation;
        }
        b.block = area;
        b.block_bytes = table_bytes;
        b.in_static = true;
        workspace = area + table_bytes;
    } else {
        rc = acquire_block(ctx, table_bytes, &b.block, &b.block_bytes);
        if (rc != TENT_OK) return rc;
        if (ws_need > ctx->order_ws_bytes) {
            // the stream that used the old workspace is the context's own: wait for it, then replace
            (void)hipStreamSynchronize(ctx->decl_stream);
            if (ctx->order_ws) (void)hipFree(ctx->order_ws);
            ctx->order_ws = nullptr;
            ctx->order_ws_bytes = 0;
            const uint64_t want = ws_need + ws_need / 4;
            if (hipMalloc(&ctx->order_ws, want) != hipSuccess) {
                (void)hipGetLastError();
                ctx->order_ws = nullptr;
                free_batch(ctx, b);
                return TENT_ERR_NOMEM;
            }
            ctx->order_ws_bytes = want;
        }
        workspace = ctx->order_ws;
    }
    cv.place(b.block);
    d.src_ptr = sp; d.dst_ptr = dp; d.src_ext = se; d.dst_ext = de;
    d.dst_order = order_dev;
    d.dst_rank = rank_dev;
    d.self = self_dev;

    // Everything from here on is enqueued on the context's own stream; nothing waits for the device
    // unless the host arrays could not go through the pinned buffer.
    hipStream_t ds = ctx->decl_stream;
    bool ok = true;
    if (st) {
        std::memcpy(st + o_sp, src_ptr, ptr_bytes);
        std::memcpy(st + o_dp, dst_ptr, ptr_bytes);
        std::memcpy(st + o_self, &d, sizeof(BatchDev));
        ok = hipMemcpyAsync(sp, st + o_sp, ptr_bytes, hipMemcpyHostToDevice, ds) == hipSuccess &&
             hipMemcpyAsync(dp, st + o_dp, ptr_bytes, hipMemcpyHostToDevice, ds) == hipSuccess &&
             hipMemcpyAsync(se, st + o_se, ns * sizeof(tent_extent), hipMemcpyHostToDevice, ds) == hipSuccess &&
             hipMemcpyAsync(de, st + o_de, nd * sizeof(tent_extent), hipMemcpyHostToDevice, ds) == hipSuccess &&
             hipMemcpyAsync(self_dev, st + o_self, sizeof(BatchDev), hipMemcpyHostToDevice, ds) == hipSuccess &&
             hipEventRecord(ctx->stage_event[which], ds) == hipSuccess;
        if (ok) ctx->stage_busy[which] = true;
    } else {
        // the pinned buffer is too small and may not grow: the arrays go through it piece by piece
        ok = upload_in_pieces(ctx, sp, src_ptr, ptr_bytes) && upload_in_pieces(ctx, dp, dst_ptr, ptr_bytes) &&
             upload_in_pieces(ctx, se, src_ext, ns * sizeof(tent_extent)) &&
             upload_in_pieces(ctx, de, dst_ext, nd * sizeof(tent_extent)) &&
             upload_in_pieces(ctx, self_dev, &d, sizeof(BatchDev));
    }
    ok = ok && hipMemsetAsync(d.s_retry, 0, std::max<uint64_t>(n_slices, 1), ds) == hipSuccess &&
         hipMemsetAsync(d.req_mode, 0, n_desc, ds) == hipSuccess &&
         hipMemsetAsync(d.plan, 0, sizeof(PlanState), ds) == hipSuccess &&
         hipMemsetAsync(b.overlap_dev, 0, sizeof(uint32_t), ds) == hipSuccess;
    if (ok && order)
        ok = device_order_destinations(de, nd, se, ns, ctx->seg_base_dev, check, order_dev, rank_dev, b.overlap_dev,
                                       workspace, ds) == hipSuccess;
    *b.verdict = 0;
    ok = ok && hipMemcpyAsync(b.verdict, b.overlap_dev, sizeof(uint32_t), hipMemcpyDeviceToHost, ds) == hipSuccess &&
         hipEventRecord(b.decl_event, ds) == hipSuccess;
    if (!ok) {
        (void)hipGetLastError();
        (void)hipStreamSynchronize(ds);
        free_batch(ctx, b);
        return TENT_ERR_HIP;
    }
    b.decl_pending = true;
    b.alive = true;
    *out = ((uint64_t)b.generation << 32) | (use_static ? (uint64_t)kStaticSlot : (uint64_t)(slot + 1));
    return TENT_OK;
}

}  // namespace

extern "C" {

const char* tent_strerror(int status)
{
    switch (status) {
        case TENT_OK:          return "ok";
        case TENT_DEFER:       return "deferred: no admitted rail";
        case TENT_ERR_INVALID: return "invalid argument";
        case TENT_ERR_RANGE:   return "value out of range";
        case TENT_ERR_STATE:   return "call out of order";
        case TENT_ERR_NOMEM:   return "out of memory";
        case TENT_ERR_HIP:     return "HIP runtime error";
        default:               return "unknown status";
    }
}

int tent_create(tent_ctx** out, const tent_config* cfg)
{
    if (!out || !cfg) return TENT_ERR_INVALID;
    *out = nullptr;
    if (cfg->slice_bytes == 0 || cfg->slice_bytes > 0x80000000ull) return TENT_ERR_INVALID;
    if (!cfg->staging_arena || cfg->staging_bytes == 0) return TENT_ERR_INVALID;
    if (cfg->max_rails > TENT_MAX_RAILS) return TENT_ERR_RANGE;
    tent_ctx* ctx = new (std::nothrow) tent_ctx;
    if (!ctx) return TENT_ERR_NOMEM;
    ctx->cfg = *cfg;
    ctx->max_rails = cfg->max_rails ? cfg->max_rails : TENT_MAX_RAILS;
    if (hipGetDevice(&ctx->device) != hipSuccess) { delete ctx; return TENT_ERR_HIP; }
    ctx->seg_capacity = kMaxSegments;
    bool ok = true;
    try { ctx->spare.reserve(kSpareBlocks); ctx->batches.reserve(16); } catch (const std::bad_alloc&) { ok = false; }
    ok = ok && hipMalloc((void**)&ctx->seg_base_dev, sizeof(uint64_t) * ctx->seg_capacity) == hipSuccess &&
         hipHostMalloc((void**)&ctx->host_plan, sizeof(PlanState), hipHostMallocDefault) == hipSuccess &&
         hipStreamCreateWithFlags(&ctx->decl_stream, hipStreamNonBlocking) == hipSuccess &&
         init_slot(ctx->static_batch);
    for (int k = 0; k < 2 && ok; ++k) {
        ok = hipHostMalloc((void**)&ctx->stage[k], kStageInitial, hipHostMallocDefault) == hipSuccess &&
             hipEventCreateWithFlags(&ctx->stage_event[k], hipEventDisableTiming) == hipSuccess;
        if (ok) ctx->stage_bytes[k] = kStageInitial;
    }
    // the static workspace's address on this GPU, looked up once per device with the device current
    int rc = ok ? TENT_OK : TENT_ERR_NOMEM;
    if (ok && ctx->device < kMaxDevices) {
        std::lock_guard<std::mutex> lk(g_static_mutex);
        if (!g_static[ctx->device].ptr) {
            void* p = nullptr;
            if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) rc = TENT_ERR_HIP;
            else g_static[ctx->device].ptr = p;
        }
    }
    if (rc != TENT_OK) {
        (void)hipGetLastError();
        (void)tent_destroy(ctx);
        return rc;
    }
    *out = ctx;
    return TENT_OK;
}

int tent_destroy(tent_ctx* ctx)
{
    if (!ctx) return TENT_ERR_INVALID;
    DeviceGuard g(ctx->device);
    (void)hipDeviceSynchronize();
    for (Batch& b : ctx->batches) {
        if (b.alive) free_batch(ctx, b);
        destroy_slot(b);
    }
    if (ctx->static_batch.alive) free_batch(ctx, ctx->static_batch);
    destroy_slot(ctx->static_batch);
    for (Block& blk : ctx->spare) (void)hipFree(blk.ptr);
    for (Timing& t : ctx->timing)
        for (auto& pr : t.pool) { (void)hipEventDestroy(pr.first); (void)hipEventDestroy(pr.second); }
    for (hipEvent_t e : ctx->sync_events) (void)hipEventDestroy(e);
    for (int k = 0; k < 2; ++k) {
        if (ctx->stage[k]) (void)hipHostFree(ctx->stage[k]);
        if (ctx->stage_event[k]) (void)hipEventDestroy(ctx->stage_event[k]);
    }
    if (ctx->order_ws) (void)hipFree(ctx->order_ws);
    if (ctx->decl_stream) (void)hipStreamDestroy(ctx->decl_stream);
    if (ctx->aux_stream) (void)hipStreamDestroy(ctx->aux_stream);
    if (ctx->seg_base_dev) (void)hipFree(ctx->seg_base_dev);
    if (ctx->host_plan) (void)hipHostFree(ctx->host_plan);
    delete ctx;
    return TENT_OK;
}

int tent_register_segment(tent_ctx* ctx, void* dev_base, uint64_t len, uint32_t* seg_out)
{
    if (!ctx || !dev_base || len == 0 || !seg_out) return TENT_ERR_INVALID;
    if (ctx->segments.size() >= ctx->seg_capacity) return TENT_ERR_RANGE;
    DeviceGuard g(ctx->device);
    if (!g.ok) return TENT_ERR_HIP;
    const uint32_t id = (uint32_t)ctx->segments.size();
    const uint64_t addr = (uint64_t)dev_base;
    try { ctx->segments.reserve(ctx->segments.size() + 1); } catch (const std::bad_alloc&) { return TENT_ERR_NOMEM; }
    HIP_TRY(hipMemcpy(ctx->seg_base_dev + id, &addr, sizeof(addr), hipMemcpyHostToDevice));
    ctx->segments.push_back({static_cast<uint8_t*>(dev_base), len});
    *seg_out = id;
    return TENT_OK;
}

int tent_declare(tent_ctx* ctx, uint32_t n_desc, const uint32_t* src_ptr, const tent_extent* src_ext,
                 const uint32_t* dst_ptr, const tent_extent* dst_ext, tent_batch_t* out)
{
    return declare_impl(ctx, n_desc, src_ptr, src_ext, dst_ptr, dst_ext, out, false);
}

int tent_declare_static(tent_ctx* ctx, uint32_t n_desc, const uint32_t* src_ptr, const tent_extent* src_ext,
                        const uint32_t* dst_ptr, const tent_extent* dst_ext, tent_batch_t* out)
{
    return declare_impl(ctx, n_desc, src_ptr, src_ext, dst_ptr, dst_ext, out, true);
}

int tent_plan(tent_ctx* ctx, tent_batch_t batch, const tent_rail_state* rails, uint32_t n_rails,
              tent_plan_info* info, void* stream)
{
    if (!ctx || !rails) return TENT_ERR_INVALID;
    Batch* b = find_batch(ctx, batch);
    if (!b) return TENT_ERR_INVALID;
    if (b->broken) return TENT_ERR_STATE;
    if (n_rails == 0 || n_rails > ctx->max_rails) return TENT_ERR_RANGE;
    RailParams rp;
    int rc = convert_rails(rails, n_rails, b->payload, &rp);
    if (rc != TENT_OK) return rc;
    DeviceGuard g(ctx->device);
    if (!g.ok) return TENT_ERR_HIP;
    rc = finish_declare(ctx, *b);
    if (rc != TENT_OK) return rc;
    if (rp.admitted == 0) return TENT_DEFER;
    if (!(ctx->cfg.flags & TENT_FLAG_BOUNDED_STAGING) && b->payload + 256ull * n_rails > ctx->cfg.staging_bytes)
        return TENT_ERR_RANGE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const BatchDev& d = b->dev;
    StreamNote note(*b, s);
    HIP_TRY(order_after_execute_bookkeeping(*b, s));

    // Retry rotation (Section 4.3, "Link-Level Resilience"): candidates are the HEALTHY rails, else the
    // DEGRADED rails without topology penalty, else every DEGRADED rail, in ascending index.
    RotateParams rot;
    std::memset(&rot, 0, sizeof(rot));
    if (b->has_retry) {
        for (int pass = 0; pass < 3 && rot.n_cand == 0; ++pass)
            for (uint32_t r = 0; r < n_rails; ++r) {
                const bool take = pass == 0 ? rails[r].health == 0
                                : pass == 1 ? rails[r].health == 1 && rails[r].penalty_q8 <= 256
                                            : rails[r].health == 1;
                if (take) rot.cand[rot.n_cand++] = (uint8_t)r;
            }
    }

    const bool replan = b->has_done || b->has_retry;
    // the run-parallel chain divides by c1, so a rail whose cost does not grow with bytes
    // (c1 = 0) sends the plan down the slice-by-slice kernel
    bool serial = (ctx->cfg.flags & TENT_FLAG_SERIAL_BINDING) != 0;
    for (uint32_t r = 0; r < n_rails; ++r)
        if (((rp.admitted >> r) & 1) && rp.c1[r] == 0) serial = true;
    if (!replan) {
        {
            StageTimer t(ctx, TENT_T_EXTENT_SCAN, s);
            HIP_TRY(launch_extent_scans(d, s));
        }
        {
            StageTimer t(ctx, TENT_T_SLICE_SCAN, s);
            HIP_TRY(launch_slice_scan(d, s));
        }
        {
            // the tile tables of the copy kernels are built beside the binding chain, in its launch
            // (the slice-by-slice binder has no such launch: there they are built here)
            StageTimer t(ctx, TENT_T_EXPAND, s);
            HIP_TRY(launch_expand(d, s));
            if (serial) HIP_TRY(launch_tile_tables(d, s));
            else        HIP_TRY(launch_tile_tables_prepare(d, s));
        }
    } else {
        StageTimer t(ctx, TENT_T_COMPACT, s);
        HIP_TRY(launch_compact(d, s));
    }
    int mode = replan ? kBindUsePending : 0;
    if (b->has_retry) {
        StageTimer t(ctx, TENT_T_BIND, s);
        HIP_TRY(launch_rotate(d, rot, s));
        mode |= kBindAfterRotation;
    }
    {
        StageTimer t(ctx, TENT_T_BIND, s);
        if (serial) HIP_TRY(launch_bind_serial(d, rp, mode, s));
        else        HIP_TRY(launch_bind_runs(d, rp, mode | (replan ? 0 : kBindBuildTables), s));
    }
    b->planned = true;
    b->bound_hint = b->dev.n_slices;
    b->tile_hint = ~0ull;
    b->last_rails = rp;
    for (uint32_t r = 0; r < n_rails; ++r) b->last_lat_ns[r] = rails[r].lat_ns;

    if (info) {
        HIP_TRY(hipMemcpyAsync(ctx->host_plan, d.plan, sizeof(PlanState), hipMemcpyDeviceToHost, s));
        HIP_TRY(hipStreamSynchronize(s));
        const PlanState& ps = *ctx->host_plan;
        std::memset(info, 0, sizeof(*info));
        b->bound_hint = ps.n_bound;
        info->n_slices = ps.n_bound;
        info->n_pending_before = ps.n_pending;
        for (uint32_t r = 0; r < TENT_MAX_RAILS; ++r) {
            info->rail_bytes[r] = ps.T[r];
            info->rail_slices[r] = ps.cnt[r];
            info->queued_after[r] = r < n_rails ? ps.A_after[r] : 0;
            info->stage_base[r] = r < n_rails ? ps.base[r] : 0;
        }
    }
    return TENT_OK;
}

int tent_plan_dispatch(tent_ctx* ctx, tent_batch_t batch, const tent_rail_state* rails, uint32_t n_rails,
                       const tent_dispatch_params* params, const uint8_t* priority, tent_dispatch_info* info,
                       void* stream)
{
    if (!ctx || !rails || !params) return TENT_ERR_INVALID;
    Batch* b = find_batch(ctx, batch);
    if (!b) return TENT_ERR_INVALID;
    if (b->broken) return TENT_ERR_STATE;
    if (n_rails == 0 || n_rails > ctx->max_rails) return TENT_ERR_RANGE;
    if (params->gamma_q8 > 65535u) return TENT_ERR_RANGE;
    RailParams rp;
    int rc = convert_rails(rails, n_rails, b->payload, &rp);
    if (rc != TENT_OK) return rc;
    {
        DeviceGuard g0(ctx->device);
        if (!g0.ok) return TENT_ERR_HIP;
        rc = finish_declare(ctx, *b);
        if (rc != TENT_OK) return rc;
    }
    if (rp.admitted == 0) return TENT_DEFER;
    if (!(ctx->cfg.flags & TENT_FLAG_BOUNDED_STAGING) && b->payload + 256ull * n_rails > ctx->cfg.staging_bytes)
        return TENT_ERR_RANGE;
    if (priority)
        for (uint32_t j = 0; j < b->dev.n_desc; ++j)
            if (priority[j] > 2) return TENT_ERR_INVALID;
    // The slot keys (m + 1) * s_d are packed with a 6-bit rail index and the tolerance multiplies a
    // cost by gamma: bound the largest cost any rail can show during this plan.
    {
        unsigned __int128 worst = 0;
        for (uint32_t d = 0; d < n_rails; ++d) {
            if (!((rp.admitted >> d) & 1)) continue;
            const unsigned __int128 c = (unsigned __int128)rp.c0[d] +
                                        ((((unsigned __int128)rp.A[d] + b->payload) * rp.c1[d]) >> 16);
            worst = std::max(worst, c);
        }
        if (worst * (b->max_req_slices + 1) >= ((unsigned __int128)1 << 57)) return TENT_ERR_RANGE;
        if (worst * (params->gamma_q8 + 1u) >= ((unsigned __int128)1 << 63)) return TENT_ERR_RANGE;
    }
    DispatchParams dp;
    std::memset(&dp, 0, sizeof(dp));
    dp.theta = params->theta_bytes;
    dp.rr_start = params->rr_start;
    dp.gamma_q8 = params->gamma_q8;
    // Priority slots (Section 4.2, "Quality of Service"): in window w rail d sits in slot (w + d) mod 3;
    // slot 0 takes HIGH only, slot 1 HIGH and MID, slot 2 everything.
    for (uint32_t d = 0; d < n_rails; ++d) {
        if (!((rp.admitted >> d) & 1)) continue;
        const uint32_t slot = (uint32_t)(((uint64_t)params->window + d) % 3);
        const uint32_t lowest = slot == 0 ? 2 : slot == 1 ? 1 : 0;
        for (uint32_t p = lowest; p <= 2; ++p) dp.adm[p] |= 1ull << d;
    }

    DeviceGuard g(ctx->device);
    if (!g.ok) return TENT_ERR_HIP;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const BatchDev& d = b->dev;
    StreamNote note(*b, s);
    HIP_TRY(order_after_execute_bookkeeping(*b, s));
    dp.all_high = priority ? 0u : 1u;
    if (priority) HIP_TRY(hipMemcpyAsync(d.priority, priority, d.n_desc, hipMemcpyHostToDevice, s));
    const bool first_plan = !b->planned;
    if (first_plan) {
        {
            StageTimer t(ctx, TENT_T_EXTENT_SCAN, s);
            HIP_TRY(launch_extent_scans(d, s));
        }
        {
            StageTimer t(ctx, TENT_T_SLICE_SCAN, s);
            HIP_TRY(launch_slice_scan(d, s));
        }
        {
            StageTimer t(ctx, TENT_T_EXPAND, s);
            HIP_TRY(launch_expand(d, s));
            HIP_TRY(launch_tile_tables_prepare(d, s));      // the tables themselves: beside the chain, in its launch
        }
    }
    {
        StageTimer t(ctx, TENT_T_BIND, s);
        HIP_TRY(launch_dispatch(d, rp, dp, first_plan, s));
    }
    b->planned = true;
    b->bound_hint = b->dev.n_slices;
    b->tile_hint = ~0ull;
    b->last_rails = rp;
    for (uint32_t r = 0; r < n_rails; ++r) b->last_lat_ns[r] = rails[r].lat_ns;

    if (info) {
        HIP_TRY(hipMemcpyAsync(ctx->host_plan, d.plan, sizeof(PlanState), hipMemcpyDeviceToHost, s));
        HIP_TRY(hipStreamSynchronize(s));
        const PlanState& ps = *ctx->host_plan;
        std::memset(info, 0, sizeof(*info));
        b->bound_hint = ps.n_bound;
        info->plan.n_slices = ps.n_bound;
        info->plan.n_pending_before = ps.n_pending;
        for (uint32_t r = 0; r < n_rails; ++r) {
            info->plan.rail_bytes[r] = ps.T[r];
            info->plan.rail_slices[r] = ps.cnt[r];
            info->plan.queued_after[r] = ps.A_after[r];
            info->plan.stage_base[r] = ps.base[r];
        }
        info->n_mice = ps.n_mice;
        info->n_elephant = ps.n_elephant;
        info->n_deferred = ps.n_deferred;
        info->rr_next = ps.rr_next;
    }
    return TENT_OK;
}

int tent_get_modes(tent_ctx* ctx, tent_batch_t batch, uint8_t* host_out, uint64_t cap)
{
    if (!ctx || !host_out) return TENT_ERR_INVALID;
    Batch* b = find_batch(ctx, batch);
    if (!b) return TENT_ERR_INVALID;
    if (cap < b->dev.n_desc) return TENT_ERR_RANGE;
    DeviceGuard g(ctx->device);
    if (!g.ok) return TENT_ERR_HIP;
    HIP_TRY(hipDeviceSynchronize());
    HIP_TRY(hipMemcpy(host_out, b->dev.req_mode, b->dev.n_desc, hipMemcpyDeviceToHost));
    return TENT_OK;
}

int tent_sim_advance(tent_ctx* ctx, tent_batch_t batch, const uint64_t* budget_bytes, uint64_t* n_done,
                     void* stream)
{
    if (!ctx || !budget_bytes) return TENT_ERR_INVALID;
    Batch* b = find_batch(ctx, batch);
    if (!b) return TENT_ERR_INVALID;
    if (!b->planned) return TENT_ERR_STATE;
    DeviceGuard g(ctx->device);
    if (!g.ok) return TENT_ERR_HIP;
    hipStream_t s = static_cast<hipStream_t>(stream);
    BudgetParams bp;
    std::memset(&bp, 0, sizeof(bp));
    for (uint32_t d = 0; d < b->last_rails.n_rails; ++d) {
        bp.queued[d] = b->last_rails.A[d];
        bp.budget[d] = budget_bytes[d];
    }
    StreamNote note(*b, s);
    HIP_TRY(launch_retire(b->dev, bp, s));
    // What stays BOUND on rail d fits in budget_d - queued_d bytes, which bounds the tiles the next execute
    // copies without asking the device (slices of a tiled batch are whole tiles).
    uint64_t tiles = 0;
    for (uint32_t d = 0; d < b->last_rails.n_rails; ++d)
        if (bp.budget[d] > bp.queued[d]) tiles += (bp.budget[d] - bp.queued[d]) / (b->dev.tile_bytes ? b->dev.tile_bytes : 1u);
    b->tile_hint = tiles;
    if (!n_done) return TENT_OK;
    HIP_TRY(hipMemcpyAsync(ctx->host_plan, b->dev.plan, sizeof(PlanState), hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    b->bound_hint = ctx->host_plan->n_done;
    *n_done = ctx->host_plan->n_done;
    return TENT_OK;
}

int tent_sim_fail(tent_ctx* ctx, tent_batch_t batch, const uint8_t* rail_failed, uint64_t* failed_per_rail,
                  void* stream)
{
    if (!ctx || !rail_failed) return TENT_ERR_INVALID;
    Batch* b = find_batch(ctx, batch);
    if (!b) return TENT_ERR_INVALID;
    if (!b->planned) return TENT_ERR_STATE;
    const uint32_t n_rails = b->last_rails.n_rails;
    FailParams fp;
    std::memset(&fp, 0, sizeof(fp));
    bool any = false;
    for (uint32_t d = 0; d < n_rails; ++d) {
        fp.failed[d] = rail_failed[d] ? 1 : 0;
        any = any || rail_failed[d];
    }
    DeviceGuard g(ctx->device);
    if (!g.ok) return TENT_ERR_HIP;
    hipStream_t s = static_cast<hipStream_t>(stream);
    StreamNote note(*b, s);
    if (any) {
        HIP_TRY(launch_fail(b->dev, fp, s));
        b->has_retry = true;
    }
    if (failed_per_rail) {
        for (uint32_t d = 0; d < n_rails; ++d) failed_per_rail[d] = 0;
        if (any) {
            HIP_TRY(hipMemcpyAsync(ctx->host_plan, b->dev.plan, sizeof(PlanState), hipMemcpyDeviceToHost, s));
            HIP_TRY(hipStreamSynchronize(s));
            for (uint32_t d = 0; d < n_rails; ++d) failed_per_rail[d] = ctx->host_plan->fail_cnt[d];
        }
    }
    return TENT_OK;
}

int tent_get_retries(tent_ctx* ctx, tent_batch_t batch, uint8_t* host_out, uint64_t cap)
{
    if (!ctx || !host_out) return TENT_ERR_INVALID;
    Batch* b = find_batch(ctx, batch);
    if (!b) return TENT_ERR_INVALID;
    if (cap < b->dev.n_slices) return TENT_ERR_RANGE;
    DeviceGuard g(ctx->device);
    if (!g.ok) return TENT_ERR_HIP;
    HIP_TRY(hipDeviceSynchronize());
    HIP_TRY(hipMemcpy(host_out, b->dev.s_retry, b->dev.n_slices, hipMemcpyDeviceToHost));
    return TENT_OK;
}

int tent_sim_latency(tent_ctx* ctx, tent_batch_t batch, const uint32_t* true_bw_MBps, void* stream)
{
    if (!ctx || !true_bw_MBps) return TENT_ERR_INVALID;
    Batch* b = find_batch(ctx, batch);
    if (!b) return TENT_ERR_INVALID;
    if (!b->planned) return TENT_ERR_STATE;
    LatencyParams lp;
    std::memset(&lp, 0, sizeof(lp));
    uint64_t max_q = 0;
    for (uint32_t d = 0; d < TENT_MAX_RAILS; ++d) lp.bw_MBps[d] = 1;
    for (uint32_t d = 0; d < b->last_rails.n_rails; ++d) {
        if (true_bw_MBps[d] == 0) return TENT_ERR_RANGE;
        lp.queued[d] = b->last_rails.A[d];
        lp.lat_ns[d] = b->last_lat_ns[d];
        lp.bw_MBps[d] = true_bw_MBps[d];
        max_q = std::max(max_q, lp.queued[d]);
    }
    if (max_q >= (1ull << 53) || b->payload >= (1ull << 53) || max_q + b->payload >= (1ull << 53)) return TENT_ERR_RANGE;
    DeviceGuard g(ctx->device);
    if (!g.ok) return TENT_ERR_HIP;
    StreamNote note(*b, static_cast<hipStream_t>(stream));
    HIP_TRY(launch_sim_latency(b->dev, lp, static_cast<hipStream_t>(stream)));
    return TENT_OK;
}

int tent_update_bandwidth(tent_ctx* ctx, tent_batch_t batch, const tent_probe_params* params, tent_rail_state* rails,
                          uint32_t n_rails, uint32_t* probe_MBps_out, void* stream)
{
    if (!ctx || !params || !rails) return TENT_ERR_INVALID;
    Batch* b = find_batch(ctx, batch);
    if (!b) return TENT_ERR_INVALID;
    if (!b->planned) return TENT_ERR_STATE;
    if (n_rails != b->last_rails.n_rails) return TENT_ERR_RANGE;
    ProbeParams pp;
    std::memset(&pp, 0, sizeof(pp));
    pp.n_rails = n_rails;
    for (uint32_t d = 0; d < n_rails; ++d) {
        if (params[d].alpha_q8 > 65535u || params[d].ewma_q8 > 256u) return TENT_ERR_RANGE;
        pp.cal[d] = params[d];
        pp.bw_MBps[d] = rails[d].bw_MBps;
    }
    DeviceGuard g(ctx->device);
    if (!g.ok) return TENT_ERR_HIP;
    hipStream_t s = static_cast<hipStream_t>(stream);
    {
        StageTimer t(ctx, TENT_T_FEEDBACK, s);
        HIP_TRY(launch_probe(b->dev, pp, s));
    }
    HIP_TRY(hipMemcpyAsync(ctx->host_plan, b->dev.plan, sizeof(PlanState), hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    for (uint32_t d = 0; d < n_rails; ++d) {
        rails[d].bw_MBps = ctx->host_plan->bw_next[d];
        if (probe_MBps_out) probe_MBps_out[d] = ctx->host_plan->probe[d];
    }
    return TENT_OK;
}

int tent_get_latencies(tent_ctx* ctx, tent_batch_t batch, uint64_t* host_out, uint64_t cap)
{
    if (!ctx || !host_out) return TENT_ERR_INVALID;
    Batch* b = find_batch(ctx, batch);
    if (!b) return TENT_ERR_INVALID;
    if (!b->planned) return TENT_ERR_STATE;
    if (cap < b->dev.n_slices) return TENT_ERR_RANGE;
    DeviceGuard g(ctx->device);
    if (!g.ok) return TENT_ERR_HIP;
    HIP_TRY(hipDeviceSynchronize());
    HIP_TRY(hipMemcpy(host_out, b->dev.s_tau, b->dev.n_slices * sizeof(uint64_t), hipMemcpyDeviceToHost));
    return TENT_OK;
}

int tent_execute(tent_ctx* ctx, tent_batch_t batch, void* stream)
{
    if (!ctx) return TENT_ERR_INVALID;
    Batch* b = find_batch(ctx, batch);
    if (!b) return TENT_ERR_INVALID;
    if (!b->planned || b->broken) return TENT_ERR_STATE;
    if (b->payload + 256ull * b->last_rails.n_rails > ctx->cfg.staging_bytes) return TENT_ERR_RANGE;
    DeviceGuard g(ctx->device);
    if (!g.ok) return TENT_ERR_HIP;
    hipStream_t s = static_cast<hipStream_t>(stream);
    StreamNote note(*b, s);
    // When the host knows that only a small part of the batch is BOUND (after the rail simulator), the
    // copies run over a list of the tiles of the BOUND slices and their launches are sized by that part.
    uint64_t max_tiles = b->bound_hint * b->dev.tiles_per_slice;
    if (b->tile_hint < max_tiles) max_tiles = b->tile_hint;
    const bool compact = b->dev.n_sc_tiles != 0 && max_tiles * 2 <= b->dev.n_sc_tiles;
    HIP_TRY(launch_finalize(b->dev, static_cast<uint8_t*>(ctx->cfg.staging_arena), compact, max_tiles, s));
    // The copies below are driven by the tables just written and read no slice state, so the slices
    // are marked DONE ahead of them: in stream order nothing changes, and the next re-plan, if it
    // is enqueued on another stream, can run beside the copies.  tent_poll, on whatever stream, waits
    // for the end of the copies (done_event), so a slice is never reported complete while its bytes move.
    HIP_TRY(launch_mark_done(b->dev, compact, s));
    // From here on a failure would leave slices marked DONE whose bytes were never moved: the batch
    // is then flagged, and every call but tent_reset and tent_release refuses it.
    auto copies = [&]() -> hipError_t {
        hipError_t e = record_execute_bookkeeping(*b, s);
        if (e != hipSuccess) return e;
        {
            StageTimer t(ctx, TENT_T_GATHER, s);
            e = compact ? launch_copy_compact(b->dev, true, max_tiles, s)
                : b->dev.n_sc_tiles ? launch_copy_ordered(b->dev, true, s) : launch_copy(b->dev, true, s);
        }
        if (e != hipSuccess) return e;
        {
            StageTimer t(ctx, TENT_T_SCATTER, s);
            e = compact ? launch_copy_compact(b->dev, false, max_tiles, s)
                : b->dev.n_sc_tiles ? launch_copy_ordered(b->dev, false, s) : launch_copy(b->dev, false, s);
        }
        if (e != hipSuccess) return e;
        return record_execute_done(*b, s);
    };
    b->has_done = true;
    b->bound_hint = 0;
    if (copies() != hipSuccess) {
        (void)hipGetLastError();
        b->broken = true;
        return TENT_ERR_HIP;
    }
    return TENT_OK;
}

int tent_execute_bounded(tent_ctx* ctx, tent_batch_t batch, uint64_t chunk_bytes, uint32_t slots, void* stream)
{
    if (!ctx) return TENT_ERR_INVALID;
    Batch* b = find_batch(ctx, batch);
    if (!b) return TENT_ERR_INVALID;
    if (!b->planned || b->broken || !(ctx->cfg.flags & TENT_FLAG_BOUNDED_STAGING)) return TENT_ERR_STATE;
    const BatchDev& d = b->dev;
    // chunks are cut on 1 MiB boundaries so that the 256 consecutive tiles (or four consecutive 1 KiB
    // ranges) of one workgroup never straddle two chunks
    if (chunk_bytes == 0 || (chunk_bytes & ((1ull << 20) - 1)) != 0 || slots < 1 || slots > 2) return TENT_ERR_INVALID;
    const uint64_t slot_bytes = chunk_bytes + 256ull * b->last_rails.n_rails;
    if (slot_bytes > ctx->cfg.staging_bytes / slots) return TENT_ERR_RANGE;
    const uint64_t n_chunks = (b->payload + chunk_bytes - 1) / chunk_bytes;
    if (n_chunks > kMaxChunks) return TENT_ERR_RANGE;
    DeviceGuard g(ctx->device);
    if (!g.ok) return TENT_ERR_HIP;
    hipStream_t s = static_cast<hipStream_t>(stream);
    StreamNote note(*b, s);
    uint8_t* arena = static_cast<uint8_t*>(ctx->cfg.staging_arena);
    const uint64_t payload = b->payload;
    HIP_TRY(launch_bounded_prepare(d, payload, chunk_bytes, (uint32_t)n_chunks, slot_bytes, slots, arena, s));
    if (slots == 1) {
        for (uint32_t c = 0; c < n_chunks; ++c) {
            {
                StageTimer t(ctx, TENT_T_GATHER, s);
                HIP_TRY(launch_bounded_copy(d, true, c, payload, chunk_bytes, slot_bytes, slots, arena, s));
            }
            {
                StageTimer t(ctx, TENT_T_SCATTER, s);
                HIP_TRY(launch_bounded_copy(d, false, c, payload, chunk_bytes, slot_bytes, slots, arena, s));
            }
        }
    } else {
        // Two slots: gathers stay on the caller's stream, scatters go to a second stream.  Scatter c
        // waits for gather c; gather c + 2 waits for scatter c, which frees its slot; gather c + 1
        // overlaps scatter c (Section 4.1: consecutive stages of the staging pipeline overlap).
        if (!ctx->aux_stream && hipStreamCreateWithFlags(&ctx->aux_stream, hipStreamNonBlocking) != hipSuccess) {
            (void)hipGetLastError();
            ctx->aux_stream = nullptr;
            return TENT_ERR_HIP;
        }
        try {
            while (ctx->sync_events.size() < 2 * n_chunks + 1) {
                hipEvent_t e = nullptr;
                if (hipEventCreateWithFlags(&e, hipEventDisableTiming) != hipSuccess) {
                    (void)hipGetLastError();
                    return TENT_ERR_HIP;
                }
                ctx->sync_events.push_back(e);
            }
        } catch (const std::bad_alloc&) { return TENT_ERR_NOMEM; }
        hipStream_t x = ctx->aux_stream;
        hipEvent_t prepared = ctx->sync_events[2 * n_chunks];
        HIP_TRY(hipEventRecord(prepared, s));
        HIP_TRY(hipStreamWaitEvent(x, prepared, 0));
        for (uint32_t c = 0; c < n_chunks; ++c) {
            hipEvent_t gathered = ctx->sync_events[2 * c], scattered = ctx->sync_events[2 * c + 1];
            if (c >= 2) HIP_TRY(hipStreamWaitEvent(s, ctx->sync_events[2 * (c - 2) + 1], 0));
            {
                StageTimer t(ctx, TENT_T_GATHER, s);
                HIP_TRY(launch_bounded_copy(d, true, c, payload, chunk_bytes, slot_bytes, slots, arena, s));
            }
            HIP_TRY(hipEventRecord(gathered, s));
            HIP_TRY(hipStreamWaitEvent(x, gathered, 0));
            {
                StageTimer t(ctx, TENT_T_SCATTER, x);
                HIP_TRY(launch_bounded_copy(d, false, c, payload, chunk_bytes, slot_bytes, slots, arena, x));
            }
            HIP_TRY(hipEventRecord(scattered, x));
        }
        // the caller's stream continues once every scatter has finished
        HIP_TRY(hipStreamWaitEvent(s, ctx->sync_events[2 * (n_chunks - 1) + 1], 0));
        if (n_chunks >= 2) HIP_TRY(hipStreamWaitEvent(s, ctx->sync_events[2 * (n_chunks - 2) + 1], 0));
    }
    HIP_TRY(launch_mark_done_bounded(d, s));
    b->prep_recorded = false;                                 // the bounded execute offers no overlap with a re-plan
    b->has_done = true;
    b->bound_hint = 0;
    HIP_TRY(record_execute_done(*b, s));
    return TENT_OK;
}

int tent_poll(tent_ctx* ctx, tent_batch_t batch, uint64_t* remaining, void* stream)
{
    if (!ctx || !remaining) return TENT_ERR_INVALID;
    Batch* b = find_batch(ctx, batch);
    if (!b) return TENT_ERR_INVALID;
    if (b->broken) return TENT_ERR_STATE;
    if (!b->planned) { *remaining = b->dev.n_slices; return TENT_OK; }
    DeviceGuard g(ctx->device);
    if (!g.ok) return TENT_ERR_HIP;
    hipStream_t s = static_cast<hipStream_t>(stream);
    // slices are marked DONE ahead of their copies: completion is only reported once the last
    // execute's copies have ended, whichever stream the caller polls on
    if (b->done_recorded && s != b->exec_stream) HIP_TRY(hipStreamWaitEvent(s, b->done_event, 0));
    HIP_TRY(launch_count_remaining(b->dev, s));
    HIP_TRY(hipMemcpyAsync(ctx->host_plan, b->dev.plan, sizeof(PlanState), hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    *remaining = ctx->host_plan->n_remaining;
    return TENT_OK;
}

int tent_reset(tent_ctx* ctx, tent_batch_t batch, void* stream)
{
    if (!ctx) return TENT_ERR_INVALID;
    Batch* b = find_batch(ctx, batch);
    if (!b) return TENT_ERR_INVALID;
    DeviceGuard g(ctx->device);
    if (!g.ok) return TENT_ERR_HIP;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (b->planned) {
        StreamNote note(*b, s);
        // the reset must not overtake the copies of an execute that runs on another stream
        if (b->done_recorded && s != b->exec_stream && !capturing(s)) HIP_TRY(hipStreamWaitEvent(s, b->done_event, 0));
        HIP_TRY(launch_reset(b->dev, s));
    }
    b->planned = false;
    b->has_done = false;
    b->has_retry = false;
    b->broken = false;
    return TENT_OK;
}

int tent_slice_count(tent_ctx* ctx, tent_batch_t batch, uint64_t* n_slices)
{
    if (!ctx || !n_slices) return TENT_ERR_INVALID;
    Batch* b = find_batch(ctx, batch);
    if (!b) return TENT_ERR_INVALID;
    *n_slices = b->dev.n_slices;
    return TENT_OK;
}

int tent_get_plan(tent_ctx* ctx, tent_batch_t batch, tent_slice* host_out, uint64_t cap)
{
    if (!ctx || !host_out) return TENT_ERR_INVALID;
    Batch* b = find_batch(ctx, batch);
    if (!b) return TENT_ERR_INVALID;
    if (!b->planned) return TENT_ERR_STATE;
    const BatchDev& d = b->dev;
    const uint64_t n = d.n_slices;
    if (cap < n) return TENT_ERR_RANGE;
    DeviceGuard g(ctx->device);
    if (!g.ok) return TENT_ERR_HIP;
    HIP_TRY(hipDeviceSynchronize());
    std::vector<uint32_t> desc, len, rail;
    std::vector<uint64_t> off, stage;
    std::vector<uint8_t> state;
    try {
        desc.resize(n); len.resize(n); rail.resize(n); off.resize(n); stage.resize(n); state.resize(n);
    } catch (const std::bad_alloc&) { return TENT_ERR_NOMEM; }
    HIP_TRY(hipMemcpy(desc.data(), d.s_desc, n * 4, hipMemcpyDeviceToHost));
    HIP_TRY(hipMemcpy(len.data(), d.s_len, n * 4, hipMemcpyDeviceToHost));
    HIP_TRY(hipMemcpy(rail.data(), d.s_rail, n * 4, hipMemcpyDeviceToHost));
    HIP_TRY(hipMemcpy(off.data(), d.s_off, n * 8, hipMemcpyDeviceToHost));
    HIP_TRY(hipMemcpy(stage.data(), d.s_stage_off, n * 8, hipMemcpyDeviceToHost));
    HIP_TRY(hipMemcpy(state.data(), d.s_state, n, hipMemcpyDeviceToHost));
    for (uint64_t i = 0; i < n; ++i)
        host_out[i] = tent_slice{desc[i], len[i], off[i], stage[i], rail[i], state[i]};
    return TENT_OK;
}

int tent_get_timings(tent_ctx* ctx, float* ms_out, uint32_t* launches_out)
{
    if (!ctx || !ms_out || !launches_out) return TENT_ERR_INVALID;
    if (!(ctx->cfg.flags & TENT_FLAG_PROFILE)) return TENT_ERR_STATE;
    DeviceGuard g(ctx->device);
    if (!g.ok) return TENT_ERR_HIP;
    int rc = TENT_OK;
    for (int st = 0; st < TENT_T_COUNT; ++st) {
        Timing& t = ctx->timing[st];
        double total = 0.0;
        for (size_t k = 0; k < t.used; ++k) {
            float ms = 0.0f;
            if (hipEventSynchronize(t.pool[k].second) != hipSuccess ||
                hipEventElapsedTime(&ms, t.pool[k].first, t.pool[k].second) != hipSuccess) {
                (void)hipGetLastError();
                rc = TENT_ERR_HIP;
            }
            total += ms;
        }
        ms_out[st] = (float)total;
        launches_out[st] = (uint32_t)t.used;
        t.used = 0;
    }
    return rc;
}

int tent_release(tent_ctx* ctx, tent_batch_t batch)
{
    if (!ctx) return TENT_ERR_INVALID;
    Batch* b = find_batch(ctx, batch);
    if (!b) return TENT_ERR_INVALID;
    DeviceGuard g(ctx->device);
    if (!g.ok) return TENT_ERR_HIP;
    wait_batch_idle(*b);
    free_batch(ctx, *b);
    return TENT_OK;
}

}  // extern "C"
