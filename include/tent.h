/*
 * tent.h -- C ABI of the MI355X slice-spraying engine.
 *
 * The engine implements the data-parallel hot path of TENT's data plane on one
 * GPU: declared transfer intents are cut into fixed-size slices, every slice is
 * late-bound to a rail by the predicted-completion cost model, and the slice
 * bytes move paged source -> per-rail contiguous staging region -> destination,
 * all in device memory.  Rails are simulated: a rail is a staging region plus a
 * telemetry record.
 *
 * Conventions for every call
 *   - Return value: TENT_OK (0) or a negative tent_status.  TENT_DEFER (+1) is
 *     returned by tent_plan when no rail is admitted.  Nothing is printed, no
 *     exception crosses the boundary, the process is never aborted.
 *   - "host" pointers are ordinary process memory and are copied before the call
 *     returns.  "device" pointers are HIP device memory owned by the caller; the
 *     library borrows them until tent_destroy.
 *   - A context is bound to the HIP device that was current in tent_create and
 *     must be used by one host thread at a time.
 *   - `stream` arguments are hipStream_t values passed as void* (NULL = the
 *     default stream).  Calls that take a stream only enqueue work unless stated.
 *   - Calls on one batch are ordered by the caller: on one stream, or across streams by events
 *     of the caller's.  One ordering the library provides by itself: tent_plan and
 *     tent_plan_dispatch on another stream than the batch's last tent_execute wait (on the
 *     device) for that execute's bookkeeping only -- staging addresses resolved, slices marked
 *     DONE -- and may then run beside its copies, which read none of what a re-plan writes.
 *     That is what overlaps the re-planning of the unfinished slices with the data movement of
 *     the finished ones.  The next tent_execute must still come after that plan (the
 *     host-side wait of tent_sim_advance with n_done != NULL, or an event).
 *   - HIP graphs: tent_reset, tent_plan with info = NULL and tent_execute allocate nothing, copy
 *     nothing from or to the host and enqueue kernels only (no memset nodes), so a caller may
 *     record them on a capturing stream and replay the graph.  The host-side bookkeeping of a
 *     batch (planned / moved) changes when the call is made, i.e. at capture time, so a recorded
 *     sequence should be a whole cycle: tent_reset, tent_plan, tent_execute.  Calls that read
 *     results back (info != NULL, tent_poll, tent_get_*, tent_sim_advance, tent_update_bandwidth)
 *     or take host arrays per call (tent_plan_dispatch with priorities) are not for capture.
 */
#ifndef TENT_H
#define TENT_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct tent_ctx tent_ctx;     /* opaque engine instance                                   */
typedef uint64_t tent_batch_t;        /* what the application holds for a batch (Section 3)      */

typedef enum {
    TENT_OK          =  0,
    TENT_DEFER       =  1,   /* no admitted rail: nothing bound (Algorithm 1, Stage 1)          */
    TENT_ERR_INVALID = -1,   /* null pointer, malformed descriptor list, unknown handle          */
    TENT_ERR_RANGE   = -2,   /* fixed-point precondition, rail count, arena or table capacity    */
    TENT_ERR_STATE   = -3,   /* call out of order (e.g. execute before plan)                     */
    TENT_ERR_NOMEM   = -4,   /* host or device allocation failed                                 */
    TENT_ERR_HIP     = -5    /* a HIP runtime call failed                                        */
} tent_status;

enum { TENT_MAX_RAILS = 64 };
enum { TENT_STATIC_WORKSPACE_BYTES = 64 << 20 };   /* static device array behind tent_declare_static, per GPU */

/* tent_config.flags */
enum {
    TENT_FLAG_SKIP_OVERLAP_CHECK = 1u << 0,   /* tent_declare does not test extents for overlap  */
    TENT_FLAG_PROFILE            = 1u << 1,   /* time every stage with HIP events (see tent_get_timings) */
    TENT_FLAG_SERIAL_BINDING     = 1u << 2,   /* bind slice by slice on one wavefront instead of run-parallel  */
    TENT_FLAG_BOUNDED_STAGING    = 1u << 3    /* the arena is a bounded buffer: plans do not require it to hold the
                                                 payload and tent_execute_bounded becomes available             */
};

typedef struct {
    uint64_t slice_bytes;      /* S in [1, 2^31]: fixed slice size (Section 4.2, "Slice Decomposition") */
    void    *staging_arena;    /* device: per-rail staging regions are carved from this           */
    uint64_t staging_bytes;    /* capacity of the arena                                           */
    uint32_t flags;
    uint32_t max_rails;        /* most rails a plan may name, 0 = TENT_MAX_RAILS (sizes per-batch tables) */
} tent_config;

/* One contiguous byte range of a registered segment (Section 3.1: a segment is a
 * named memory range; here it is reduced to a device base pointer and a length). */
typedef struct {
    uint32_t seg;              /* id returned by tent_register_segment                            */
    uint32_t len;              /* bytes, > 0                                                      */
    uint64_t off;              /* byte offset inside the segment                                  */
} tent_extent;

/* Telemetry of one rail: the quantities of Eq. 1 (Section 4.2) in integer units. */
typedef struct {
    uint32_t bw_MBps;          /* B_d: bandwidth estimate in 10^6 bytes/s, > 0                    */
    uint32_t lat_ns;           /* beta0_d: fixed latency                                          */
    uint64_t queued_bytes;     /* A_d: bytes already in flight on the rail                        */
    uint16_t beta1_q8;         /* beta1_d in Q8.8 (256 = 1.0)                                     */
    uint16_t penalty_q8;       /* topology penalty P_d in Q8.8 (256 = 1.0)                        */
    uint8_t  health;           /* 0 healthy, 1 degraded (cost counts twice), 2 excluded (never chosen) */
} tent_rail_state;

typedef struct {
    uint64_t n_slices;                       /* slices bound by this call                          */
    uint64_t n_pending_before;               /* slices that were not DONE when the call started    */
    uint64_t rail_bytes[TENT_MAX_RAILS];     /* bytes bound per rail by this call                  */
    uint64_t rail_slices[TENT_MAX_RAILS];    /* slices bound per rail by this call                 */
    uint64_t queued_after[TENT_MAX_RAILS];   /* A_d after this call = queued_bytes + rail_bytes    */
    uint64_t stage_base[TENT_MAX_RAILS];     /* byte offset of each rail's region in the arena     */
} tent_plan_info;

enum { TENT_SLICE_PENDING = 0, TENT_SLICE_BOUND = 1, TENT_SLICE_DONE = 2 };

/* Calibration of one rail's bandwidth probe (Section 4.2, Eq. 2 and the smoothing filter). */
typedef struct {
    uint32_t hw_MBps;          /* B_hw: bandwidth reported by the hardware, 10^6 bytes/s            */
    uint32_t alpha_q8;         /* alpha in Q8.8 (256 = 1.0), at most 65535                          */
    uint32_t delta_ns;         /* delta: latency that carries no rate information                   */
    uint32_t ewma_q8;          /* weight of the new probe in Q8.8, 0..256 (256 replaces the estimate) */
} tent_probe_params;

/* Request-level dispatch (Algorithm 1, Stage 3; Section 4.2 "Slice Dispatching", "Quality of Service"). */
typedef struct {
    uint64_t theta_bytes;      /* theta: a transfer shorter than this is a mice flow                 */
    uint32_t gamma_q8;         /* gamma in Q8.8 (at most 65535): mice candidates cost at most
                                  s_min + floor(gamma_q8 * s_min / 256)                               */
    uint32_t window;           /* index of the current priority window (see tent_plan_dispatch)      */
    uint64_t rr_start;         /* round-robin counter before the call                                */
} tent_dispatch_params;

typedef struct {
    tent_plan_info plan;       /* as for tent_plan; n_pending_before counts only slices of requests that were dispatched */
    uint64_t n_mice;           /* requests dispatched as mice flows                                  */
    uint64_t n_elephant;       /* requests dispatched as elephant flows                              */
    uint64_t n_deferred;       /* requests left pending because no rail admitted their priority      */
    uint64_t rr_next;          /* round-robin counter after the call = rr_start + n_mice             */
} tent_dispatch_info;

enum { TENT_PRIO_LOW = 0, TENT_PRIO_MID = 1, TENT_PRIO_HIGH = 2 };
enum { TENT_MODE_NONE = 0, TENT_MODE_MICE = 1, TENT_MODE_ELEPHANT = 2, TENT_MODE_DEFERRED = 3 };

/* Rail health monitor (Section 4.3, "Health Monitoring"): parameters and the record kept per rail. */
typedef struct {
    uint32_t err_threshold;    /* a rail pauses once 2*hard + congestion errors exceed 2*err_threshold */
    uint32_t recover_windows;  /* clean windows after which a DEGRADED rail is HEALTHY again           */
    uint32_t cooldown_windows; /* length of the first pause; every further pause is twice as long      */
    uint32_t degrade_q8;       /* a window whose probe is below degrade_q8/256 of the estimate is a
                                  degradation event (Q8.8; 0 switches the test off)                   */
} tent_monitor_params;

typedef struct {
    uint32_t state;            /* 0 HEALTHY, 1 DEGRADED, 2 PAUSED: the value for tent_rail_state.health */
    uint32_t score;            /* weighted errors of the current run of windows with errors            */
    uint32_t clean;            /* consecutive clean windows of a DEGRADED rail                         */
    uint32_t cooldown_left;    /* windows a PAUSED rail stays excluded                                 */
    uint32_t cooldown_next;    /* length of the next pause                                             */
} tent_rail_monitor;

/* One row of the slice table: the task triple <path, offset, length> of
 * Algorithm 1 plus the bookkeeping of the staging hop. */
typedef struct {
    uint32_t desc;             /* descriptor (transfer) the slice belongs to                      */
    uint32_t len;              /* bytes                                                           */
    uint64_t off;              /* absolute byte offset inside the transfer                        */
    uint64_t stage_off;        /* byte offset inside the rail's staging region                    */
    uint32_t rail;             /* rail index; 0xFFFFFFFF while never bound                        */
    uint32_t state;            /* TENT_SLICE_*                                                    */
} tent_slice;

/* Stage indices of tent_get_timings. */
enum {
    TENT_T_EXTENT_SCAN = 0,    /* prefix sums over extent lengths (source and destination)        */
    TENT_T_SLICE_SCAN  = 1,    /* per-descriptor slice counts and their exclusive scan            */
    TENT_T_EXPAND      = 2,    /* slice-table expansion                                           */
    TENT_T_COMPACT     = 3,    /* pending-list compaction (re-planning only)                      */
    TENT_T_BIND        = 4,    /* rail assignment                                                 */
    TENT_T_GATHER      = 5,    /* paged source -> staging                                         */
    TENT_T_SCATTER     = 6,    /* staging -> destination                                          */
    TENT_T_FEEDBACK    = 7,    /* bandwidth probe over the completed slices (tent_update_bandwidth) */
    TENT_T_COUNT       = 8
};

/* Create an engine on the current HIP device.  `cfg` is host memory. */
int tent_create(tent_ctx **out, const tent_config *cfg);

/* Release every batch and all device memory the library allocated.  Waits for the device. */
int tent_destroy(tent_ctx *ctx);

/* Register a device memory range as a segment.  *seg_out receives its id (0, 1, ...). */
int tent_register_segment(tent_ctx *ctx, void *dev_base, uint64_t len, uint32_t *seg_out);

/*
 * Declare a batch of transfers (Section 3: the application states what to move
 * and receives a handle).  Transfer j moves the byte string formed by
 * concatenating src_ext[src_ptr[j] .. src_ptr[j+1]) onto the byte string formed
 * by dst_ext[dst_ptr[j] .. dst_ptr[j+1]); both strings must have the same
 * length.  All four arrays are host memory in CSR form (ptr arrays have
 * n_desc+1 entries, ptr[0] = 0, nondecreasing).
 * Errors: TENT_ERR_INVALID for null pointers, n_desc = 0, an empty transfer, a
 * zero-length extent, an extent outside its segment, or unequal source and
 * destination lengths; TENT_ERR_RANGE when the batch holds more than 2^32-2 slices.
 * The call returns as soon as the host arrays are checked and copied (Section 4.1: submitting a
 * transfer returns immediately; batches of more than 128 Ki extents are walked by up to four host
 * threads that end with the call): the upload of the descriptors, the ordering of the destination extents by
 * address and the overlap check run on a stream of the library's own (default priority) and hold up
 * none of the caller's streams.  Unless TENT_FLAG_SKIP_OVERLAP_CHECK is set, a destination extent
 * that overlaps another destination extent or any source extent of the batch makes the batch
 * invalid; that verdict comes from the device and is delivered by the first tent_plan or
 * tent_plan_dispatch on the batch, which waits for it, returns TENT_ERR_INVALID and releases the
 * batch.
 * Device tables for the batch are set up here, not in plan or execute: they come from one device
 * allocation per batch, and the allocations of released batches are kept and handed to later
 * declarations of similar size, so a loop of declare ... release settles into allocating nothing.
 */
int tent_declare(tent_ctx *ctx, uint32_t n_desc,
                 const uint32_t *src_ptr, const tent_extent *src_ext,
                 const uint32_t *dst_ptr, const tent_extent *dst_ext,
                 tent_batch_t *out);

/*
 * tent_declare for callers that cannot allocate: code that runs where hipMalloc is forbidden (tight
 * serving loops, harnesses that ban allocation, set-up phases of graph-driven pipelines).  Same
 * arguments, same checks and the same batch as tent_declare, but the batch's device tables and the
 * workspace of the address sort are carved from a static device array of the library
 * (TENT_STATIC_WORKSPACE_BYTES = 64 MiB per GPU, held by every GPU the library runs on until the
 * process ends) and the call allocates nothing, neither on the device nor on the host; host arrays
 * larger than the context's pinned buffer are uploaded through it piece by piece, each piece waited for.
 * TENT_ERR_RANGE when tables plus workspace exceed the static array (about 75 bytes per extent,
 * 70 bytes per slice and 60 bytes per 4 KiB tile of payload: batches up to about 2 GiB of payload in
 * 32 KiB pages fit).
 * One static batch exists per GPU: the array keeps the last call's contents, and every call clears
 * what must start at zero.  A new call from the same context waits for and replaces that context's
 * previous static batch; a call from another context on the same GPU invalidates the other context's
 * static batch (its handle turns TENT_ERR_INVALID) without waiting for it, so calls that overlap on
 * one GPU race and are the caller's to order.  The returned handle works with every other entry
 * point; tent_release gives the array up without freeing anything.
 */
int tent_declare_static(tent_ctx *ctx, uint32_t n_desc,
                        const uint32_t *src_ptr, const tent_extent *src_ext,
                        const uint32_t *dst_ptr, const tent_extent *dst_ext,
                        tent_batch_t *out);

/*
 * Split and bind (Section 4.2; Algorithm 1 Stages 1-2; Eq. 1).
 * On a batch without DONE or failed slices the slice table is (re)built on the device:
 * slice k of transfer j covers bytes [k*S, min((k+1)*S, len_j)).  Then every
 * slice that is not DONE is bound, in ascending slice index, to the admitted
 * rail (health != 2) with the smallest
 *     c0_d + (((A_d + len) * c1_d) >> 16),
 *     c1_d = floor(1e6 * beta1_q8 * penalty_q8 / bw_MBps),  c0_d = (lat_ns*1000*penalty_q8) >> 8
 * (picoseconds; ties to the lowest rail index; both coefficients are doubled for a rail with
 * health = 1: Section 4.3, a degraded rail keeps half its weight), after which A_d += len.  The
 * slice's staging offset is the number of bytes bound to that rail earlier in
 * this call.  Rail d's staging region starts at the sum over d' < d of the
 * rail totals rounded up to 256 bytes.  Slices that failed on a rail (tent_sim_fail) are
 * bound by rotation ahead of this pass; see there.
 * `rails` is host memory (n_rails <= TENT_MAX_RAILS).  `info` is host memory or
 * NULL; when it is non-NULL the call waits for the stream and fills it, when it
 * is NULL the call only enqueues work on `stream`.
 * Returns TENT_DEFER (and binds nothing) when every rail is excluded;
 * TENT_ERR_INVALID for a health value above 2 (and for a batch that failed its overlap check, see
 * tent_declare); TENT_ERR_RANGE when n_rails exceeds the context's max_rails, bw_MBps = 0,
 * c1_d >= 2^32, (max A_d + the batch's payload) * max c1_d >= 2^63, or the arena is smaller than the
 * batch's payload + 256*n_rails; TENT_ERR_STATE for a batch whose last tent_execute failed half way
 * (see there).
 */
int tent_plan(tent_ctx *ctx, tent_batch_t batch, const tent_rail_state *rails, uint32_t n_rails,
              tent_plan_info *info, void *stream);

/*
 * Split and dispatch request by request (Algorithm 1, Stages 1-3; Section 4.2 "Slice Dispatching"
 * and "Quality of Service") -- the alternative to tent_plan's per-slice rule.  Transfers are taken
 * in declaration order; for each one with slices that are not DONE:
 *   Stage 1  admitted rails = rails with health != 2 whose priority slot accepts priority[j]
 *            (TENT_PRIO_*; NULL = every transfer is HIGH): rail d sits in slot (window + d) mod 3,
 *            slot 0 accepts HIGH only, slot 1 HIGH and MID, slot 2 everything.  With no admitted rail
 *            the transfer is deferred: its slices are left PENDING.
 *   Stage 2  s_d = c0_d + (((A_d + L) * c1_d) >> 16) with A_d as it stands before the transfer
 *            (coefficients as for tent_plan).
 *   Stage 3  transfer length < theta_bytes (mice, L = transfer length): the whole transfer goes to
 *            candidate number rr mod |C| of C = admitted rails with
 *            s_d <= s_min + floor(gamma_q8 * s_min / 256), ascending rail index, and rr advances by one;
 *            otherwise (elephant, L = length of the transfer's first slice): its slices that are not
 *            DONE are dealt in ascending index, each to the admitted rail with the smallest
 *            (m_d + 1) * max(s_d, 1), m_d = slices of this transfer already dealt to d, ties to the
 *            lowest rail index (weighted proportional spraying with weights 1 / s_d).
 * Every dealt slice becomes BOUND, adds its bytes to A_d and takes the next bytes of the rail's
 * staging region; region bases as for tent_plan.  Retry counts play no part here.
 * `rails`, `params`, `priority` (n_desc bytes or NULL) and `info` (or NULL) are host memory; with
 * info = NULL the call only enqueues.  Returns TENT_DEFER when every rail is excluded (nothing is
 * touched); TENT_ERR_INVALID for a priority above 2; TENT_ERR_RANGE as for tent_plan, for
 * gamma_q8 > 65535, and when (largest slice count of a transfer + 1) * (largest cost a rail can
 * reach) is 2^57 or more.
 */
int tent_plan_dispatch(tent_ctx *ctx, tent_batch_t batch, const tent_rail_state *rails, uint32_t n_rails,
                       const tent_dispatch_params *params, const uint8_t *priority,
                       tent_dispatch_info *info, void *stream);

/* Copy what the last tent_plan_dispatch did with every transfer (TENT_MODE_*, one byte each) to
 * host memory for verification.  Waits for the device.  TENT_ERR_RANGE if cap < number of transfers. */
int tent_get_modes(tent_ctx *ctx, tent_batch_t batch, uint8_t *host_out, uint64_t cap);

/*
 * Rail simulator used by the re-planning workload (not an operation of the
 * paper): rail d drains, in order, its queued_bytes and then the slices bound
 * to it by the last tent_plan.  A BOUND slice stays BOUND iff
 * queued_bytes_d + stage_off + len <= budget_bytes[d]; otherwise it returns to
 * PENDING and will be re-planned (Section 4.3, idempotent retry).
 * `budget_bytes` is host memory with n_rails entries.  With n_done != NULL the call waits for
 * the stream and *n_done (host) receives the number of slices that stayed BOUND; with
 * n_done == NULL it only enqueues.  Either way the next tent_execute sizes its copy launches by
 * what can have stayed BOUND (at most budget_d - queued_bytes_d bytes per rail, and the count
 * when it was read back).
 */
int tent_sim_advance(tent_ctx *ctx, tent_batch_t batch, const uint64_t *budget_bytes,
                     uint64_t *n_done, void *stream);

/*
 * Rail simulator, hard errors (Section 4.3, "Link-Level Resilience"; the injection itself is not an
 * operation of the paper): every BOUND slice on a rail d with rail_failed[d] != 0 returns to PENDING
 * and its retry count goes up by one (saturating at 255).  Call it after tent_plan and before
 * tent_sim_advance / tent_execute.  `rail_failed` is host memory with one entry per rail of the last
 * tent_plan; `failed_per_rail` (host, same length, or NULL) receives the number of slices that failed
 * on each rail, and when it is non-NULL the call waits for the stream.
 *
 * The next tent_plan treats slices with a retry count differently: they are issued first, in
 * ascending slice index, without the cost model -- slice i on its k-th retry takes candidate number
 * (i + k) mod |C| of the candidate set C = the HEALTHY rails, or, when there is none, the DEGRADED
 * rails with penalty_q8 <= 256, or, when there is none either, all DEGRADED rails (ascending rail
 * index) -- and their bytes are added to A_d and to the rails' staging regions before the remaining
 * slices are bound by predicted cost.
 */
int tent_sim_fail(tent_ctx *ctx, tent_batch_t batch, const uint8_t *rail_failed,
                  uint64_t *failed_per_rail, void *stream);

/* Copy the slices' retry counts (one byte per slice) to host memory for verification.  Waits for
 * the device.  TENT_ERR_RANGE if cap is smaller than the slice count. */
int tent_get_retries(tent_ctx *ctx, tent_batch_t batch, uint8_t *host_out, uint64_t cap);

/*
 * Rail health monitor (Section 4.3, "Health Monitoring"), host arithmetic only, no context needed.
 * tent_monitor_init sets n_rails records to HEALTHY.  tent_monitor_update advances them by one
 * measurement window and writes each rail's state into rails[d].health:
 *   - a PAUSED rail ignores its inputs; its cooldown runs down by one and at zero it returns as
 *     DEGRADED;
 *   - otherwise errors = 2*hard_errors[d] + congestion_errors[d] are added to the score (a window
 *     without errors clears the score); a score above 2*err_threshold pauses the rail for
 *     cooldown_next windows and doubles cooldown_next;
 *   - otherwise any error, or a probe with probe_MBps[d] != 0 and
 *     256*probe_MBps[d] < degrade_q8*bw_before_MBps[d], makes the rail DEGRADED;
 *   - otherwise a DEGRADED rail counts a clean window and after recover_windows of them becomes
 *     HEALTHY, with cooldown_next back at cooldown_windows.
 * All arrays are host memory with n_rails entries (probe_MBps as returned by tent_update_bandwidth,
 * bw_before_MBps the estimates the planner held during the window).
 * TENT_ERR_INVALID for null pointers or a record with an unknown state, TENT_ERR_RANGE for n_rails
 * outside [1, TENT_MAX_RAILS].
 */
int tent_monitor_init(const tent_monitor_params *params, tent_rail_monitor *mon, uint32_t n_rails);
int tent_monitor_update(const tent_monitor_params *params, tent_rail_monitor *mon, tent_rail_state *rails,
                        uint32_t n_rails, const uint32_t *hard_errors, const uint32_t *congestion_errors,
                        const uint32_t *probe_MBps, const uint32_t *bw_before_MBps);

/*
 * Rail simulator, second half (not an operation of the paper): the end-to-end latency of
 * every BOUND slice, tau = lat_ns_d + ceil((queued_bytes_d + stage_off + len) * 1000 / true_bw_MBps[d])
 * nanoseconds, i.e. the rail drains what was queued before the last tent_plan, then the slices
 * staged ahead of this one, then the slice, at its true bandwidth.  lat_ns and queued_bytes are
 * those of the last tent_plan.  `true_bw_MBps` is host memory with n_rails entries, all > 0.
 * Call it after tent_sim_advance and before tent_execute.  Only enqueues on `stream`.
 * TENT_ERR_RANGE when queued bytes plus payload reach 2^53.
 */
int tent_sim_latency(tent_ctx *ctx, tent_batch_t batch, const uint32_t *true_bw_MBps, void *stream);

/*
 * Telemetry feedback (Section 4.2, Eq. 2): over the measurement window formed by the BOUND
 * slices of the batch and their recorded latencies,
 *     B_probe_d = min{ hw_MBps_d, max_i floor(alpha_q8 * len_i * 1000 / (256 * (tau_i - delta_ns))) }
 * (a slice with tau_i <= delta_ns counts as a sample at hw_MBps_d), and the estimate follows
 *     bw_MBps_d <- max(1, (ewma_q8 * B_probe_d + (256 - ewma_q8) * bw_MBps_d) >> 8).
 * A rail without a BOUND slice keeps its estimate.  `params` (host, n_rails entries) is read,
 * `rails` (host, n_rails entries) has its bw_MBps fields updated in place, `probe_MBps_out` (host,
 * n_rails entries or NULL) receives B_probe_d, 0 where the rail had no sample.  n_rails must equal
 * the rail count of the last tent_plan.  Waits for `stream`.
 */
int tent_update_bandwidth(tent_ctx *ctx, tent_batch_t batch, const tent_probe_params *params,
                          tent_rail_state *rails, uint32_t n_rails, uint32_t *probe_MBps_out, void *stream);

/* Copy the recorded slice latencies (ns, one per slice; meaningful for slices that were BOUND at
 * the last tent_sim_latency) to host memory for verification.  Waits for the device. */
int tent_get_latencies(tent_ctx *ctx, tent_batch_t batch, uint64_t *host_out, uint64_t cap);

/*
 * Move every BOUND slice: gather its bytes from the paged source extents into
 * its rail's staging region, then scatter from staging to the destination
 * extents at the slice's absolute offset (Section 4.1 staging hop; Section 4.4
 * direct-to-offset writes), and mark it DONE.  Enqueues on `stream` and
 * returns; the caller synchronises the stream or polls.  The DONE marks are enqueued
 * ahead of the copies (the copies are driven by address tables, not by slice
 * state), which is what lets a re-plan on another stream run beside the copies; tent_poll, on
 * any stream, waits for the end of the copies before it counts, so completion is never reported
 * while bytes are still moving.  TENT_ERR_STATE if the batch was never planned.  A batch with no
 * BOUND slice is a no-op.
 * Should a launch fail after the slices were marked (TENT_ERR_HIP), the batch is flagged: every
 * later call on it but tent_reset (which clears the flag and returns all slices to PENDING, so
 * the bytes are moved again) and tent_release returns TENT_ERR_STATE.
 */
int tent_execute(tent_ctx *ctx, tent_batch_t batch, void *stream);

/*
 * Move every BOUND slice through a staging arena that is smaller than the payload (Section 4.1:
 * the payload is partitioned into chunks that pass through an intermediate buffer).  The payload --
 * the transfers' bytes laid end to end in declaration order -- is cut into chunks of chunk_bytes;
 * for every chunk in turn the BOUND bytes of the chunk are gathered into the arena and then written
 * to their destination.  Inside the arena every rail keeps one contiguous region per chunk: the
 * chunk's bytes on rail d form an interval [lo_d, hi_d) of the rail's staging offsets and sit at
 * region_base_d + (offset - lo_d), region_base_d being the exclusive sum over rails of (hi_d - lo_d)
 * rounded up to 256 bytes.  The arena is used as `slots` (1 or 2) slots of chunk_bytes + 256 * n_rails
 * bytes; chunk c lives in slot c mod slots.  With two slots the gather of chunk c + 1 overlaps the
 * scatter of chunk c: gathers are enqueued on `stream`, scatters on a stream of the library's own
 * (default priority), ordered by events, and `stream` is made to wait for the last scatter, so work
 * enqueued on `stream` afterwards sees the batch complete.  Slices are marked DONE as by
 * tent_execute.  Only enqueues.
 * Which to use: one slot.  Both stages of a chunk are bound by the device memory's bandwidth, so
 * overlapping them adds none; measured on MI355X, two slots ran between 5 % faster and 2 % slower
 * than one and need twice the arena.  Two slots are there for a caller whose second stage is not
 * a device copy of its own device's memory.
 * Lengths and addresses may be anything: when every extent length and the slice size are multiples of
 * 1 KiB the chunks are moved by table-driven copies, otherwise byte-exactly in ranges of 1 KiB of the
 * payload (slower).
 * Needs a context created with TENT_FLAG_BOUNDED_STAGING (else TENT_ERR_STATE).  TENT_ERR_INVALID
 * unless chunk_bytes is a positive multiple of 1 MiB and slots is 1 or 2; TENT_ERR_RANGE when the
 * slots exceed the arena or when the payload needs more than 4096 chunks.  Should a chunk's regions not fit the arena after all
 * (possible only when the BOUND slices of a rail are not a contiguous run of its staging offsets),
 * nothing is moved and the slices stay BOUND: tent_poll then still reports them.
 * With the flag set tent_execute returns TENT_ERR_RANGE when the arena cannot hold the payload.
 */
int tent_execute_bounded(tent_ctx *ctx, tent_batch_t batch, uint64_t chunk_bytes, uint32_t slots, void *stream);

/* Batch-level completion (Section 4.4): *remaining (host) receives the number of
 * slices not DONE.  Waits for `stream`, which is first made to wait for the copies of the batch's
 * last execute if that ran on another stream: 0 means every byte of the batch has landed. */
int tent_poll(tent_ctx *ctx, tent_batch_t batch, uint64_t *remaining, void *stream);

/* Return every slice of the batch to PENDING (the next tent_plan rebuilds the table). */
int tent_reset(tent_ctx *ctx, tent_batch_t batch, void *stream);

/* Number of slices of the batch (known after tent_declare). */
int tent_slice_count(tent_ctx *ctx, tent_batch_t batch, uint64_t *n_slices);

/* Copy the slice table to host memory for verification.  `cap` = entries available in
 * host_out; TENT_ERR_RANGE if too small.  Waits for the device. */
int tent_get_plan(tent_ctx *ctx, tent_batch_t batch, tent_slice *host_out, uint64_t cap);

/* With TENT_FLAG_PROFILE every stage (TENT_T_*) of tent_plan / tent_execute is bracketed by a
 * pair of HIP events on the caller's stream.  This call waits for the recorded events and
 * returns, per stage, the summed milliseconds and the number of bracketed intervals since
 * the previous call (0 for stages that did not run), then starts a new accounting period.
 * `ms_out` and `launches_out` are host memory with TENT_T_COUNT entries each. */
int tent_get_timings(tent_ctx *ctx, float *ms_out, uint32_t *launches_out);

/* Give up the batch.  Waits (on the host) for the work that the library's calls enqueued for this
 * batch, on whichever streams, and for nothing else; its device tables are kept for a later
 * declaration of similar size or freed. */
int tent_release(tent_ctx *ctx, tent_batch_t batch);

/*
 * Timed probe copy: an aid for laying out the caller's pools, not an operation of the paper.
 * On MI355X a copy whose read side and write side lie in the same third of the device memory runs
 * several per cent slower than one that crosses thirds, and nothing tells which third an address
 * is in; a caller times this probe for pairs of candidate windows and keeps the partners of a
 * copy (source pool / staging arena, staging arena / destination pool) in different ones.
 * The probe copies `bytes` from `read_window` to `write_window` (both device memory, at least
 * `bytes` long, contents of the write window are overwritten): pages of `page_bytes` are read in
 * a scattered order and written in 4 KiB blocks to eight frontiers that advance through the
 * write window side by side, as a gather into several rails' regions does.  Every block of
 * the read window lands exactly once.  `page_bytes` is a power of two >= 4096,
 * `bytes / page_bytes` a power of two.  Needs no context.  The copy runs `repeats` times on
 * `stream`, the call waits for each, and `*ms_out` (host) receives the shortest duration.
 * TENT_ERR_INVALID for a null pointer or sizes that break the rules above.
 */
int tent_probe_copy(const void *read_window, void *write_window, uint64_t bytes, uint32_t page_bytes,
                    uint32_t repeats, void *stream, float *ms_out);

/* Static description of a status code. */
const char *tent_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* TENT_H */
