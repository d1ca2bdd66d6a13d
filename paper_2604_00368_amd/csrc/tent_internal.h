// Internal declarations shared by the engine's translation units (host runtime + HIP kernels).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/tent.h"

namespace tent {

// Rail cost coefficients and simulator inputs, passed to kernels by value (kernarg segment),
// so that a plan needs no host-to-device upload.  Cost of rail d for a slice of L bytes
// (Eq. 1 of the paper scaled by the topology penalty, in picoseconds):
//     c0[d] + (((A[d] + L) * c1[d]) >> 16)
struct RailParams {
    uint64_t c0[TENT_MAX_RAILS];
    uint64_t c1[TENT_MAX_RAILS];
    uint64_t A[TENT_MAX_RAILS];      // queued bytes at the start of the plan
    uint64_t admitted;               // bit d set: rail d may receive slices
    uint32_t n_rails;
    uint32_t pad;
};

// Rail simulator inputs for slice latencies.
struct LatencyParams {
    uint64_t queued[TENT_MAX_RAILS];
    uint32_t lat_ns[TENT_MAX_RAILS];
    uint32_t bw_MBps[TENT_MAX_RAILS];   // true bandwidth, > 0
};

// Bandwidth-probe calibration and current estimates.
struct ProbeParams {
    tent_probe_params cal[TENT_MAX_RAILS];
    uint32_t bw_MBps[TENT_MAX_RAILS];   // estimates before the window
    uint32_t n_rails;
};

struct BudgetParams {
    uint64_t queued[TENT_MAX_RAILS];
    uint64_t budget[TENT_MAX_RAILS];
};

// Candidate rails of the retry rotation (Section 4.3, "Link-Level Resilience"), in rotation order.
struct RotateParams {
    uint8_t  cand[TENT_MAX_RAILS];
    uint32_t n_cand;
};

// Request-level dispatch (Algorithm 1): thresholds and, per priority level, the rails whose current
// priority slot admits a request of that level (already intersected with the non-excluded rails).
struct DispatchParams {
    uint64_t theta;              // requests shorter than this are mice flows
    uint64_t rr_start;           // round-robin counter before the call
    uint64_t adm[3];             // admitted-rail masks for priorities LOW, MID, HIGH
    uint32_t gamma_q8;           // cost tolerance of the mice candidate set, Q8.8
    uint32_t all_high;           // 1: no priority array was given, every request counts as HIGH
};

// Rails that report a hard error to the rail simulator.
struct FailParams {
    uint8_t failed[TENT_MAX_RAILS];
};

// Device-resident result block of one plan (read back only when the caller asks for it).
struct PlanState {
    uint64_t n_pending;                   // slices considered by the plan
    uint64_t n_bound;                     // slices bound by the plan
    uint64_t T[TENT_MAX_RAILS];           // bytes bound per rail
    uint64_t cnt[TENT_MAX_RAILS];         // slices bound per rail
    uint64_t A_after[TENT_MAX_RAILS];     // queued bytes after the plan
    uint64_t base[TENT_MAX_RAILS];        // staging region base of each rail (bytes into the arena)
    uint64_t n_runs;                      // runs of equal-length slices seen by the plan
    uint64_t n_done;                      // tent_sim_advance: slices that stayed bound
    uint64_t n_remaining;                 // tent_poll: slices not DONE
    uint64_t peak[TENT_MAX_RAILS];        // bandwidth probe: 1 + best sample of the window, 0 = no sample
    uint32_t probe[TENT_MAX_RAILS];       // B_probe per rail (0 = no sample)
    uint32_t bw_next[TENT_MAX_RAILS];     // smoothed estimate after the window
    uint64_t n_retry;                     // retried slices considered by the plan (bound by rotation)
    uint64_t Tr[TENT_MAX_RAILS];          // bytes the rotation pass bound per rail
    uint64_t cr[TENT_MAX_RAILS];          // slices the rotation pass bound per rail
    uint64_t fail_cnt[TENT_MAX_RAILS];    // tent_sim_fail: slices that failed per rail
    uint64_t n_mice, n_elephant, n_deferred;   // tent_plan_dispatch: requests per mode
    uint64_t rr_next;                     // round-robin counter after the call
    uint64_t bounded_overflow;            // tent_execute_bounded: chunks whose regions do not fit the arena
    uint64_t n_act;                       // tent_execute with few BOUND slices: entries of the list of tiles that move
    uint64_t compact_overflow;            // nonzero: more tiles move than the launch was sized for (nothing is marked DONE)
};

// What the binding chain needs to know about a run of equal-length slices: 32 bytes, read as two 16-byte halves.
struct RunRec {
    uint32_t len;                  // slice length of the run
    uint32_t m;                    // slices in the run
    uint64_t level;                // estimated cost level at the end of the run, ~0 = no estimate
    double   level_f;              // the same as a double
    double   inv_len;              // 1.0 / len
};

// What a copy workgroup needs to know about its slice, in one 16-byte scalar load.
struct SliceRec {
    uint64_t lin;                  // staging address of the slice's first byte
    uint32_t len;                  // bytes to move; 0 when the slice is not BOUND
    uint32_t pad;
};

// Device view of one batch: descriptor tables, prefix sums and the slice table (SoA).
struct BatchDev {
    uint32_t n_desc;
    uint64_t n_src_ext, n_dst_ext;
    uint64_t n_slices;
    uint64_t slice_bytes;

    const uint32_t*    src_ptr;    // [n_desc+1]
    const uint32_t*    dst_ptr;    // [n_desc+1]
    const tent_extent* src_ext;    // [n_src_ext]
    const tent_extent* dst_ext;    // [n_dst_ext]
    uint64_t* src_pre;             // [n_src_ext+1] exclusive prefix of extent lengths over the whole batch
    uint64_t* dst_pre;             // [n_dst_ext+1]
    uint64_t* first;               // [n_desc+1] first slice index of each descriptor

    uint32_t* s_desc;              // [n_slices]
    uint64_t* s_off;
    uint32_t* s_len;
    uint32_t* s_src_e0;            // extent holding the slice's first source byte
    uint32_t* s_dst_e0;
    uint32_t* s_rail;
    uint64_t* s_stage_off;
    uint8_t*  s_state;
    uint64_t* s_tau;               // recorded end-to-end latency in ns (rail simulator / telemetry)
    uint8_t*  s_retry;             // times the slice failed on a rail (saturates at 255)
    uint8_t*  priority;            // [n_desc] request priority of the last tent_plan_dispatch (0 LOW, 1 MID, 2 HIGH)
    uint8_t*  req_mode;            // [n_desc] what the last tent_plan_dispatch did with the request

    struct SliceRec* s_rec;        // packed copy record per slice, rebuilt by every tent_execute
    const BatchDev* self;          // device copy of this structure (generic copy path)

    // Tile tables: for every slice, tiles_per_slice entries per side; entry t holds the device
    // address of byte t*tile_bytes of the slice on the paged side.  Bit 63 marks a tile that
    // needs the generic path (it crosses an extent boundary).
    uint64_t* src_tile;            // [n_slices * tiles_per_slice]
    uint64_t* dst_tile;
    uint32_t  tile_bytes;          // 1 KiB, 2 KiB or 4 KiB
    uint32_t  tiles_per_slice;

    // Table-driven copies (only when every boundary falls on a tile boundary; n_sc_tiles = 0
    // otherwise and the per-slice tile tables above are used instead).  Two enumerations of the
    // payload in tiles: source bytes in declaration order (gather: each rail region is written front
    // to back) and destination bytes in ascending device address (scatter: sequential writes).
    const uint32_t* dst_order;     // [n_dst_ext] destination extents sorted by device address
    const uint32_t* dst_rank;      // [n_dst_ext] the inverse: position of every destination extent in that order
    uint64_t* ord_pre;             // [n_dst_ext+1] exclusive prefix of their lengths in that order
    uint64_t  n_sc_tiles;          // payload / tile_bytes
    uint64_t* ga_src;              // [n_sc_tiles] gather: source address of the tile
    uint64_t* ga_lin;              // [n_sc_tiles] gather: staging address, 0 = not to be moved
    uint32_t* ga_slice;            // [n_sc_tiles] slice that holds the tile
    uint32_t* ga_x;                // [n_sc_tiles] byte offset of the tile inside that slice
    uint64_t* ga_dst;              // [n_sc_tiles] destination address of the tile in declaration order (bounded staging only)
    uint64_t* ch_lo;               // [kMaxChunks * TENT_MAX_RAILS] bounded staging (any geometry): first staging offset per chunk and rail
    uint64_t* ch_hi;               // same shape: end of the interval
    uint64_t* ch_base;             // same shape: region base inside the arena
    uint64_t* tile_scan;           // [n_slices+1] scan workspace of the per-execute tile list: tiles of the BOUND slices before slice i
    uint64_t* tile_partials;       // its per-block partial sums
    uint64_t* act_src;             // [act_capacity] per listed tile (BOUND slices in ascending index, tiles in order): source address,
    uint64_t* act_lin;             //                staging address,
    uint64_t* act_dst;             //                destination address
    uint64_t  act_capacity;
    uint64_t* sc_dst;              // [n_sc_tiles] scatter: destination address of the tile
    uint64_t* sc_lin;              // [n_sc_tiles] scatter: staging address, 0 = not to be moved
    uint32_t* sc_slice;
    uint32_t* sc_x;

    // Run-parallel binding: maximal runs of equal-length pending slices (at most two per transfer)
    uint32_t* run_start;           // [run_capacity + 1] first pending position of every run
    uint64_t* run_T;               // [run_capacity * run_stride] bytes bound per rail before the run
    uint32_t* run_K;               // [run_capacity * run_stride] slots each rail takes in the run
    uint32_t  run_capacity;        // 2 * n_desc
    uint32_t  run_stride;          // entries per row: the context's rail limit rounded up to 16, 32 or 64
    RunRec*   run_rec;             // [run_capacity + 1] one record per run (the last one is a spare the chain's look-ahead may read)
    uint64_t* len_pre;             // [n_slices + 1] bytes of the pending slices before every pending position

    uint32_t* pending;             // [n_slices] ascending ids of slices not DONE and never failed (re-planning)
    uint32_t* retry_ids;           // [n_slices] ascending ids of slices not DONE with a retry count > 0
    uint64_t* rot_bytes;           // [ceil(n_slices / kRotChunk) * TENT_MAX_RAILS] rotation pass: bytes per chunk and rail
    uint32_t* rot_cnt;             // same shape: slices per chunk and rail
    uint64_t* scan_tmp;            // [max(n_ext, n_slices, n_desc)+1] scan workspace
    uint64_t* scan_partials;       // per-block partial sums of the scans
    uint64_t* scan_partials2;      // the same for the second of two scans that share their launches
    PlanState* plan;               // one result block
    const uint64_t* seg_base;      // context-wide table of segment base addresses
};

enum : uint32_t { kScanBlock = 256, kScanItems = 8, kScanTile = kScanBlock * kScanItems };
enum : uint32_t { kCopyBlockBytes = 4096 };          // bytes one copy workgroup moves (256 lanes x 16 B)
enum : uint32_t { kOrderedLanes = 256 };             // lanes of a table-driven copy workgroup (4 KiB each): 128 and 256
                                                     // measure the same on MI355X, 64 / 512 / 1024 are slower
constexpr uint64_t kTileSlow = 1ull << 63;
enum : uint32_t { kMaxChunks = 4096 };               // most chunks one bounded execute may use
enum : uint32_t { kRotChunk = 1024 };                // retried slices one rotation workgroup handles
// `mode` argument of the bind kernels
enum : int { kBindUsePending = 1, kBindAfterRotation = 2, kBindBuildTables = 4 };

// ---- launch wrappers (each enqueues on `s` and returns the launch status) -------------------
hipError_t launch_extent_scans(const BatchDev& b, hipStream_t s);
hipError_t launch_extent_scan(const tent_extent* ext, uint64_t n_ext, uint64_t* pre, uint64_t* partials,
                              hipStream_t s);
hipError_t launch_slice_scan(const BatchDev& b, hipStream_t s);
hipError_t launch_expand(const BatchDev& b, hipStream_t s);
hipError_t launch_compact(const BatchDev& b, hipStream_t s);
hipError_t launch_bind_serial(const BatchDev& b, const RailParams& rp, int mode, hipStream_t s);
hipError_t launch_bind_runs(const BatchDev& b, const RailParams& rp, int mode, hipStream_t s);
hipError_t launch_rotate(const BatchDev& b, const RotateParams& rot, hipStream_t s);
hipError_t launch_fail(const BatchDev& b, const FailParams& fp, hipStream_t s);
hipError_t launch_bounded_prepare(const BatchDev& b, uint64_t payload, uint64_t chunk_bytes, uint32_t n_chunks,
                                  uint64_t slot_bytes, uint32_t slots, uint8_t* arena, hipStream_t s);
hipError_t launch_bounded_copy(const BatchDev& b, bool gather, uint32_t chunk, uint64_t payload, uint64_t chunk_bytes,
                               uint64_t slot_bytes, uint32_t slots, uint8_t* arena, hipStream_t s);
hipError_t launch_mark_done_bounded(const BatchDev& b, hipStream_t s);
hipError_t launch_dispatch(const BatchDev& b, const RailParams& rp, const DispatchParams& dp, bool build_tables,
                           hipStream_t s);
hipError_t launch_tile_tables(const BatchDev& b, hipStream_t s);
hipError_t launch_tile_tables_prepare(const BatchDev& b, hipStream_t s);   // what the builders need when they run inside the chain launch
hipError_t launch_finalize(const BatchDev& b, uint8_t* arena, bool compact, uint64_t max_tiles, hipStream_t s);
hipError_t launch_copy(const BatchDev& b, bool gather, hipStream_t s);
hipError_t launch_copy_ordered(const BatchDev& b, bool gather, hipStream_t s);
hipError_t launch_copy_compact(const BatchDev& b, bool gather, uint64_t max_tiles, hipStream_t s);
hipError_t launch_mark_done(const BatchDev& b, bool compact, hipStream_t s);
hipError_t launch_retire(const BatchDev& b, const BudgetParams& bp, hipStream_t s);
hipError_t launch_count_remaining(const BatchDev& b, hipStream_t s);
hipError_t launch_reset(const BatchDev& b, hipStream_t s);
hipError_t launch_sim_latency(const BatchDev& b, const LatencyParams& lp, hipStream_t s);
hipError_t launch_probe(const BatchDev& b, const ProbeParams& pp, hipStream_t s);

uint64_t scan_partials_capacity(uint64_t n);

hipError_t order_workspace_bytes(uint64_t n_dst, uint64_t n_src, bool check, uint64_t* bytes_out);
hipError_t device_order_destinations(const tent_extent* dst_ext, uint64_t n_dst, const tent_extent* src_ext,
                                     uint64_t n_src, const uint64_t* seg_base, bool check, uint32_t* order_out,
                                     uint32_t* rank_out, uint32_t* overlap_dev, void* workspace, hipStream_t s);

}  // namespace tent
