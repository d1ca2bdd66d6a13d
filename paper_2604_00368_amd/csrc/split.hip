// Slice splitter: prefix sums over extent lengths, per-transfer slice counts and their
// exclusive scan, slice-table expansion, and the pending-list compaction used when a
// batch is re-planned.  Follows the paper's slice decomposition (Section 4.2): a
// transfer of len bytes becomes ceil(len / S) slices; slice k covers [k*S, min((k+1)*S, len))
// and keeps that absolute offset so it can be written straight to its destination.
#include "scan.h"
#include "tile_tables.h"

namespace tent {

uint64_t scan_partials_capacity(uint64_t n) { return (n + kScanTile - 1) / kScanTile + 2; }

// ---- S1: exclusive prefix of extent lengths over the whole batch -----------------------------
struct ExtentLen {
    const tent_extent* ext;
    __device__ uint64_t operator()(uint64_t e) const { return ext[e].len; }
};

hipError_t launch_extent_scan(const tent_extent* ext, uint64_t n_ext, uint64_t* pre, uint64_t* partials,
                              hipStream_t s)
{
    return exclusive_scan(ExtentLen{ext}, n_ext, pre, partials, s);
}

// both sides' prefixes in the same three launches
hipError_t launch_extent_scans(const BatchDev& b, hipStream_t s)
{
    return exclusive_scan2(ExtentLen{b.src_ext}, ExtentLen{b.dst_ext}, b.n_src_ext, b.n_dst_ext, b.src_pre, b.dst_pre,
                           b.scan_partials, b.scan_partials2, s);
}

// ---- S2: slices per transfer, exclusive scan -> first slice index of every transfer ---------
struct SliceCount {
    const uint32_t* ptr;
    const uint64_t* pre;
    uint64_t S;
    __device__ uint64_t operator()(uint64_t j) const
    {
        uint64_t len = pre[ptr[j + 1]] - pre[ptr[j]];
        return (len + S - 1) / S;
    }
};

hipError_t launch_slice_scan(const BatchDev& b, hipStream_t s)
{
    return exclusive_scan(SliceCount{b.src_ptr, b.src_pre, b.slice_bytes}, b.n_desc, b.first, b.scan_partials, s);
}

// ---- S3: slice table expansion ---------------------------------------------------------------
__global__ void __launch_bounds__(256) expand_kernel(BatchDev b)
{
    const uint64_t n = b.first[b.n_desc];
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        // owning transfer: transfers without slices cannot occur (every transfer has len > 0)
        const uint32_t j = (uint32_t)last_not_above(b.first, 0, b.n_desc, i);
        const uint32_t slo = b.src_ptr[j], shi = b.src_ptr[j + 1];
        const uint32_t dlo = b.dst_ptr[j], dhi = b.dst_ptr[j + 1];
        const uint64_t len_j = b.src_pre[shi] - b.src_pre[slo];
        const uint64_t off = (i - b.first[j]) * b.slice_bytes;
        const uint64_t rest = len_j - off;
        b.s_desc[i] = j;
        b.s_off[i] = off;
        b.s_len[i] = (uint32_t)(rest < b.slice_bytes ? rest : b.slice_bytes);
        b.s_src_e0[i] = (uint32_t)last_not_above(b.src_pre, slo, shi, b.src_pre[slo] + off);
        b.s_dst_e0[i] = (uint32_t)last_not_above(b.dst_pre, dlo, dhi, b.dst_pre[dlo] + off);
        b.s_rail[i] = 0xFFFFFFFFu;
        b.s_stage_off[i] = 0;
        b.s_state[i] = TENT_SLICE_PENDING;
    }
}

hipError_t launch_expand(const BatchDev& b, hipStream_t s)
{
    uint64_t blocks = (b.n_slices + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(expand_kernel, dim3((uint32_t)blocks), dim3(256), 0, s, b);
    return hipGetLastError();
}

// ---- S3b: tile tables ------------------------------------------------------------------------
// The builders are in tile_tables.h.  The destination-ordered table needs the exclusive prefix of
// the destination extent lengths in ascending address order first.
struct OrderedLen {
    const tent_extent* ext;
    const uint32_t* order;
    __device__ uint64_t operator()(uint64_t r) const { return ext[order[r]].len; }
};

__global__ void __launch_bounds__(256) tile_tables_kernel(BatchDev b) { build_tile_tables(b, blockIdx.x, gridDim.x); }

hipError_t launch_tile_tables_prepare(const BatchDev& b, hipStream_t s)
{
    if (b.n_sc_tiles == 0) return hipSuccess;
    return exclusive_scan(OrderedLen{b.dst_ext, b.dst_order}, b.n_dst_ext, b.ord_pre, b.scan_partials, s);
}

hipError_t launch_tile_tables(const BatchDev& b, hipStream_t s)
{
    hipError_t e = launch_tile_tables_prepare(b, s);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(tile_tables_kernel, dim3(tile_table_blocks(b)), dim3(256), 0, s, b);
    return hipGetLastError();
}

// Copy records: staging address (arena + region base of the rail + offset inside the region) and
// length of every BOUND slice; slices in any other state get length 0 and are skipped by the copy.
__global__ void __launch_bounds__(256) finalize_kernel(BatchDev b, uint8_t* arena)
{
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < b.n_slices; i += stride) {
        SliceRec r{0, 0, 0};
        if (b.s_state[i] == TENT_SLICE_BOUND) {
            r.lin = (uint64_t)arena + b.plan->base[b.s_rail[i]] + b.s_stage_off[i];
            r.len = b.s_len[i];
        }
        b.s_rec[i] = r;
    }
}

// Staging address of every source-ordered and destination-ordered tile whose slice is about to
// move (0 otherwise).
__global__ void __launch_bounds__(256) finalize_tiles_kernel(BatchDev b)
{
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t q = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; q < b.n_sc_tiles; q += stride) {
        const SliceRec g = b.s_rec[b.ga_slice[q]];
        b.ga_lin[q] = g.len ? g.lin + b.ga_x[q] : 0;
        const SliceRec r = b.s_rec[b.sc_slice[q]];
        b.sc_lin[q] = r.len ? r.lin + b.sc_x[q] : 0;
    }
}

// When only a small part of the batch moves (re-planning epochs), the copy launches should not pay for
// every tile of the batch.  The tiles of the BOUND slices are listed instead: a scan over the slices
// gives each BOUND slice the position of its first tile in the list, and one wavefront per BOUND slice
// resolves the three addresses of each of its tiles (source, staging, destination) from the slice
// table and the extent lists.  The work is proportional to what moves, not to the batch.
struct BoundTiles {
    const SliceRec* rec;
    uint32_t tile_shift;
    __device__ uint64_t operator()(uint64_t i) const { return rec[i].len >> tile_shift; }   // 0 unless BOUND
};

__global__ void __launch_bounds__(256) tile_list_kernel(BatchDev b, uint32_t tile_shift, uint64_t max_tiles)
{
    const uint64_t i = (uint64_t)blockIdx.x * 4 + (threadIdx.x >> 6);      // one wavefront per slice
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        const uint64_t n_act = b.tile_scan[b.n_slices];
        b.plan->n_act = n_act < b.act_capacity ? n_act : b.act_capacity;
        // the copy launches are sized by the host's bound on the BOUND slices; should more tiles move than
        // that (or than the list holds), the copies would be incomplete, so nothing may be marked DONE
        b.plan->compact_overflow = (n_act > max_tiles || n_act > b.act_capacity) ? 1 : 0;
    }
    if (i >= b.n_slices) return;
    const SliceRec r = b.s_rec[i];
    const uint32_t n_t = r.len >> tile_shift;
    if (n_t == 0) return;
    const uint64_t at = b.tile_scan[i];
    const uint32_t j = b.s_desc[i];
    const uint64_t off = b.s_off[i];
    const uint32_t s_hi = b.src_ptr[j + 1], d_hi = b.dst_ptr[j + 1];
    const uint64_t s_pos0 = b.src_pre[b.src_ptr[j]] + off, d_pos0 = b.dst_pre[b.dst_ptr[j]] + off;
    const uint32_t s_e0 = b.s_src_e0[i], d_e0 = b.s_dst_e0[i];
    for (uint32_t t = threadIdx.x & 63; t < n_t; t += 64) {
        const uint64_t p = at + t;
        if (p >= b.act_capacity) break;
        const uint64_t x = (uint64_t)t << tile_shift;
        const uint64_t se = last_not_above(b.src_pre, s_e0, s_hi, s_pos0 + x);
        const tent_extent sx = b.src_ext[se];
        const uint64_t de = last_not_above(b.dst_pre, d_e0, d_hi, d_pos0 + x);
        const tent_extent dx = b.dst_ext[de];
        b.act_src[p] = b.seg_base[sx.seg] + sx.off + (s_pos0 + x - b.src_pre[se]);
        b.act_lin[p] = r.lin + x;
        b.act_dst[p] = b.seg_base[dx.seg] + dx.off + (d_pos0 + x - b.dst_pre[de]);
    }
}

hipError_t launch_finalize(const BatchDev& b, uint8_t* arena, bool compact, uint64_t max_tiles, hipStream_t s)
{
    uint64_t blocks = (b.n_slices + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(finalize_kernel, dim3((uint32_t)blocks), dim3(256), 0, s, b, arena);
    if (b.n_sc_tiles && compact) {
        uint32_t tile_shift = 0;
        while ((1u << tile_shift) < b.tile_bytes) ++tile_shift;
        hipError_t e = exclusive_scan(BoundTiles{b.s_rec, tile_shift}, b.n_slices, b.tile_scan, b.tile_partials, s);
        if (e != hipSuccess) return e;
        const uint64_t lists = (b.n_slices + 3) / 4;
        if (lists > 0x7FFFFFFFull) return hipErrorInvalidValue;
        hipLaunchKernelGGL(tile_list_kernel, dim3((uint32_t)lists), dim3(256), 0, s, b, tile_shift, max_tiles);
    } else if (b.n_sc_tiles) {
        blocks = (b.n_sc_tiles + 255) / 256;
        if (blocks > 65536) blocks = 65536;
        hipLaunchKernelGGL(finalize_tiles_kernel, dim3((uint32_t)blocks), dim3(256), 0, s, b);
    }
    return hipGetLastError();
}

// ---- E1: ascending lists of slices that are not DONE ------------------------------------------
// Two lists from one scan: slices that never failed (bound by predicted cost) are counted in the
// low half of the scanned word, slices with a retry count (bound by rotation) in the high half.
struct NotDoneSplit {
    const uint8_t* state;
    const uint8_t* retry;
    __device__ uint64_t operator()(uint64_t i) const
    {
        if (state[i] == TENT_SLICE_DONE) return 0;
        return retry[i] ? (1ull << 32) : 1ull;
    }
};

__global__ void __launch_bounds__(256) compact_kernel(BatchDev b)
{
    const uint64_t n = b.n_slices;
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        if (b.s_state[i] == TENT_SLICE_DONE) continue;
        const uint64_t at = b.scan_tmp[i];
        if (b.s_retry[i]) b.retry_ids[at >> 32] = (uint32_t)i;
        else              b.pending[at & 0xFFFFFFFFu] = (uint32_t)i;
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        b.plan->n_pending = b.scan_tmp[n] & 0xFFFFFFFFu;
        b.plan->n_retry = b.scan_tmp[n] >> 32;
    }
}

hipError_t launch_compact(const BatchDev& b, hipStream_t s)
{
    hipError_t e = exclusive_scan(NotDoneSplit{b.s_state, b.s_retry}, b.n_slices, b.scan_tmp, b.scan_partials, s);
    if (e != hipSuccess) return e;
    uint64_t blocks = (b.n_slices + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(compact_kernel, dim3((uint32_t)blocks), dim3(256), 0, s, b);
    return hipGetLastError();
}

// ---- slice state bookkeeping ------------------------------------------------------------------
__global__ void __launch_bounds__(256) mark_done_kernel(BatchDev b, int compact)
{
    if (compact && b.plan->compact_overflow != 0) return;       // incomplete copies: the slices stay BOUND
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < b.n_slices; i += stride)
        if (b.s_state[i] == TENT_SLICE_BOUND) b.s_state[i] = TENT_SLICE_DONE;
}

hipError_t launch_mark_done(const BatchDev& b, bool compact, hipStream_t s)
{
    uint64_t blocks = (b.n_slices + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(mark_done_kernel, dim3((uint32_t)blocks), dim3(256), 0, s, b, compact ? 1 : 0);
    return hipGetLastError();
}

__global__ void __launch_bounds__(256) reset_kernel(BatchDev b)
{
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < b.n_slices; i += stride) {
        b.s_state[i] = TENT_SLICE_PENDING;
        b.s_retry[i] = 0;
    }
}

hipError_t launch_reset(const BatchDev& b, hipStream_t s)
{
    uint64_t blocks = (b.n_slices + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(reset_kernel, dim3((uint32_t)blocks), dim3(256), 0, s, b);
    return hipGetLastError();
}

// Rail simulator: a bound slice completes iff the rail's byte budget covers the bytes queued
// ahead of the plan, the slices staged before it, and the slice itself; otherwise it returns to
// the pending set.  The count of completed slices is an integer sum, so its value does not
// depend on the order of the atomic adds.
__global__ void __launch_bounds__(256) retire_kernel(BatchDev b, BudgetParams bp)
{
    __shared__ unsigned long long block_done;
    if (threadIdx.x == 0) block_done = 0;
    __syncthreads();
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    unsigned long long mine = 0;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < b.n_slices; i += stride) {
        if (b.s_state[i] != TENT_SLICE_BOUND) continue;
        const uint32_t d = b.s_rail[i];
        const uint64_t last = bp.queued[d] + b.s_stage_off[i] + b.s_len[i];
        const bool fits = last >= bp.queued[d] && last <= bp.budget[d];
        if (fits) ++mine; else b.s_state[i] = TENT_SLICE_PENDING;
    }
    if (mine) atomicAdd(&block_done, mine);
    __syncthreads();
    if (threadIdx.x == 0 && block_done) atomicAdd((unsigned long long*)&b.plan->n_done, block_done);
}

__global__ void zero_counter_kernel(uint64_t* p) { *p = 0; }

hipError_t launch_retire(const BatchDev& b, const BudgetParams& bp, hipStream_t s)
{
    hipLaunchKernelGGL(zero_counter_kernel, dim3(1), dim3(1), 0, s, &b.plan->n_done);
    uint64_t blocks = (b.n_slices + 255) / 256;
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(retire_kernel, dim3((uint32_t)blocks), dim3(256), 0, s, b, bp);
    return hipGetLastError();
}

__global__ void __launch_bounds__(256) count_remaining_kernel(BatchDev b)
{
    __shared__ unsigned long long block_cnt;
    if (threadIdx.x == 0) block_cnt = 0;
    __syncthreads();
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    unsigned long long mine = 0;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < b.n_slices; i += stride)
        mine += b.s_state[i] != TENT_SLICE_DONE;
    if (mine) atomicAdd(&block_cnt, mine);
    __syncthreads();
    if (threadIdx.x == 0 && block_cnt) atomicAdd((unsigned long long*)&b.plan->n_remaining, block_cnt);
}

hipError_t launch_count_remaining(const BatchDev& b, hipStream_t s)
{
    hipLaunchKernelGGL(zero_counter_kernel, dim3(1), dim3(1), 0, s, &b.plan->n_remaining);
    uint64_t blocks = (b.n_slices + 255) / 256;
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(count_remaining_kernel, dim3((uint32_t)blocks), dim3(256), 0, s, b);
    return hipGetLastError();
}

}  // namespace tent
