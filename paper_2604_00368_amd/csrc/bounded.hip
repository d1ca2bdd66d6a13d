// Bounded, pipelined staging (Section 4.1 of the paper: the payload is partitioned into chunks that
// pass through an intermediate buffer of fixed size).  The payload -- the transfers' bytes laid end to
// end in declaration order -- is cut into chunks of chunk_bytes; chunks pass through the staging
// arena one after the other (gather of the chunk, then scatter of the chunk).  Inside the arena every
// rail keeps one contiguous region per chunk (chunk c lives in slot c mod slots of the arena, so that
// with two slots a chunk can be gathered while its predecessor is still being scattered): the chunk's bytes on rail d form an interval
// [lo_d, hi_d) of the rail's staging offsets, they sit at region_base_d + (offset - lo_d), and the
// region bases are the exclusive sum of the interval lengths rounded up to 256 bytes.
//
// Both copies walk the chunk's tiles in declaration order (a chunk is a contiguous range of that
// enumeration), so a chunk's launch touches only its own table entries.
//
// Geometry whose lengths are no multiple of the tile size has no such enumeration.  There the same
// steps run over the payload in ranges of 1 KiB, one wavefront per range: the wavefront finds the
// slice that holds the range's first byte (transfers are laid end to end, so a payload position
// gives the transfer by a search over their first positions and the slice by a division), walks
// the slices that intersect the range and moves each piece byte-exactly through the extent lists.
#include "copy_generic.h"

namespace tent {
namespace {

constexpr uint64_t kNoTile = ~0ull;
constexpr uint64_t kRegMask = (1ull << 56) - 1;

__global__ void __launch_bounds__(256) bounded_clear_kernel(BatchDev b, uint32_t n_chunks)
{
    const uint32_t at = blockIdx.x * blockDim.x + threadIdx.x;
    if (at < n_chunks * TENT_MAX_RAILS) {
        b.ch_lo[at] = kNoTile;
        b.ch_hi[at] = 0;
    }
    if (at == 0) b.plan->bounded_overflow = 0;
}

// Per tile (declaration order): rail and staging offset of its first byte, or kNoTile when its slice is
// not BOUND; per (chunk, rail): the interval of staging offsets the chunk touches.  A workgroup covers
// 256 consecutive tiles, which lie in one chunk because a chunk holds a multiple of 256 tiles.
__global__ void __launch_bounds__(256) bounded_tiles_kernel(BatchDev b, uint64_t chunk_tiles)
{
    __shared__ unsigned long long lo[TENT_MAX_RAILS], hi[TENT_MAX_RAILS];
    if (threadIdx.x < TENT_MAX_RAILS) { lo[threadIdx.x] = kNoTile; hi[threadIdx.x] = 0; }
    __syncthreads();
    const uint64_t first = ((uint64_t)blockIdx.y * gridDim.x + blockIdx.x) * 256;
    const uint64_t q = first + threadIdx.x;
    if (q < b.n_sc_tiles) {
        const uint32_t i = b.ga_slice[q];
        uint64_t code = kNoTile;
        if (b.s_state[i] == TENT_SLICE_BOUND) {
            const uint32_t d = b.s_rail[i];
            const uint64_t reg = b.s_stage_off[i] + b.ga_x[q];
            code = ((uint64_t)d << 56) | reg;
            atomicMin(&lo[d], (unsigned long long)reg);
            atomicMax(&hi[d], (unsigned long long)(reg + b.tile_bytes));
        }
        b.ga_lin[q] = code;
    }
    __syncthreads();
    if (first < b.n_sc_tiles && threadIdx.x < TENT_MAX_RAILS && lo[threadIdx.x] != kNoTile) {
        const uint64_t c = first / chunk_tiles;
        atomicMin((unsigned long long*)&b.ch_lo[c * TENT_MAX_RAILS + threadIdx.x], lo[threadIdx.x]);
        atomicMax((unsigned long long*)&b.ch_hi[c * TENT_MAX_RAILS + threadIdx.x], hi[threadIdx.x]);
    }
}

// One wavefront per chunk: region bases of the rails inside the arena for that chunk.
__global__ void __launch_bounds__(64) bounded_bases_kernel(BatchDev b, uint64_t slot_bytes)
{
    const uint64_t row = (uint64_t)blockIdx.x * TENT_MAX_RAILS + threadIdx.x;
    const uint64_t lo = b.ch_lo[row], hi = b.ch_hi[row];
    const uint64_t need = (lo != kNoTile && hi > lo) ? ((hi - lo + 255) & ~255ull) : 0;
    uint64_t inc = need;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint64_t up = (uint64_t)__shfl_up((unsigned long long)inc, d, 64);
        if ((int)threadIdx.x >= d) inc += up;
    }
    b.ch_base[row] = inc - need;
    if (threadIdx.x == 63 && inc > slot_bytes) atomicAdd((unsigned long long*)&b.plan->bounded_overflow, 1ull);
}

// Turn every tile's (rail, staging offset) into its address inside the slot of its chunk (0 = tile not
// to be moved), so that the copy kernels need no dependent look-ups.
__global__ void __launch_bounds__(256) bounded_resolve_kernel(BatchDev b, uint64_t chunk_tiles, uint8_t* arena,
                                                              uint64_t slot_bytes, uint32_t slots)
{
    const uint64_t q = ((uint64_t)blockIdx.y * gridDim.x + blockIdx.x) * 256 + threadIdx.x;
    if (q >= b.n_sc_tiles) return;
    const uint64_t c = b.ga_lin[q];
    uint64_t addr = 0;
    if (c != kNoTile) {
        const uint64_t chunk = q / chunk_tiles;
        const uint64_t row = chunk * TENT_MAX_RAILS + (c >> 56);
        addr = (uint64_t)arena + (chunk % slots) * slot_bytes + b.ch_base[row] + ((c & kRegMask) - b.ch_lo[row]);
    }
    b.ga_lin[q] = addr;
}

// Copy the tiles [q_begin, q_end) of one chunk between their paged side and the arena.
template <bool kGather>
__global__ void __launch_bounds__(kOrderedLanes) bounded_copy_kernel(const uint64_t* __restrict__ paged,
                                                           const uint64_t* __restrict__ staged,
                                                           const uint64_t* __restrict__ overflow,
                                                           uint64_t q_begin, uint64_t q_end, uint32_t tile_shift)
{
    const uint64_t w = (uint64_t)blockIdx.y * gridDim.x + blockIdx.x;
    const uint64_t at = w * (kOrderedLanes * 16) + (uint64_t)threadIdx.x * 16;
    const uint64_t q = q_begin + (at >> tile_shift);
    if (q >= q_end) return;
    const uint64_t near_tile = staged[q];
    const uint64_t far_tile = paged[q];
    if (near_tile == 0 || *overflow != 0) return;
    const uint64_t in_tile = at & ((1ull << tile_shift) - 1);
    const uint64_t far = far_tile + in_tile, near = near_tile + in_tile;
    typedef uint32_t vec4u __attribute__((ext_vector_type(4)));
    typedef __attribute__((address_space(1))) vec4u vec4u_any __attribute__((aligned(1)));   // device memory, any alignment
    // the paged side is streamed (nontemporal); the arena side uses ordinary accesses so that a slot
    // small enough for the memory-side cache can be served from it when the chunk is scattered
    if (kGather) {
        const vec4u v = __builtin_nontemporal_load((const vec4u_any*)far);
        *(vec4u_any*)near = v;
    } else {
        const vec4u v = *(const vec4u_any*)near;
        __builtin_nontemporal_store(v, (vec4u_any*)far);
    }
}

// ---- geometry without a tile enumeration: ranges of 1 KiB of the payload -----------------------
constexpr uint32_t kRangeBytes = 1024;

// Payload position of the first byte of transfer j (the source extent prefix runs over the whole batch).
__device__ __forceinline__ uint64_t transfer_start(const BatchDev& b, uint32_t j) { return b.src_pre[b.src_ptr[j]]; }

// Slice that holds payload position p (p < payload).
__device__ __forceinline__ uint64_t slice_at(const BatchDev& b, uint64_t p)
{
    uint32_t lo = 0, hi = b.n_desc;                       // last transfer that starts at or before p
    while (hi - lo > 1) {
        const uint32_t mid = lo + ((hi - lo) >> 1);
        if (transfer_start(b, mid) <= p) lo = mid; else hi = mid;
    }
    return b.first[lo] + (p - transfer_start(b, lo)) / b.slice_bytes;
}

// Per (chunk, rail): the interval of staging offsets that the BOUND bytes of the chunk touch.  A
// workgroup covers four consecutive ranges, which lie in one chunk (chunks are multiples of 1 MiB).
__global__ void __launch_bounds__(256) bounded_ranges_kernel(BatchDev b, uint64_t payload, uint64_t chunk_bytes)
{
    __shared__ unsigned long long lo[TENT_MAX_RAILS], hi[TENT_MAX_RAILS];
    if (threadIdx.x < TENT_MAX_RAILS) { lo[threadIdx.x] = kNoTile; hi[threadIdx.x] = 0; }
    __syncthreads();
    const uint64_t first = ((uint64_t)blockIdx.y * gridDim.x + blockIdx.x) * (4ull * kRangeBytes);
    const uint64_t p0 = first + (uint64_t)(threadIdx.x >> 6) * kRangeBytes;
    if (p0 < payload) {
        const uint64_t p1 = p0 + kRangeBytes < payload ? p0 + kRangeBytes : payload;
        uint64_t i = slice_at(b, p0);
        for (;;) {
            const uint64_t at = transfer_start(b, b.s_desc[i]) + b.s_off[i];      // payload position of the slice
            const uint64_t end = at + b.s_len[i];
            if ((threadIdx.x & 63) == 0 && b.s_state[i] == TENT_SLICE_BOUND) {
                const uint64_t from = at > p0 ? at : p0, to = end < p1 ? end : p1;
                const uint64_t reg = b.s_stage_off[i] + (from - at);
                const uint32_t d = b.s_rail[i];
                atomicMin(&lo[d], (unsigned long long)reg);
                atomicMax(&hi[d], (unsigned long long)(reg + (to - from)));
            }
            if (end >= p1) break;
            ++i;
        }
    }
    __syncthreads();
    if (first < payload && threadIdx.x < TENT_MAX_RAILS && lo[threadIdx.x] != kNoTile) {
        const uint64_t c = first / chunk_bytes;
        atomicMin((unsigned long long*)&b.ch_lo[c * TENT_MAX_RAILS + threadIdx.x], lo[threadIdx.x]);
        atomicMax((unsigned long long*)&b.ch_hi[c * TENT_MAX_RAILS + threadIdx.x], hi[threadIdx.x]);
    }
}

// Move the BOUND bytes of payload positions [c_lo, c_hi) -- one chunk -- between their paged side and the
// chunk's slot, one wavefront per range of 1 KiB.
template <bool kGather>
__global__ void __launch_bounds__(256) bounded_ranges_copy_kernel(BatchDev b, uint64_t c_lo, uint64_t c_hi,
                                                                  uint8_t* slot, uint64_t row)
{
    const uint64_t w = ((uint64_t)blockIdx.y * gridDim.x + blockIdx.x) * 4 + (threadIdx.x >> 6);
    const uint64_t p0 = c_lo + w * kRangeBytes;
    if (p0 >= c_hi || b.plan->bounded_overflow != 0) return;
    const uint64_t p1 = p0 + kRangeBytes < c_hi ? p0 + kRangeBytes : c_hi;
    uint64_t i = slice_at(b, p0);
    for (;;) {
        const uint64_t at = transfer_start(b, b.s_desc[i]) + b.s_off[i];
        const uint64_t end = at + b.s_len[i];
        if (b.s_state[i] == TENT_SLICE_BOUND) {
            const uint64_t from = at > p0 ? at : p0, to = end < p1 ? end : p1;
            const uint64_t x = from - at;                                         // offset inside the slice
            const uint32_t d = b.s_rail[i];
            uint8_t* staged = slot + b.ch_base[row + d] + (b.s_stage_off[i] + x - b.ch_lo[row + d]);
            copy_range_generic<kGather>(b, i, x, x + (to - from), staged);
        }
        if (end >= p1) break;
        ++i;
    }
}

__global__ void __launch_bounds__(256) mark_done_bounded_kernel(BatchDev b)
{
    if (b.plan->bounded_overflow != 0) return;                      // nothing moved: leave the slices BOUND
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < b.n_slices; i += stride)
        if (b.s_state[i] == TENT_SLICE_BOUND) b.s_state[i] = TENT_SLICE_DONE;
}

bool grid_for(uint64_t blocks, dim3* grid)
{
    const uint32_t gx = blocks < 65536 ? (uint32_t)blocks : 65536u;
    const uint64_t gy = (blocks + gx - 1) / gx;
    if (gy > 0x7FFFFFFFull) return false;
    *grid = dim3(gx, (uint32_t)gy);
    return true;
}

}  // namespace

hipError_t launch_bounded_prepare(const BatchDev& b, uint64_t payload, uint64_t chunk_bytes, uint32_t n_chunks,
                                  uint64_t slot_bytes, uint32_t slots, uint8_t* arena, hipStream_t s)
{
    const uint32_t cells = n_chunks * TENT_MAX_RAILS;
    hipLaunchKernelGGL(bounded_clear_kernel, dim3((cells + 255) / 256), dim3(256), 0, s, b, n_chunks);
    dim3 grid;
    if (b.n_sc_tiles == 0) {                                  // no tile enumeration: ranges of the payload
        if (!grid_for((payload + 4 * kRangeBytes - 1) / (4 * kRangeBytes), &grid)) return hipErrorInvalidValue;
        hipLaunchKernelGGL(bounded_ranges_kernel, grid, dim3(256), 0, s, b, payload, chunk_bytes);
        hipLaunchKernelGGL(bounded_bases_kernel, dim3(n_chunks), dim3(64), 0, s, b, slot_bytes);
        return hipGetLastError();
    }
    if (!grid_for((b.n_sc_tiles + 255) / 256, &grid)) return hipErrorInvalidValue;
    hipLaunchKernelGGL(bounded_tiles_kernel, grid, dim3(256), 0, s, b, chunk_bytes / b.tile_bytes);
    hipLaunchKernelGGL(bounded_bases_kernel, dim3(n_chunks), dim3(64), 0, s, b, slot_bytes);
    hipLaunchKernelGGL(bounded_resolve_kernel, grid, dim3(256), 0, s, b, chunk_bytes / b.tile_bytes, arena, slot_bytes,
                       slots);
    return hipGetLastError();
}

hipError_t launch_bounded_copy(const BatchDev& b, bool gather, uint32_t chunk, uint64_t payload, uint64_t chunk_bytes,
                               uint64_t slot_bytes, uint32_t slots, uint8_t* arena, hipStream_t s)
{
    if (b.n_sc_tiles == 0) {
        const uint64_t c_lo = (uint64_t)chunk * chunk_bytes;
        if (c_lo >= payload) return hipSuccess;
        const uint64_t c_hi = c_lo + chunk_bytes < payload ? c_lo + chunk_bytes : payload;
        dim3 grid;
        if (!grid_for((c_hi - c_lo + 4 * kRangeBytes - 1) / (4 * kRangeBytes), &grid)) return hipErrorInvalidValue;
        uint8_t* slot = arena + (chunk % slots) * slot_bytes;
        const uint64_t row = (uint64_t)chunk * TENT_MAX_RAILS;
        if (gather)
            hipLaunchKernelGGL(bounded_ranges_copy_kernel<true>, grid, dim3(256), 0, s, b, c_lo, c_hi, slot, row);
        else
            hipLaunchKernelGGL(bounded_ranges_copy_kernel<false>, grid, dim3(256), 0, s, b, c_lo, c_hi, slot, row);
        return hipGetLastError();
    }
    uint32_t tile_shift = 0;
    while ((1u << tile_shift) < b.tile_bytes) ++tile_shift;
    const uint64_t chunk_tiles = chunk_bytes >> tile_shift;
    const uint64_t q_begin = (uint64_t)chunk * chunk_tiles;
    if (q_begin >= b.n_sc_tiles) return hipSuccess;
    const uint64_t q_end = q_begin + chunk_tiles < b.n_sc_tiles ? q_begin + chunk_tiles : b.n_sc_tiles;
    const uint64_t bytes = (q_end - q_begin) << tile_shift;
    dim3 grid;
    if (!grid_for((bytes + kOrderedLanes * 16 - 1) / (kOrderedLanes * 16), &grid)) return hipErrorInvalidValue;
    if (gather)
        hipLaunchKernelGGL(bounded_copy_kernel<true>, grid, dim3(kOrderedLanes), 0, s, b.ga_src, b.ga_lin,
                           &b.plan->bounded_overflow, q_begin, q_end, tile_shift);
    else
        hipLaunchKernelGGL(bounded_copy_kernel<false>, grid, dim3(kOrderedLanes), 0, s, b.ga_dst, b.ga_lin,
                           &b.plan->bounded_overflow, q_begin, q_end, tile_shift);
    return hipGetLastError();
}

hipError_t launch_mark_done_bounded(const BatchDev& b, hipStream_t s)
{
    uint64_t blocks = (b.n_slices + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(mark_done_bounded_kernel, dim3((uint32_t)blocks), dim3(256), 0, s, b);
    return hipGetLastError();
}

}  // namespace tent
