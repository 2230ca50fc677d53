// Internal declarations shared by the HIP sources of libvbcast (not installed).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace vbcast {

// Algorithm codes as in the public header (VBCAST_NATIVE ... VBCAST_SCATTER_RDB);
// the host code checks that the two agree.
enum : int32_t { kAlgoNative = 0, kAlgoTuned = 1, kAlgoBinomial = 2, kAlgoScatterRdb = 3 };

// One transfer of a step: copy `len` bytes at byte offset `off` from rank
// `src`'s buffer to the same offset in rank `dst`'s buffer.
struct Row {
    uint32_t src;
    uint32_t dst;
    uint64_t off;
    uint64_t len;
};
static_assert(sizeof(Row) == 24, "Row layout");

// One copy tile: the part of row `row` inside the `idx`-th tile-aligned window
// the row touches.
struct Tile {
    uint32_t row;
    uint32_t idx;
};

// Everything the generation kernels read and write, all device pointers.
// Per-step arrays are indexed by step; row and tile arrays have a fixed stride
// per step (`P` rows, `P + 1` tile-scan entries, `tile_cap` tiles).
struct PlanArrays {
    int32_t P, root, algo;
    int32_t L;          // ceil(log2 P)
    int32_t n_scatter;  // scatter steps: L, or 0 for the binomial broadcast
    int32_t n_steps;    // all steps (0 when P == 1)
    int32_t tile_log2;  // copy tile of the per-step executor (tile maps)
    int32_t slab_log2;  // slab of the one-launch executor
    int32_t n_xcd;      // accelerator dies (XCDs) of the device; workgroup b runs on XCD b mod n_xcd
    uint32_t tile_cap;  // tile slots per step
    uint64_t n, ss;

    uint64_t *chunk_off;  // [P + 1]
    uint64_t *chunk_len;  // [P]
    int32_t *rel, *left, *right, *sw_step, *sw_flag;  // [P], by absolute rank

    uint8_t *const *bases;  // [P] rank buffers, by absolute rank

    Row *rows;            // [n_steps][P]
    uint64_t *chain;      // [P][L + P - 1] chunk-major view of the scatter and ring rows
                          // (ring algorithms only): entry s of chunk c = the buffer
                          // that holds the chunk after step s, bit 0 set = the step's
                          // table has no row for this chunk (nothing is copied)
    uint32_t *tile_ptr;   // [n_steps][P + 1] exclusive scan of tiles per row
    Tile *tiles;          // [n_steps][tile_cap]

    uint32_t *step_rows;    // [n_steps]
    uint32_t *step_tiles;   // [n_steps]
    uint32_t *step_posted;  // [n_steps] sends posted, zero-length included
    uint32_t *step_mismatch;  // [n_steps] sender/receiver decisions that disagree
    uint64_t *step_bytes;   // [n_steps]
    uint64_t *census;       // [n_steps][4] inter msgs, inter bytes, intra msgs, intra bytes
};

// Rank buffers are ordinary device allocations.  Pointers that come out of a
// table are generic to the compiler; these types put them back into the global
// address space so that copies compile to global (not flat) memory instructions.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(1))) u32x4 gmem_u32x4;
typedef __attribute__((address_space(1))) uint8_t gmem_u8;

__device__ __forceinline__ const gmem_u32x4 *gmem_words(const uint8_t *p) {
    return (const gmem_u32x4 *)(uintptr_t)p;
}
__device__ __forceinline__ gmem_u32x4 *gmem_words(uint8_t *p) {
    return (gmem_u32x4 *)(uintptr_t)p;
}
__device__ __forceinline__ const gmem_u8 *gmem_bytes(const uint8_t *p) {
    return (const gmem_u8 *)(uintptr_t)p;
}
__device__ __forceinline__ gmem_u8 *gmem_bytes(uint8_t *p) { return (gmem_u8 *)(uintptr_t)p; }

// Enqueue the three generation kernels (descriptors, rows, tile maps); tile maps
// are (re)built for the first `tile_map_steps` steps only.
hipError_t launch_plan_kernels(const PlanArrays &pa, int tile_map_steps, hipStream_t stream);

// Enqueue the census kernel: per step, rows and bytes that cross / stay inside a
// node when ranks sit on nodes in blocks of `ranks_per_node`; fills pa.census.
hipError_t launch_plan_census(const PlanArrays &pa, int ranks_per_node, hipStream_t stream);

// Enqueue the copy kernel of one step; `n_tiles` > 0 workgroups, dealt to the
// device's `n_xcd` accelerator dies so that each takes a contiguous share.
hipError_t launch_step_copy(const Row *rows, const Tile *tiles, uint8_t *const *bases,
                            uint32_t n_tiles, int tile_log2, int n_xcd, hipStream_t stream);

// Most ranks a broadcast may have for the one-launch kernel to work its hops out
// itself: it keeps the rank buffers' addresses and the hops of the chunks it is
// busy with in LDS, 8 bytes per rank and per step (ceil(log2 P) + P - 1 steps).
constexpr int kInlineMaxRanks = 1024;
constexpr int kInlineMaxHops = 1040;   // >= 10 + 1023

// The slab size (log2 of bytes, 10..16) launch_ring_chain walks the message in, given
// pa.n, pa.ss and pa.slab_log2, and through *workgroups (may be null) how many
// workgroups share the slabs at that size when `wgs_at_plan_tile` would at the plan's.
// A result above log2(pa.ss) means: chunks shorter than 1 KiB, one wavefront per chunk.
int chain_slab_log2(const PlanArrays &pa, uint32_t wgs_at_plan_tile, uint64_t *workgroups);

// Enqueue steps [first_step, last_step) of a scatter + ring broadcast (native or
// tuned) as one launch that walks every slab of the message through those steps
// (all of them: 0 and pa.n_steps).  `wgs_at_plan_tile` persistent workgroups
// would share the slabs at the plan's slab size; the launch may pick a smaller
// slab (and proportionally more workgroups) or one wavefront per chunk for short
// chunks.  With `from_tables` the kernel looks the hops up in pa.chain and
// pa.chunk_off, which launch_plan_kernels must have filled on this stream before;
// without, it derives them itself from pa.P, pa.root, pa.algo, pa.n and reads
// only pa.bases (pa.P <= kInlineMaxRanks, else hipErrorInvalidValue).
hipError_t launch_ring_chain(const PlanArrays &pa, uint32_t wgs_at_plan_tile, int first_step,
                             int last_step, bool from_tables, hipStream_t stream);

}  // namespace vbcast
