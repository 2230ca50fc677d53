// Step execution: one launch moves every row of one step.
//
// A row copies `len` bytes at offset `off` from one rank buffer to the same
// offset in another [Sec. IV, listing: the send and the matching receive use
// the same displacement].  Rank buffers are 16-byte aligned, so source and
// destination of a row are always equally aligned and the copy can use 16-byte
// accesses throughout, with at most 15 single bytes at either end of a row.
//
// Rows are cut at multiples of the tile size measured from the start of the
// buffer, so every tile except a row's first and last is a whole, aligned
// window; one workgroup of 256 lanes copies one tile.  Consecutive lanes touch
// consecutive 16-byte words (one wavefront = 1 KiB contiguous per access), and
// a lane issues all its loads before its first store.  Loads are non-temporal:
// within a launch nothing is read twice, and keeping the read stream from
// claiming L2 lines made the launch 9-11 % faster; non-temporal stores made it
// slower and are not used.

#include "vbcast_internal.h"

namespace vbcast {

namespace {

constexpr int kThreads = 256;

template <int TILE_LOG2>
__global__ __launch_bounds__(kThreads) void step_copy(const Row *__restrict__ rows,
                                                      const Tile *__restrict__ tiles,
                                                      uint8_t *const *__restrict__ bases,
                                                      uint32_t n_tiles, uint32_t n_xcd) {
    constexpr uint64_t TILE = 1ull << TILE_LOG2;
    constexpr int WORDS = (int)(TILE / 16);      // 16-byte words in a full tile
    constexpr int PER_LANE = WORDS / kThreads;   // words per lane in a full tile
    static_assert(PER_LANE >= 1, "tile too small for the workgroup");

    // Workgroups go to the XCDs round-robin (workgroup id mod the number of
    // XCDs): give each XCD a contiguous share of the step's tiles rather than
    // every n-th tile, so that its addresses spread over all of its L2 channels.
    const uint32_t per_xcd = gridDim.x / n_xcd;  // the grid is a multiple of n_xcd
    const uint32_t tile_id = (blockIdx.x % n_xcd) * per_xcd + (blockIdx.x / n_xcd);
    if (tile_id >= n_tiles) return;
    const Tile t = tiles[tile_id];
    const Row r = rows[t.row];
    const uint8_t *__restrict__ src = bases[r.src];
    uint8_t *__restrict__ dst = bases[r.dst];

    const uint64_t window = ((r.off >> TILE_LOG2) + t.idx) << TILE_LOG2;
    const uint64_t end = r.off + r.len;
    const uint64_t lo = window > r.off ? window : r.off;
    const uint64_t hi = window + TILE < end ? window + TILE : end;

    const uint32_t tid = threadIdx.x;

    if (hi - lo == TILE) {  // whole aligned window
        const gmem_u32x4 *s = gmem_words(src + lo);
        gmem_u32x4 *d = gmem_words(dst + lo);
        u32x4 v[PER_LANE];
#pragma unroll
        for (int k = 0; k < PER_LANE; ++k) v[k] = __builtin_nontemporal_load(&s[tid + k * kThreads]);
#pragma unroll
        for (int k = 0; k < PER_LANE; ++k) d[tid + k * kThreads] = v[k];
        return;
    }

    // Ragged tile: bytes up to the next 16-byte boundary, 16-byte words, bytes
    // after the last boundary.
    uint64_t body = (lo + 15) & ~15ull;
    if (body > hi) body = hi;
    uint64_t tail = hi & ~15ull;
    if (tail < body) tail = body;

    const gmem_u8 *sb = gmem_bytes(src);
    gmem_u8 *db = gmem_bytes(dst);
    if (tid < (uint32_t)(body - lo)) db[lo + tid] = sb[lo + tid];
    if (tid >= 64 && tid - 64 < (uint32_t)(hi - tail)) db[tail + tid - 64] = sb[tail + tid - 64];

    const gmem_u32x4 *s = gmem_words(src + body);
    gmem_u32x4 *d = gmem_words(dst + body);
    const uint32_t words = (uint32_t)((tail - body) >> 4);
    uint32_t w = tid;
    for (; w + 3 * kThreads < words; w += 4 * kThreads) {
        const u32x4 a = __builtin_nontemporal_load(&s[w]), b = __builtin_nontemporal_load(&s[w + kThreads]),
                    c = __builtin_nontemporal_load(&s[w + 2 * kThreads]),
                    e = __builtin_nontemporal_load(&s[w + 3 * kThreads]);
        d[w] = a;
        d[w + kThreads] = b;
        d[w + 2 * kThreads] = c;
        d[w + 3 * kThreads] = e;
    }
    for (; w < words; w += kThreads) d[w] = __builtin_nontemporal_load(&s[w]);
}

}  // namespace

hipError_t launch_step_copy(const Row *rows, const Tile *tiles, uint8_t *const *bases,
                            uint32_t n_tiles, int tile_log2, int n_xcd, hipStream_t stream) {
    const uint32_t x = n_xcd > 0 ? (uint32_t)n_xcd : 1u;
    const dim3 grid((n_tiles + x - 1u) / x * x), block(kThreads);
    switch (tile_log2) {
        case 12: hipLaunchKernelGGL(step_copy<12>, grid, block, 0, stream, rows, tiles, bases, n_tiles, x); break;
        case 13: hipLaunchKernelGGL(step_copy<13>, grid, block, 0, stream, rows, tiles, bases, n_tiles, x); break;
        case 14: hipLaunchKernelGGL(step_copy<14>, grid, block, 0, stream, rows, tiles, bases, n_tiles, x); break;
        case 15: hipLaunchKernelGGL(step_copy<15>, grid, block, 0, stream, rows, tiles, bases, n_tiles, x); break;
        case 16: hipLaunchKernelGGL(step_copy<16>, grid, block, 0, stream, rows, tiles, bases, n_tiles, x); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace vbcast
