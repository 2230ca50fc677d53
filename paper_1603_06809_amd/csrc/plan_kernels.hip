// Schedule generation on the GPU: chunk and rank descriptors, per-step row
// tables of the binomial scatter and of the native / tuned ring allgather, and
// the tile maps the copy kernel is launched over.
//
// Layout of the work: one workgroup of 4 wavefronts (64 lanes each) per step,
// lanes over the senders' relative ranks in ascending order.  Rows that exist
// are compacted with a wavefront ballot (index inside the wave = number of set
// bits below the lane), the tiles per row are turned into an exclusive prefix
// sum with a wavefront scan, and one exchange of the per-wave totals through LDS
// per round of 256 ranks carries both across the wavefronts, together with the
// step's counts and byte sum.

#include "vbcast_internal.h"

namespace vbcast {

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;

__device__ __forceinline__ uint32_t lane() { return __lane_id(); }

template <class T>
__device__ __forceinline__ T wave_inclusive_scan(T v) {
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        T o = __shfl_up(v, d, 64);
        if ((int)lane() >= d) v += o;
    }
    return v;
}

// Exclusive scan over the workgroup in thread order; returns this thread's
// prefix and the workgroup total.  `slots` is LDS for kWaves values.
template <class T>
__device__ __forceinline__ T block_exclusive_scan(T v, T *slots, T &total) {
    const int w = threadIdx.x >> 6;
    T incl = wave_inclusive_scan(v);
    if (lane() == 63) slots[w] = incl;
    __syncthreads();
    T before = 0, all = 0;
#pragma unroll
    for (int k = 0; k < kWaves; ++k) {
        T t = slots[k];
        if (k < w) before += t;
        all += t;
    }
    __syncthreads();
    total = all;
    return before + incl - v;
}

__device__ __forceinline__ uint32_t lowbit(uint32_t x) { return x & (0u - x); }

// ---------------------------------------------------------------------------
// Kernel 1: descriptors.  One workgroup.
//
// Chunk c (relative index) has length clamp(n - c * ss, 0, ss); its offset is
// the running sum of the lengths before it [Sec. IV, listing: counts and
// displacements].  Rank r has relative rank (r - root) mod P, ring neighbours
// r -+ 1 mod P, and the tuned ring's switch point (step, flag) [Sec. IV,
// listing: the scan over halving distances].  That scan stops at the largest
// power of two dividing the right neighbour's relative rank (receive-only
// tail) or, failing that, the rank's own (send-only tail); a relative rank of
// 0 is divisible by every distance, so the root and its left neighbour stop at
// the very first distance with step = P.  Lowest-set-bit arithmetic gives the
// same result without a loop.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void plan_descriptors(PlanArrays pa) {
    __shared__ uint64_t slots[kWaves];
    const int P = pa.P;
    uint64_t carry = 0;
    for (int base = 0; base < P; base += kThreads) {
        const int c = base + (int)threadIdx.x;
        uint64_t len = 0;
        if (c < P) {
            const uint64_t disp = (uint64_t)c * pa.ss;
            if (disp < pa.n) len = (pa.n - disp < pa.ss) ? pa.n - disp : pa.ss;
        }
        uint64_t total;
        const uint64_t before = block_exclusive_scan<uint64_t>(len, slots, total);
        if (c < P) {
            pa.chunk_len[c] = len;
            pa.chunk_off[c] = carry + before;
        }
        carry += total;
    }
    if (threadIdx.x == 0) pa.chunk_off[P] = carry;

    for (int r = threadIdx.x; r < P; r += kThreads) {
        int rel = r - pa.root;
        if (rel < 0) rel += P;
        const int right_rel = (rel + 1 < P) ? rel + 1 : rel + 1 - P;
        int step = -1, flag = -1;
        if (P > 1) {
            if (right_rel == 0) {
                step = P;
                flag = 1;
            } else if (rel == 0) {
                step = P;
                flag = 0;
            } else if ((right_rel & 1) == 0) {
                const int span = (int)lowbit((uint32_t)right_rel);
                step = (right_rel + span > P) ? P - right_rel : span;
                flag = 1;
            } else {
                const int span = (int)lowbit((uint32_t)rel);
                step = (rel + span > P) ? P - rel : span;
                flag = 0;
            }
        }
        pa.rel[r] = rel;
        pa.left[r] = (r + P - 1) % P;
        pa.right[r] = (r + 1) % P;
        pa.sw_step[r] = step;
        pa.sw_flag[r] = flag;
    }
}

// ---------------------------------------------------------------------------
// Kernel 2: row tables.  One workgroup per step.
//
// Scatter level t (distance m = 2^(L-1-t)) [Sec. III-A, Figs. 1-2]: every
// relative rank rho that is a multiple of 2m and has rho + m < P sends the
// chunks [rho + m, min(rho + 2m, P)) as one message to rho + m.
//
// Binomial-broadcast level and recursive-doubling exchange [Abstract, Sec. I: the
// neighbouring algorithms, named there]: see the two branches below.
//
// Ring step i = 1..P-1 [Sec. III-A Fig. 3; Sec. IV listing]: the rank with
// relative rank rho sends the chunk with relative index (rho - i + 1) mod P to
// its right neighbour.  NATIVE posts every such send.  TUNED posts it while
// the sender's step <= P - i and afterwards only if the sender's tail is
// send-only; the receiver decides symmetrically from its own (step, flag), and
// the two decisions are compared (they always agree).  Every scatter and ring
// decision is also written into the chunk-major chain view used by the
// one-launch executor.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void plan_rows(PlanArrays pa) {
    __shared__ uint32_t wave_rows[kWaves], wave_tiles[kWaves], wave_posted[kWaves], wave_mismatch[kWaves];
    __shared__ uint64_t wave_bytes[kWaves];

    const int P = pa.P;
    const int s = blockIdx.x;
    // what kind of step this is
    enum { SCATTER, RING, TREE, EXCHANGE };
    int kind;
    if (s < pa.n_scatter) kind = SCATTER;
    else if (pa.algo == kAlgoBinomial) kind = TREE;
    else if (pa.algo == kAlgoScatterRdb) kind = EXCHANGE;
    else kind = RING;
    const int m = (kind == SCATTER || kind == TREE) ? (1 << (pa.L - 1 - s)) : 0;  // tree distance
    const int i = s - pa.n_scatter + 1;                                          // ring step
    const int dist = kind == EXCHANGE ? (1 << (s - pa.n_scatter)) : 0;           // exchange distance
    const int tl = pa.tile_log2;

    Row *rows = pa.rows + (size_t)s * P;
    uint32_t *tile_ptr = pa.tile_ptr + (size_t)s * (P + 1);

    uint32_t n_rows = 0, n_tiles = 0, n_posted = 0, n_mismatch = 0;
    uint64_t n_bytes = 0;

    for (int base = 0; base < P; base += kThreads) {
        const int rho = base + (int)threadIdx.x;
        bool posted = false, mismatch = false;
        int dst_rel = 0;
        uint64_t off = 0, len = 0;
        if (rho < P) {
            if (kind == SCATTER) {
                if ((rho & (2 * m - 1)) == 0 && rho + m < P) {
                    dst_rel = rho + m;
                    const int end = (rho + 2 * m < P) ? rho + 2 * m : P;
                    off = pa.chunk_off[dst_rel];
                    len = pa.chunk_off[end] - off;
                    posted = len > 0;
                }
            } else if (kind == TREE) {
                // binomial broadcast: the scatter's tree, the whole message on every edge
                if ((rho & (2 * m - 1)) == 0 && rho + m < P) {
                    dst_rel = rho + m;
                    off = 0;
                    len = pa.n;
                    posted = true;
                }
            } else if (kind == EXCHANGE) {
                // recursive doubling: swap the aligned block gathered so far with the
                // rank whose relative rank differs in this one bit
                const int mine = rho & ~(dist - 1);
                dst_rel = rho ^ dist;
                off = pa.chunk_off[mine];
                len = pa.chunk_off[mine + dist] - off;
                posted = true;
            } else {
                int c = rho + 1 - i;
                if (c < 0) c += P;
                dst_rel = (rho + 1 < P) ? rho + 1 : 0;
                off = pa.chunk_off[c];
                len = pa.chunk_len[c];
                if (pa.algo == kAlgoNative) {
                    posted = true;
                } else {
                    int snd = rho + pa.root;
                    if (snd >= P) snd -= P;
                    int rcv = dst_rel + pa.root;
                    if (rcv >= P) rcv -= P;
                    const bool sends = pa.sw_step[snd] <= P - i || pa.sw_flag[snd] == 0;
                    const bool recvs = pa.sw_step[rcv] <= P - i || pa.sw_flag[rcv] == 1;
                    posted = sends;
                    mismatch = sends != recvs;
                }
            }
        }
        const bool valid = posted && len > 0;
        const size_t chain_stride = (size_t)pa.L + (size_t)P - 1;
        if (kind == RING && rho < P) {
            // the same decision, filed under the chunk instead of the step
            int c = rho + 1 - i;
            if (c < 0) c += P;
            int dst = dst_rel + pa.root;
            if (dst >= P) dst -= P;
            pa.chain[(size_t)c * chain_stride + (size_t)s] =
                reinterpret_cast<uint64_t>(pa.bases[dst]) | (valid ? 0ull : 1ull);
        }
        if (kind == SCATTER && rho < P && (pa.algo == kAlgoNative || pa.algo == kAlgoTuned)) {
            // The scatter level seen from chunk c = rho: the message of the subtree root
            // (c with its low bits cleared) to that root + m carries this chunk iff bit
            // m of c is set; after the level the chunk sits at c with the bits below m
            // cleared.
            const int c = rho;
            const bool moves = (c & m) != 0 && pa.chunk_len[c] > 0;
            int holder = (c & ~(m - 1)) + pa.root;
            if (holder >= P) holder -= P;
            pa.chain[(size_t)c * chain_stride + (size_t)s] =
                reinterpret_cast<uint64_t>(pa.bases[holder]) | (moves ? 0ull : 1ull);
        }
        uint32_t tiles_here = 0;
        if (valid) tiles_here = (uint32_t)(((off + len - 1) >> tl) - (off >> tl)) + 1u;

        // One exchange of wave totals through LDS serves all five quantities: the
        // compacted row index and the tile offset need a prefix, the counts of
        // posted sends, of disagreeing pairs and the byte sum only a total.
        const int w = threadIdx.x >> 6;
        const uint64_t row_votes = __ballot(valid);
        const uint32_t row_below = __popcll(row_votes & ((1ull << lane()) - 1ull));
        const uint32_t tile_incl = wave_inclusive_scan<uint32_t>(tiles_here);
        uint64_t byte_sum = valid ? len : 0;
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) byte_sum += __shfl_xor(byte_sum, d, 64);
        const uint32_t posted_here = __popcll(__ballot(posted));
        const uint32_t mismatch_here = __popcll(__ballot(mismatch));
        if (lane() == 63) {
            wave_rows[w] = __popcll(row_votes);
            wave_tiles[w] = tile_incl;
            wave_posted[w] = posted_here;
            wave_mismatch[w] = mismatch_here;
            wave_bytes[w] = byte_sum;
        }
        __syncthreads();
        uint32_t rows_before = 0, tiles_before = 0;
        uint32_t rows_total = 0, tiles_total = 0, posted_total = 0, mismatch_total = 0;
        uint64_t bytes_total = 0;
#pragma unroll
        for (int k = 0; k < kWaves; ++k) {
            if (k < w) {
                rows_before += wave_rows[k];
                tiles_before += wave_tiles[k];
            }
            rows_total += wave_rows[k];
            tiles_total += wave_tiles[k];
            posted_total += wave_posted[k];
            mismatch_total += wave_mismatch[k];
            bytes_total += wave_bytes[k];
        }
        __syncthreads();   // the slots are written again in the next round
        const uint32_t row_idx = rows_before + row_below;
        const uint32_t tile_before = tiles_before + tile_incl - tiles_here;

        if (valid) {
            int src = rho + pa.root;
            if (src >= P) src -= P;
            int dst = dst_rel + pa.root;
            if (dst >= P) dst -= P;
            Row r;
            r.src = (uint32_t)src;
            r.dst = (uint32_t)dst;
            r.off = off;
            r.len = len;
            rows[n_rows + row_idx] = r;
            tile_ptr[n_rows + row_idx] = n_tiles + tile_before;
        }
        n_rows += rows_total;
        n_tiles += tiles_total;
        n_posted += posted_total;
        n_mismatch += mismatch_total;
        n_bytes += bytes_total;
    }
    if (threadIdx.x == 0) {
        tile_ptr[n_rows] = n_tiles;
        pa.step_rows[s] = n_rows;
        pa.step_tiles[s] = n_tiles;
        pa.step_posted[s] = n_posted;
        pa.step_mismatch[s] = n_mismatch;
        pa.step_bytes[s] = n_bytes;
    }
}

// ---------------------------------------------------------------------------
// Kernel 3: tile maps.  grid = (tile slots / 256, steps).  Each lane owns one
// tile slot of its step and finds, by bisection over the step's exclusive tile
// scan (staged in LDS when it fits), the row the tile belongs to.
// ---------------------------------------------------------------------------
constexpr int kStageMax = 8192;

__global__ __launch_bounds__(kThreads) void plan_tiles(PlanArrays pa) {
    __shared__ uint32_t stage[kStageMax];
    const int s = blockIdx.y;
    const uint32_t n_tiles = pa.step_tiles[s];
    if (blockIdx.x * (uint32_t)kThreads >= n_tiles) return;  // whole workgroup leaves
    const uint32_t n_rows = pa.step_rows[s];
    const uint32_t *ptr = pa.tile_ptr + (size_t)s * (pa.P + 1);
    if (n_rows + 1 <= (uint32_t)kStageMax) {
        for (uint32_t k = threadIdx.x; k <= n_rows; k += kThreads) stage[k] = ptr[k];
        __syncthreads();
        ptr = stage;
    }
    const uint32_t b = blockIdx.x * (uint32_t)kThreads + threadIdx.x;
    if (b >= n_tiles || b >= pa.tile_cap) return;
    uint32_t lo = 0, hi = n_rows;  // ptr[lo] <= b < ptr[hi]
    while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if (ptr[mid] <= b)
            lo = mid;
        else
            hi = mid;
    }
    Tile t;
    t.row = lo;
    t.idx = b - ptr[lo];
    pa.tiles[(size_t)s * pa.tile_cap + b] = t;
}

// ---------------------------------------------------------------------------
// Census.  One workgroup per step walks the step's stored rows and counts
// those whose two ranks sit on different nodes under blocked placement (rank r
// on node r / ranks_per_node) [Sec. V-A], and their bytes; wave reductions, then
// an LDS exchange of the four sums.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void plan_census(PlanArrays pa, int ranks_per_node) {
    __shared__ uint64_t slots[kWaves];
    const int s = blockIdx.x;
    const uint32_t n_rows = pa.step_rows[s];
    const Row *rows = pa.rows + (size_t)s * pa.P;
    uint64_t v[4] = {0, 0, 0, 0};
    for (uint32_t k = threadIdx.x; k < n_rows; k += kThreads) {
        const Row r = rows[k];
        const bool inter = (int)r.src / ranks_per_node != (int)r.dst / ranks_per_node;
        v[inter ? 0 : 2] += 1;
        v[inter ? 1 : 3] += r.len;
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        uint64_t total;
        (void)block_exclusive_scan<uint64_t>(v[q], slots, total);
        if (threadIdx.x == 0) pa.census[(size_t)s * 4 + q] = total;
    }
}

}  // namespace

hipError_t launch_plan_census(const PlanArrays &pa, int ranks_per_node, hipStream_t stream) {
    if (pa.n_steps == 0) return hipSuccess;
    hipLaunchKernelGGL(plan_census, dim3(pa.n_steps), dim3(kThreads), 0, stream, pa, ranks_per_node);
    return hipGetLastError();
}

hipError_t launch_plan_kernels(const PlanArrays &pa, int tile_map_steps, hipStream_t stream) {
    hipLaunchKernelGGL(plan_descriptors, dim3(1), dim3(kThreads), 0, stream, pa);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (pa.n_steps == 0) return hipSuccess;
    hipLaunchKernelGGL(plan_rows, dim3(pa.n_steps), dim3(kThreads), 0, stream, pa);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (tile_map_steps <= 0) return hipSuccess;
    if (tile_map_steps > pa.n_steps) tile_map_steps = pa.n_steps;
    const uint32_t gx = (pa.tile_cap + kThreads - 1) / kThreads;
    hipLaunchKernelGGL(plan_tiles, dim3(gx, tile_map_steps), dim3(kThreads), 0, stream, pa);
    return hipGetLastError();
}

}  // namespace vbcast
