// Scatter and ring executed in dependency order by one launch.
//
// In the ring a chunk travels: the chunk with relative index c starts at the
// rank that holds it after the scatter and in ring step i is passed from
// relative rank c + i - 1 to c + i [Sec. III-A: every rank forwards what it
// received one step earlier].  So the transfer of a chunk in step i + 1 depends
// only on that chunk's transfer in step i - never on another chunk - which is
// all the ordering MPI's blocking calls impose; there is no barrier between
// ring steps in the paper's code either [Sec. IV, listing].  The tuned ring
// drops some transfers of a chain (the receiver already holds the chunk from
// the scatter); the chain then continues from that receiver's copy.  The
// scatter is the same kind of chain: chunk c goes down the binomial tree from
// the root to rank c, one hop at every level whose distance bit is set in c
// [Sec. III-A, Figs. 1-2], and every rank that holds the chunk "from the
// scatter" got it from this very chain.  So the whole broadcast splits into
// independent chains, one per piece of a chunk, each starting in the root's
// buffer.
//
// (Chunks of at least 1 KiB; shorter ones take the per-wavefront kernel at the
// end of this file.)  The message space [0, n) is cut into tile-aligned
// slabs.  A workgroup takes a slab and walks it through all scatter levels and
// ring steps: in a step it copies the slab's part of each chunk from the step's
// source rank to its destination rank (the same rows the step tables hold), then
// fences and goes on with the next step, whose source is what it has just
// written.  Which buffer a chunk is in after a step, and whether the step moves
// it at all, the kernel either works out itself from (P, root, n, schedule) -
// no table is read and the broadcast is this one launch - or looks up in the
// chunk-major "chain" view that the table kernels write next to the step tables
// (see the two Hops types below).  Every lane re-reads from memory exactly the
// words it wrote one step earlier; they are still in the compute unit's
// write-through L1 (or the XCD's L2), so the only traffic that has to reach HBM
// is the write of every rank's copy.  The resident workgroups together hold
// (workgroups x tile) bytes in flight, sized so that a compute unit's share fits
// its L1; a workgroup that finishes a slab takes the next one a whole grid
// further on, so all workgroups do the same amount of work.
//
// Between two steps a workgroup-scope fence orders the stores of one step
// before the loads of the next: writer and reader of every byte are the same
// lane, and all wavefronts of a workgroup share one L1 (the code is not built
// for threadgroup-split mode).  Wider scopes are not needed and are costly here:
// an agent-scope acquire invalidates the whole L2 of the XCD.

#include "vbcast_internal.h"

namespace vbcast {

namespace {

constexpr int kThreads = 256;
constexpr uint32_t kLine = 128;    // bytes of a cache line
constexpr int kMinSlabLog2 = 10;   // smallest slab: one wavefront, one word per lane
constexpr int kFillSlabLog2 = 12;  // slabs are not made smaller than this just to get more of them

// Whether the whole-tile path lets the wavefronts of a workgroup take turns (one
// wavefront copies the slab per hop) instead of sharing every hop: worth it from
// 16 KiB slabs on, where a hop moves enough for the barrier not to matter.
template <int TILE_LOG2, int THREADS>
constexpr bool kTakeTurns = TILE_LOG2 >= 14 && THREADS >= 128;

__device__ __forceinline__ void step_fence() {
    // Writer and reader of every byte are in the same workgroup (in fact the
    // same lane), so workgroup scope is the right one: all wavefronts of a
    // workgroup sit behind one L1, which their own stores keep consistent, and
    // nothing has to be written back or invalidated.  In this execution mode the
    // fence emits no instruction; it keeps the compiler from moving the next
    // step's loads above this step's stores.
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
}

// Waits until every load issued so far has returned.  Loads and stores of a
// wavefront complete through one in-order counter, so a wait that the compiler
// places between two stores of a step (it does, when the stores sit in separate
// conditional blocks) also waits for the first store to be acknowledged by the
// L2: one more round trip in the step.  Waiting once, right after the step's
// loads, leaves nothing to wait for between the stores.
__device__ __forceinline__ void wait_for_loads() {
    // s_waitcnt vmcnt(0), with the export and LDS/scalar counters left alone
    __builtin_amdgcn_s_waitcnt(0x0F70);
}

__device__ __forceinline__ uint32_t lowbit(uint32_t x) { return x & (0u - x); }

// Two ways to know the hops of a chunk's chain.  Both answer, for the chunk with
// relative index c and step s (scatter levels 0..L-1, then ring steps):
//   entry(c, s)   the buffer that holds the chunk after step s, with bit 0 set
//                 when step s has no transfer for this chunk (it is not on the
//                 chunk's tree path at that level, the tuned ring drops it, or the
//                 chunk is empty) - buffers are 16-byte aligned, the bit is free;
//   source(c, s)  the buffer step s reads the chunk from: the root's before the
//                 first step [Sec. III-A: the scatter starts from the root], else
//                 the holder after step s - 1;
//   chunk_begin(c) the chunk's byte offset in the message.
// prepare(...) is called by all threads of a workgroup before it walks a slab (by
// all lanes of a wavefront before it walks a chunk, in the small-chunk kernel) and
// names the chunks that entry() will be asked about until the next prepare.

// Worked out by the kernel itself.  Scatter level t has distance m = 2^(L-1-t):
// chunk c rides the message from its subtree's root (c with the bits below 2m
// cleared) to that root + m iff bit m of c is set, and afterwards sits at c with
// the bits below m cleared [Sec. III-A, Figs. 1-2].  Ring step i passes chunk c
// from relative rank c + i - 1 to c + i [Sec. III-A, Fig. 3].  The tuned ring
// leaves that transfer out once the receiver has begun to get back what it has
// held since the scatter [Sec. IV]: relative rank r came out of the scatter with
// span(r) chunks - all P for the root, else the largest power of two dividing r,
// cut at the end of the ranks - and the last span(r) - 1 chunks the ring would
// bring it are those, so it receives in steps i <= P - span(r) only.
//
// The hops of a chunk are computed when a workgroup turns to a slab of that
// chunk, one hop per lane, and kept in LDS while the slab is walked: a step then
// gets its entry with one LDS read instead of a chain of scalar arithmetic that
// would sit in the dependent path of every step.  The rank buffers' addresses
// are copied to LDS once per workgroup, so that computing a chunk's hops reads
// no memory at all (a load from memory waits behind the kernel's own stores).
struct InlineHops {
    // LDS words: the rank buffers, then `chunks` sets of entries
    static constexpr int lds_words(int chunks) { return kInlineMaxRanks + chunks * kInlineMaxHops; }

    uint8_t *const *bases;   // [P] rank buffers, by absolute rank
    int P, L, root;
    bool tuned;
    uint64_t n, ss;
    const uint64_t *rank_buffer;   // LDS copy of bases
    uint64_t *first_slots;   // LDS: entries of chunk `first_chunk`, indexed by step
    uint64_t *other_slots;   // LDS: entries of the other chunk prepared (if any)
    int first_chunk;

    __device__ __forceinline__ static InlineHops make(const uint64_t *, const uint64_t *,
                                                       uint8_t *const *bases, int P, int L, int root,
                                                       int tuned, uint64_t n, uint64_t ss) {
        return InlineHops{bases, P, L, root, tuned != 0, n, ss, nullptr, nullptr, nullptr, -1};
    }
    // All threads of the workgroup, once, before anything else: `lds` = lds_words(..) words.
    __device__ __forceinline__ void begin(uint64_t *lds) {
        for (int r = threadIdx.x; r < P; r += blockDim.x) lds[r] = reinterpret_cast<uint64_t>(bases[r]);
        rank_buffer = lds;
        __syncthreads();
    }
    __device__ __forceinline__ uint64_t chunk_begin(int c) const {
        const uint64_t at = (uint64_t)c * ss;
        return at < n ? at : n;
    }
    __device__ __forceinline__ uint64_t compute(int c, uint32_t s) const {
        int holder;   // relative rank
        bool moves;
        if (s < (uint32_t)L) {
            const int m = 1 << (L - 1 - (int)s);
            holder = c & ~(m - 1);
            moves = (c & m) != 0;
        } else {
            const int i = (int)s - L + 1;
            holder = c + i;
            if (holder >= P) holder -= P;
            int span = P;
            if (holder != 0) {
                span = (int)lowbit((uint32_t)holder);
                if (span > P - holder) span = P - holder;
            }
            moves = !tuned || span <= P - i;
        }
        if ((uint64_t)c * ss >= n) moves = false;   // an empty chunk
        int rank = holder + root;
        if (rank >= P) rank -= P;
        return rank_buffer[rank] | (moves ? 0ull : 1ull);
    }
    // Entries of steps [first_step - 1, last_step) of `c` into `slots`, one step per
    // lane of the `lanes` lanes that call this together (`lane` = 0..lanes-1).
    __device__ __forceinline__ void fill(uint64_t *slots, int c, uint32_t first_step,
                                         uint32_t last_step, uint32_t lane, uint32_t lanes) const {
        for (uint32_t s = (first_step ? first_step - 1 : 0) + lane; s < last_step; s += lanes)
            slots[s] = compute(c, s);
    }
    // Workgroup: the one or two chunks of the next slab (`lds` as given to begin,
    // two sets of entries).
    __device__ __forceinline__ void prepare(uint64_t *lds, int c0, int c1, uint32_t first_step,
                                            uint32_t last_step) {
        __syncthreads();   // nobody reads the previous slab's entries any more
        first_slots = lds + kInlineMaxRanks;
        other_slots = first_slots + kInlineMaxHops;
        first_chunk = c0;
        fill(first_slots, c0, first_step, last_step, threadIdx.x, blockDim.x);
        if (c1 != c0) fill(other_slots, c1, first_step, last_step, threadIdx.x, blockDim.x);
        __syncthreads();
    }
    // Wavefront `wave` of the workgroup: its one chunk (`lds` as given to begin, one
    // set of entries per wavefront).  A wavefront's LDS accesses are carried out in
    // the order it issues them, so its own reads see its writes.
    __device__ __forceinline__ void prepare_wave(uint64_t *lds, uint32_t wave, int c,
                                                 uint32_t first_step, uint32_t last_step) {
        first_slots = other_slots = lds + kInlineMaxRanks + (size_t)wave * kInlineMaxHops;
        first_chunk = c;
        fill(first_slots, c, first_step, last_step, threadIdx.x & 63u, 64u);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
    // (c, s) is the same in all lanes of the calling wavefront, everywhere in this
    // file: say so, and what is done with the entry stays scalar.
    __device__ __forceinline__ uint64_t entry(int c, uint32_t s) const {
        const uint64_t v = (c == first_chunk ? first_slots : other_slots)[s];
        const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
        const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
        return ((uint64_t)hi << 32) | lo;
    }
    __device__ __forceinline__ uint64_t source(int c, uint32_t s) const {
        return s == 0 ? reinterpret_cast<uint64_t>(bases[root]) : entry(c, s - 1);
    }
};

// Looked up in what the table kernels wrote: chain[c * hops + s] is entry(c, s),
// chunk_off[c] the chunk's offset.  The lookups are scalar loads that miss the
// scalar cache (the table is far larger) and return after one trip to the L2
// and back on a path of their own, not behind the compute unit's stores.  Where
// the wavefronts take turns, the wavefront that has just had its turn waits for
// such a load before it rejoins the barrier, so a workgroup starts a step no
// sooner than the L2 answers a read - a little slower when the device is
// otherwise idle, a few per cent faster when all compute units stream at once
// (measured: the same kernel with the entries in LDS, which come back at once,
// loses 3-4 % on a 64 GiB broadcast and wins on short ones).
struct TableHops {
    const uint64_t *chain;
    const uint64_t *chunk_off;
    uint8_t *const *bases;
    size_t hops;             // L + P - 1 entries per chunk
    int root;

    __device__ __forceinline__ static TableHops make(const uint64_t *chain, const uint64_t *chunk_off,
                                                      uint8_t *const *bases, int P, int L, int root,
                                                      int, uint64_t, uint64_t) {
        return TableHops{chain, chunk_off, bases, (size_t)L + (size_t)P - 1, root};
    }
    static constexpr int lds_words(int) { return 1; }
    __device__ __forceinline__ uint64_t chunk_begin(int c) const { return chunk_off[c]; }
    __device__ __forceinline__ void begin(uint64_t *) {}
    __device__ __forceinline__ void prepare(uint64_t *, int, int, uint32_t, uint32_t) {}
    __device__ __forceinline__ void prepare_wave(uint64_t *, uint32_t, int, uint32_t, uint32_t) {}
    __device__ __forceinline__ uint64_t entry(int c, uint32_t s) const {
        return chain[(size_t)c * hops + s];
    }
    __device__ __forceinline__ uint64_t source(int c, uint32_t s) const {
        return s == 0 ? reinterpret_cast<uint64_t>(bases[root]) : entry(c, s - 1);
    }
};

__device__ __forceinline__ const uint8_t *buffer_of(uint64_t entry) {
    return reinterpret_cast<const uint8_t *>(entry & ~15ull);
}

// The cache line in which chunks c - 1 and c meet (none when chunk c starts on a
// line boundary, or is empty): bytes below the cut follow chunk c - 1's chain,
// bytes from the cut on chunk c's, one lane per byte, through steps [first_step,
// last_step).  Every buffer gets this line in two parts, in different steps, and
// a step on a partly written line costs about twice a step on whole lines; as a
// chain of its own - one workgroup per line, beside the workgroups that walk the
// slabs - it is 128 bytes that take a few hundred microseconds at most and hold
// nothing else up.  Called by all threads of the workgroup.
template <int THREADS, class Hops>
__device__ __forceinline__ void walk_cut_line(Hops &hops, uint64_t *lds, int c, uint64_t n,
                                              uint32_t first_step, uint32_t last_step) {
    const uint64_t cut = hops.chunk_begin(c);
    if (cut >= n || (cut & (kLine - 1)) == 0) return;   // the same for the whole workgroup
    hops.prepare(lds, c - 1, c, first_step, last_step);
    const uint64_t line = cut & ~(uint64_t)(kLine - 1);
    constexpr int PER_LANE = THREADS >= (int)kLine ? 1 : (int)kLine / THREADS;
    uint64_t at[PER_LANE];
    bool in_a[PER_LANE], in_b[PER_LANE];
#pragma unroll
    for (int k = 0; k < PER_LANE; ++k) {
        const uint32_t b = threadIdx.x + (uint32_t)k * THREADS;
        at[k] = line + b;
        const bool in_line = b < kLine && at[k] < n;
        in_a[k] = in_line && at[k] < cut;
        in_b[k] = in_line && at[k] >= cut;
    }
    const uint8_t *srcA = buffer_of(hops.source(c - 1, first_step));
    const uint8_t *srcB = buffer_of(hops.source(c, first_step));
    uint64_t eA = hops.entry(c - 1, first_step);
    uint64_t eB = hops.entry(c, first_step);
    for (uint32_t i = first_step + 1; i <= last_step; ++i) {
        const uint32_t nx = i < last_step ? i : first_step;
        const uint64_t nA = hops.entry(c - 1, nx);
        const uint64_t nB = hops.entry(c, nx);
        uint8_t *dA = reinterpret_cast<uint8_t *>(eA & ~15ull);
        uint8_t *dB = reinterpret_cast<uint8_t *>(eB & ~15ull);
        const bool runA = !(eA & 1), runB = !(eB & 1);
        uint8_t one[PER_LANE];
        bool on[PER_LANE];
#pragma unroll
        for (int k = 0; k < PER_LANE; ++k) {
            on[k] = (in_a[k] && runA) || (in_b[k] && runB);
            if (on[k]) one[k] = *gmem_bytes((in_a[k] ? srcA : srcB) + at[k]);
        }
        wait_for_loads();
#pragma unroll
        for (int k = 0; k < PER_LANE; ++k)
            if (on[k]) *gmem_bytes((in_a[k] ? dA : dB) + at[k]) = one[k];
        step_fence();
        srcA = dA;
        srcB = dB;
        eA = nA;
        eB = nB;
    }
}

// Steps [first_step, last_step) of every slab of the message.  `chain` and
// `chunk_off` are read only by TableHops, `tuned` only by InlineHops.  The
// pointers are separate restrict-qualified kernel arguments on purpose: that is
// what lets the compiler fetch entries and buffer addresses with scalar loads
// although the kernel stores through pointers it has loaded.
template <int TILE_LOG2, int THREADS, class Hops>
__global__ __launch_bounds__(THREADS) void ring_chain(const uint64_t *__restrict__ chain,
                                                       const uint64_t *__restrict__ chunk_off,
                                                       uint8_t *const *__restrict__ bases, int P,
                                                       int L, int root, int tuned, uint64_t n,
                                                       uint64_t ss, uint32_t n_slabs,
                                                       uint32_t slab_wgs, uint32_t cut_wgs,
                                                       uint32_t xcd_run, uint32_t n_xcd,
                                                       uint32_t first_step, uint32_t last_step) {
    __shared__ uint64_t hop_slots[Hops::lds_words(2)];
    Hops hops = Hops::make(chain, chunk_off, bases, P, L, root, tuned, n, ss);
    hops.begin(hop_slots);
    if (blockIdx.x >= slab_wgs) {
        // the `cut_wgs` workgroups after those that walk slabs: one line each
        walk_cut_line<THREADS>(hops, hop_slots, (int)(blockIdx.x - slab_wgs) + 1, n, first_step, last_step);
        return;
    }
    const uint32_t scatter_hops = (uint32_t)L;
    constexpr uint64_t TILE = 1ull << TILE_LOG2;
    // Workgroups are handed to the XCDs round-robin (workgroup id mod n_xcd).
    // Give each XCD runs of `xcd_run` consecutive slabs (64 KiB) instead of every
    // n-th slab, so that the addresses one XCD touches spread over all of its L2
    // channels, while the XCDs together still sweep one contiguous window.
    const uint32_t W = slab_wgs;  // a multiple of n_xcd; W / n_xcd is a multiple of xcd_run
    const uint32_t in_xcd = blockIdx.x / n_xcd;
    const uint32_t first = (in_xcd / xcd_run) * n_xcd * xcd_run + (blockIdx.x % n_xcd) * xcd_run +
                           (in_xcd % xcd_run);
    for (uint32_t slab = first; slab < n_slabs; slab += W) {
        const uint64_t lo = (uint64_t)slab << TILE_LOG2;
        const uint64_t hi = lo + TILE < n ? lo + TILE : n;
        const int c0 = (int)(lo / ss);
        const int c1 = (int)((hi - 1) / ss);
        hops.prepare(hop_slots, c0, c1, first_step, last_step);
        if (c1 == c0 && hi - lo == TILE && kTakeTurns<TILE_LOG2, THREADS>) {
            // A whole tile inside one chunk, slabs of 16 KiB and more: the wavefronts
            // of the workgroup take turns.  Wavefront w copies the whole slab in the
            // hops h with (h - first_step) mod WAVES == w, and a workgroup barrier
            // separates consecutive hops.  The loads of a hop are then issued by
            // another wavefront than the stores of the hop before, so they do not
            // queue behind the acknowledgement of those stores (a wavefront's loads
            // and stores complete through one in-order counter); a wavefront's own
            // previous stores are WAVES - 1 hops old when it loads again, and its
            // next chain entries arrive while the others take their turns.  Stores of
            // one wavefront are visible to the loads another wavefront of the same
            // workgroup issues after the barrier: they share the compute unit's L1
            // and its in-order path to the L2 (workgroup-scope release / acquire,
            // which in this execution mode needs no wait on the stores).
            constexpr uint32_t WAVES = THREADS / 64;
            constexpr int NW = (int)(TILE / 16) / 64;     // words per lane of the wavefront whose turn it is
            constexpr int BATCH = NW < 16 ? NW : 16;      // words loaded before the first store
            // the wavefront's number is the same in all its lanes: say so, and the turn
            // test is a scalar branch and the chain entries are scalar values
            const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
            const uint32_t lane_off = (threadIdx.x & 63u) * 16u;
            uint32_t mine = first_step + wave;            // this wavefront's next hop
            uint64_t e = 0, before = 0;                   // its entry, and the entry of the hop before
            if (mine < last_step) {
                e = hops.entry(c0, mine);
                before = hops.source(c0, mine);
            }
            // A hop that follows a dropped transfer (tuned ring) does not read what the
            // hop before wrote but the copy its source rank got from the scatter
            // [Sec. IV: that rank stopped receiving because it already held the chunk]:
            // nothing in the last few hops feeds it, and it comes from HBM, not from
            // cache.  The wavefront whose turn it will be issues those loads as soon as
            // it knows - right after its previous turn, WAVES hops ahead, once the
            // scatter hops are behind it - and only stores when its turn comes.
            u32x4 v[BATCH];
            bool loaded = false;   // v holds the words of hop `mine` already
            bool fetch = false;    // the entries of hop `mine` are still to be read
            bool early = false;    // hop `mine` reads a scatter copy: load it now
            for (uint32_t h = first_step; h < last_step; ++h) {
                const bool turn = h == mine;
                if (!turn && fetch) {
                    // read them while the next wavefront works, not before it may start
                    fetch = false;
                    e = hops.entry(c0, mine);
                    before = hops.source(c0, mine);
                    early = NW == BATCH && (before & 1) && !(e & 1) && h > scatter_hops;
                }
                const bool active = !(e & 1);
                if constexpr (NW == BATCH) {
                    // one place that loads, one that stores: the words stay in the same
                    // registers whether they were loaded early or in the turn itself
                    if ((turn && active && !loaded) || (!turn && early)) {
                        const uint8_t *src = reinterpret_cast<const uint8_t *>(before & ~15ull) + lo;
#pragma unroll
                        for (int k = 0; k < BATCH; ++k) v[k] = *gmem_words(src + lane_off + k * 1024);
                        loaded = true;
                        early = false;
                    }
                    if (turn && active) {
                        uint8_t *dst = reinterpret_cast<uint8_t *>(e & ~15ull) + lo;
#pragma unroll
                        for (int k = 0; k < BATCH; ++k) *gmem_words(dst + lane_off + k * 1024) = v[k];
                    }
                } else {
                    if (turn && active) {
                        const uint8_t *src = reinterpret_cast<const uint8_t *>(before & ~15ull) + lo;
                        uint8_t *dst = reinterpret_cast<uint8_t *>(e & ~15ull) + lo;
#pragma unroll
                        for (int b = 0; b < NW; b += BATCH) {
#pragma unroll
                            for (int k = 0; k < BATCH; ++k)
                                v[k] = *gmem_words(src + lane_off + (b + k) * 1024);
#pragma unroll
                            for (int k = 0; k < BATCH; ++k)
                                *gmem_words(dst + lane_off + (b + k) * 1024) = v[k];
                        }
                    }
                }
                if (turn) {
                    loaded = false;
                    mine += WAVES;
                    fetch = mine < last_step;
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
                __builtin_amdgcn_s_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
            }
        } else if (c1 == c0 && hi - lo == TILE) {
            // The common case with smaller slabs, a whole tile inside one chunk: every
            // lane owns the same PER_LANE words in every step, only the two buffers change.
            constexpr int PER_LANE = (int)(TILE / 16) / THREADS;
            const uint32_t lane_off = threadIdx.x * 16u;
            const uint8_t *src = buffer_of(hops.source(c0, first_step)) + lo;
            uint64_t e = hops.entry(c0, first_step);
            for (uint32_t i = first_step + 1; i <= last_step; ++i) {
                uint8_t *dst = reinterpret_cast<uint8_t *>(e & ~15ull) + lo;
                const bool moves = !(e & 1);
                u32x4 v[PER_LANE];
                if (moves) {
#pragma unroll
                    for (int k = 0; k < PER_LANE; ++k)
                        v[k] = *gmem_words(src + lane_off + k * (THREADS * 16));
                }
                // the next step's entry, while the loads are under way
                const uint64_t nxt = hops.entry(c0, i < last_step ? i : first_step);
                if (moves) {
#pragma unroll
                    for (int k = 0; k < PER_LANE; ++k)
                        *gmem_words(dst + lane_off + k * (THREADS * 16)) = v[k];
                }
                step_fence();
                src = dst;
                e = nxt;
            }
        } else {
            // Two chunks meet in this slab (or the message ends in it).  The slab is
            // still a row of 16-byte words at fixed places: a lane keeps its PER_LANE
            // words and only picks, per word, which of the two chains the word belongs
            // to.  The word that holds the cut between the chunks and the word that
            // holds the end of the message go byte by byte, one lane per byte (lanes
            // 0-15 and 16-31).  With `cut_wgs` the cache line in which the two chunks
            // meet is left out here and walked by a workgroup of its own
            // (walk_cut_line): every buffer gets that line in two parts, in different
            // steps, a line that is only partly written is not re-read from the L1, and
            // walked with the slab it makes every step of the whole slab wait for it.
            constexpr int PER_LANE = (int)(TILE / 16) / THREADS;
            const uint32_t tid = threadIdx.x;
            const uint64_t cut = c1 > c0 ? hops.chunk_begin(c1) : hi;
            const bool apart = c1 > c0 && cut_wgs != 0;
            const uint64_t a_end = apart ? cut & ~(uint64_t)(kLine - 1) : cut;                  // A = [lo, a_end)
            const uint64_t b_begin = apart ? (cut + kLine - 1) & ~(uint64_t)(kLine - 1) : cut;  // B = [b_begin, hi)
            const uint8_t *srcA = buffer_of(hops.source(c0, first_step));
            const uint8_t *srcB = buffer_of(hops.source(c1, first_step));

            uint64_t word_at[PER_LANE];
            bool word_a[PER_LANE], word_b[PER_LANE];
#pragma unroll
            for (int k = 0; k < PER_LANE; ++k) {
                word_at[k] = lo + (uint64_t)(tid + k * THREADS) * 16u;
                word_a[k] = word_at[k] + 16 <= a_end;
                word_b[k] = word_at[k] >= b_begin && word_at[k] + 16 <= hi;
            }
            // byte lanes: lanes 0-15 take the word holding `cut` (unless its line is left
            // out), 16-31 the word holding `hi` (unless it is the same word, or left out)
            const uint64_t byte_at = (tid < 16 ? (cut & ~15ull) : (hi & ~15ull)) + (tid & 15u);
            const bool byte_lane =
                tid < 32 && byte_at >= lo && byte_at < hi &&
                (tid < 16 ? (!apart && (cut & 15u) != 0)
                          : ((hi & 15u) != 0 &&
                             (apart ? (hi & ~15ull) >= b_begin : (hi & ~15ull) != (cut & ~15ull))));
            const bool byte_a = byte_lane && byte_at < cut;
            const bool byte_b = byte_lane && byte_at >= cut;

            uint64_t eA = hops.entry(c0, first_step);
            uint64_t eB = hops.entry(c1, first_step);
            for (uint32_t i = first_step + 1; i <= last_step; ++i) {
                const uint32_t nx = i < last_step ? i : first_step;  // the next step's entries, early
                const uint64_t nA = hops.entry(c0, nx);
                const uint64_t nB = hops.entry(c1, nx);
                uint8_t *dA = reinterpret_cast<uint8_t *>(eA & ~15ull);
                uint8_t *dB = reinterpret_cast<uint8_t *>(eB & ~15ull);
                const bool runA = !(eA & 1), runB = !(eB & 1);
                u32x4 v[PER_LANE];
                bool on[PER_LANE];
#pragma unroll
                for (int k = 0; k < PER_LANE; ++k) {
                    on[k] = (word_a[k] && runA) || (word_b[k] && runB);
                    const uint8_t *s = word_a[k] ? srcA : srcB;
                    if (on[k]) v[k] = *gmem_words(s + word_at[k]);
                }
                const bool byte_on = (byte_a && runA) || (byte_b && runB);
                uint8_t one = 0;
                if (byte_on) one = *gmem_bytes((byte_a ? srcA : srcB) + byte_at);
                wait_for_loads();
#pragma unroll
                for (int k = 0; k < PER_LANE; ++k) {
                    uint8_t *d = word_a[k] ? dA : dB;
                    if (on[k]) *gmem_words(d + word_at[k]) = v[k];
                }
                if (byte_on) *gmem_bytes((byte_a ? dA : dB) + byte_at) = one;
                step_fence();
                srcA = dA;
                srcB = dB;
                eA = nA;
                eB = nB;
            }
        }
    }
}

// Small chunks (shorter than the smallest slab, 1 KiB): one wavefront walks a
// whole chunk through all steps, one 16-byte word per lane.  Wavefronts are
// independent: a lane only ever re-reads what it wrote itself.  Lanes 0-15 also
// take the bytes before the chunk's first 16-byte boundary, lanes 16-31 the bytes
// after its last one.
template <class Hops>
__global__ __launch_bounds__(kThreads) void ring_chain_small(const uint64_t *__restrict__ chain,
                                                             const uint64_t *__restrict__ chunk_off,
                                                             uint8_t *const *__restrict__ bases,
                                                             int P, int L, int root, int tuned,
                                                             uint64_t n, uint64_t ss,
                                                             uint32_t first_step, uint32_t last_step) {
    __shared__ uint64_t hop_slots[Hops::lds_words(kThreads / 64)];
    Hops hops = Hops::make(chain, chunk_off, bases, P, L, root, tuned, n, ss);
    hops.begin(hop_slots);
    // the chunk is the same for all lanes of a wavefront: say so, and what depends
    // on it alone stays in scalar registers
    const int c = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * (kThreads / 64) + (threadIdx.x / 64)));
    if (c >= P) return;
    const uint32_t lane = threadIdx.x % 64;
    const uint64_t a = hops.chunk_begin(c), b = hops.chunk_begin(c + 1);
    if (a >= b) return;
    uint64_t body = (a + 15) & ~15ull;
    if (body > b) body = b;
    uint64_t tail = b & ~15ull;
    if (tail < body) tail = body;
    const bool head_lane = lane < 16 && lane < (uint32_t)(body - a);
    const bool tail_lane = lane >= 16 && lane < 32 && lane - 16 < (uint32_t)(b - tail);
    const bool byte_lane = head_lane || tail_lane;
    const uint64_t byte_at = head_lane ? a + lane : tail + (lane - 16);
    const bool word_lane = lane < (uint32_t)((tail - body) >> 4);   // fewer than 64 words
    const uint64_t word_at = body + (uint64_t)lane * 16u;

    hops.prepare_wave(hop_slots, threadIdx.x / 64, c, first_step, last_step);
    const uint8_t *src = buffer_of(hops.source(c, first_step));
    uint64_t e = hops.entry(c, first_step);
    for (uint32_t i = first_step + 1; i <= last_step; ++i) {
        const uint64_t nxt = hops.entry(c, i < last_step ? i : first_step);
        uint8_t *dst = reinterpret_cast<uint8_t *>(e & ~15ull);
        if (!(e & 1)) {
            u32x4 v;
            uint8_t one = 0;
            if (word_lane) v = *gmem_words(src + word_at);
            if (byte_lane) one = *gmem_bytes(src + byte_at);
            wait_for_loads();
            if (word_lane) *gmem_words(dst + word_at) = v;
            if (byte_lane) *gmem_bytes(dst + byte_at) = one;
        }
        step_fence();
        src = dst;
        e = nxt;
    }
}

template <class Hops>
hipError_t launch_with(const PlanArrays &pa, uint32_t wgs_at_plan_tile, int first_step,
                       int last_step, hipStream_t stream) {
    if (pa.n == 0 || pa.P < 2 || first_step >= last_step) return hipSuccess;
    if (first_step < 0 || last_step > pa.n_steps) return hipErrorInvalidValue;
    const uint32_t s0 = (uint32_t)first_step, s1 = (uint32_t)last_step;
    const int tuned = pa.algo == kAlgoTuned ? 1 : 0;
    uint64_t grid64 = 0;
    const int tl = chain_slab_log2(pa, wgs_at_plan_tile, &grid64);
    if ((1ull << tl) > pa.ss) {
        // chunks shorter than 1 KiB: one wavefront per chunk
        const uint32_t per_wg = kThreads / 64;
        hipLaunchKernelGGL(ring_chain_small<Hops>, dim3(((uint32_t)pa.P + per_wg - 1) / per_wg),
                           dim3(kThreads), 0, stream, pa.chain, pa.chunk_off, pa.bases, pa.P, pa.L,
                           pa.root, tuned, pa.n, pa.ss, s0, s1);
        return hipGetLastError();
    }
    const uint64_t n_slabs64 = (pa.n + (1ull << tl) - 1) >> tl;
    if (n_slabs64 > 0xffffffffull) return hipErrorInvalidValue;
    const uint32_t n_slabs = (uint32_t)n_slabs64;
    uint32_t grid = grid64 > n_slabs ? n_slabs : (uint32_t)grid64;
    const uint32_t n_xcd = pa.n_xcd > 0 ? (uint32_t)pa.n_xcd : 1u;
    grid = (grid + n_xcd - 1u) / n_xcd * n_xcd;  // whole rounds over the XCDs
    // slabs per XCD run: 64 KiB worth, but a divisor of the workgroups per XCD
    uint32_t xcd_run = tl < 16 ? (1u << (16 - tl)) : 1u;
    while ((grid / n_xcd) % xcd_run != 0) xcd_run >>= 1;
    // Behind the workgroups that walk slabs, one per chunk boundary for the cache line
    // the boundary falls in (it leaves at once where the boundary falls between two
    // lines).  A compute unit's L1 serves one dependent step at a time whichever
    // workgroup issued it, so the line's steps add to the time of the slab walker it
    // shares the unit with: worth it against the slab steps they no longer slow down
    // as long as every unit gets at most one line (measured: P = 256, 30 MB 1.73 ->
    // 1.63 ms; P = 129, 2.5 MB 90 -> 80 us; but P = 513, 32 MiB 3.64 -> 3.72 ms with
    // 512 of them), and for slabs of 4 KiB and more (in a smaller slab the line is a
    // large part of the slab anyway: P = 129, 192 KiB, 1 KiB slabs: 42 us with the
    // slabs, 68 us apart).
    const uint32_t cut_wgs =
        tl >= kFillSlabLog2 && pa.ss % kLine != 0 && (uint32_t)pa.P - 1u <= wgs_at_plan_tile
            ? (uint32_t)pa.P - 1u
            : 0u;
    const dim3 g(grid + cut_wgs);
    // one 16-byte word per lane in the two smallest slabs, so fewer lanes there
#define VB_LAUNCH(TL, LANES)                                                                 \
    hipLaunchKernelGGL((ring_chain<TL, LANES, Hops>), g, dim3(LANES), 0, stream, pa.chain,   \
                       pa.chunk_off, pa.bases, pa.P, pa.L, pa.root, tuned, pa.n, pa.ss, n_slabs,  \
                       grid, cut_wgs, xcd_run, n_xcd, s0, s1)
    switch (tl) {
        case 10: VB_LAUNCH(10, 64); break;
        case 11: VB_LAUNCH(11, 128); break;
        case 12: VB_LAUNCH(12, 256); break;
        case 13: VB_LAUNCH(13, 256); break;
        case 14: VB_LAUNCH(14, 256); break;
        case 15: VB_LAUNCH(15, 256); break;
        case 16: VB_LAUNCH(16, 256); break;
        default: return hipErrorInvalidValue;
    }
#undef VB_LAUNCH
    return hipGetLastError();
}

}  // namespace

int chain_slab_log2(const PlanArrays &pa, uint32_t wgs_at_plan_tile, uint64_t *workgroups) {
    // The plan's slab size, halved (with twice the workgroups, so the bytes in flight
    // stay the same)
    //  - while a slab is longer than a chunk: it must not hold more than one chunk
    //    boundary (down to 1 KiB);
    //  - down to 4 KiB, while chunks are not a whole number of slabs and hold fewer
    //    than four: slabs in which two chunks meet cost more per step (partly
    //    written lines, single bytes), so they should be few and small;
    //  - down to 8 KiB, while the workgroups would get fewer than four slabs each,
    //    and down to 4 KiB, while there are fewer slabs than workgroups: a medium
    //    message is then spread over more compute units, each step of its chains
    //    moving less per workgroup;
    //  - down to 4 KiB, while chunks are not a whole number of slabs, the workgroups
    //    get 4 to 15 slabs each, and the lines in which chunks meet are walked apart
    //    from the slabs (see launch_with): slabs in which two chunks meet do not take
    //    turns, and smaller ones cost less (30 MB on 16, 64, 256 ranks: 6, 5, 3 % less).
    int tl = pa.slab_log2;
    uint64_t grid64 = wgs_at_plan_tile;
    while (tl > kMinSlabLog2) {
        const uint64_t slab = 1ull << tl;
        const uint64_t n_slabs = (pa.n + slab - 1) >> tl;
        const bool too_long = slab > pa.ss;
        const bool many_cuts = tl > kFillSlabLog2 && pa.ss % slab != 0 && slab * 4 > pa.ss;
        const bool too_few = (tl > kFillSlabLog2 + 1 && n_slabs < 4 * grid64) ||
                             (tl > kFillSlabLog2 && n_slabs < grid64);
        const bool ragged_mid = tl > kFillSlabLog2 && (uint32_t)pa.P - 1u <= wgs_at_plan_tile &&
                                pa.ss % slab != 0 && n_slabs >= 4 * grid64 && n_slabs < 16 * grid64;
        if (!too_long && !many_cuts && !too_few && !ragged_mid) break;
        --tl;
        grid64 *= 2;
    }
    if (workgroups) *workgroups = grid64;
    return tl;
}

hipError_t launch_ring_chain(const PlanArrays &pa, uint32_t wgs_at_plan_tile, int first_step,
                             int last_step, bool from_tables, hipStream_t stream) {
    if (pa.algo != kAlgoNative && pa.algo != kAlgoTuned) return hipErrorInvalidValue;
    if (!from_tables && pa.P > kInlineMaxRanks) return hipErrorInvalidValue;
    return from_tables ? launch_with<TableHops>(pa, wgs_at_plan_tile, first_step, last_step, stream)
                       : launch_with<InlineHops>(pa, wgs_at_plan_tile, first_step, last_step, stream);
}

}  // namespace vbcast
