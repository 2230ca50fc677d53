/*
 * vbcast - the large-message MPI broadcast (binomial scatter followed by a ring
 * allgather) of P virtual ranks whose buffers all live in one GPU's memory.
 *
 * The library follows MPI_Bcast(buffer, count, datatype, root, comm) as the
 * paper's MPI_Bcast_native / MPI_Bcast_opt use it [Sec. I; Sec. IV, listing]:
 *   - comm      -> a virtual communicator: P device buffers, one per rank;
 *   - buffer    -> implicit, rank r broadcasts into / out of its own buffer;
 *   - datatype  -> its size in bytes; the message is n = count * dtype_size bytes
 *                  of opaque data (the paper sends MPI_BYTE);
 *   - root      -> absolute rank whose buffer holds the message on entry.
 * After bcast_run has completed on its stream, the first n bytes of every
 * rank's buffer equal the root's [Sec. III-A]; bytes at offsets >= n are never
 * touched.
 *
 * Two schedules are the subject of the paper [Sec. III-A and Sec. IV]:
 *   VBCAST_NATIVE  scatter + "enclosed" ring: every rank sends and receives one
 *                  chunk in each of the P-1 ring steps;
 *   VBCAST_TUNED   scatter + "non-enclosed" ring: a rank stops receiving once it
 *                  holds the whole message and its left neighbour stops sending
 *                  to it; same number of steps, fewer bytes.
 * Two more are the neighbouring algorithms of the same MPI_Bcast, which the paper
 * names [Abstract, Sec. I] and which complete the selection by message size and
 * process count (vbcast_select_algo):
 *   VBCAST_BINOMIAL     the whole message goes down the binomial tree, one level
 *                       per step (short messages);
 *   VBCAST_SCATTER_RDB  scatter, then log2 P exchanges in which a rank swaps all
 *                       it has gathered with the rank whose relative rank differs
 *                       in one bit (medium messages, power-of-two P only).
 *
 * A schedule is a list of steps: ceil(log2 P) scatter levels, then P-1 ring
 * steps (or log2 P exchanges; the binomial broadcast is ceil(log2 P) tree levels
 * and has no scatter).  A step is a table of rows (src rank, dst rank, byte offset, byte
 * length), ordered by the sender's rank relative to the root; a row means
 * "copy length bytes at that offset from src's buffer to the same offset in
 * dst's buffer".  Rows with length 0 are not stored.  All rows of a step are
 * independent; steps must run in order.  Tables are generated on the GPU.
 * The default executor of the two scatter + ring schedules copies the same rows
 * without going step by step: one kernel carries every piece of every chunk
 * through its transfers in the order they depend on each other, and for all but
 * long broadcasts it derives those rows itself instead of reading the tables
 * (vbcast_set_ring_executor, vbcast_set_chain_schedule).
 *
 * Conventions
 *   - All functions return 0 (VBCAST_SUCCESS) or a VBCAST_ERR_* code; nothing
 *     is thrown or printed.  bcast_strerror() gives a text; for VBCAST_ERR_HIP
 *     it includes the HIP runtime's own message for the calling thread's last
 *     failure.
 *   - "host pointer" / "device pointer" is stated per argument.  Streams are
 *     hipStream_t passed as void* (NULL = the default stream).
 *   - Argument checks happen before any GPU call, so invalid arguments are
 *     rejected without touching a device.
 *   - The library owns what it creates (communicator, plan, tables, graph) and
 *     nothing else: it never allocates, frees or initialises a rank buffer.
 *   - Not thread-safe per object: do not use one communicator or plan from two
 *     threads at once.  Two runs that overlap in time on the same rank buffers
 *     race.
 */
#ifndef VBCAST_H
#define VBCAST_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct vbcast_comm vbcast_comm; /* P virtual ranks = P device buffers */
typedef struct vbcast_plan vbcast_plan; /* tables, tile maps, instantiated graph */

enum {
    VBCAST_NATIVE = 0,      /* scatter + native ring allgather            */
    VBCAST_TUNED = 1,       /* scatter + tuned ring allgather             */
    VBCAST_BINOMIAL = 2,    /* binomial-tree broadcast of the whole message */
    VBCAST_SCATTER_RDB = 3  /* scatter + recursive-doubling allgather, power-of-two P */
};

/* Message-size classes of MPICH's broadcast [Sec. V]. */
#define VBCAST_SHORT_MSG_BYTES 12288  /* below: short message        */
#define VBCAST_LONG_MSG_BYTES 524288  /* from here on: long message  */

/* How bcast_run executes the ring phase (see vbcast_set_ring_executor). */
enum { VBCAST_RING_STEPS = 0, VBCAST_RING_CHAINS = 1 };

/* Where the one-launch executor takes its schedule from (see vbcast_set_chain_schedule). */
enum { VBCAST_CHAIN_AUTO = 0, VBCAST_CHAIN_INLINE = 1, VBCAST_CHAIN_TABLES = 2 };

enum {
    VBCAST_SUCCESS = 0,
    VBCAST_ERR_ARG = 1,   /* null pointer, P < 1, bad algo, bad step range, bad option */
    VBCAST_ERR_ROOT = 2,  /* root outside [0, P) */
    VBCAST_ERR_COUNT = 3, /* count * dtype_size overflows or exceeds the rank buffers */
    VBCAST_ERR_ALIGN = 4, /* a rank buffer is not 16-byte aligned */
    VBCAST_ERR_HIP = 5,   /* a HIP runtime call failed */
    VBCAST_ERR_NOMEM = 6, /* host or device allocation failed */
    VBCAST_ERR_LIMIT = 7  /* more ranks than the static tables of bcast_run_static hold */
};

/* Largest communicator accepted (tables grow with P * P). */
#define VBCAST_MAX_RANKS 8192

/*
 * Create a communicator of P ranks [Sec. III-A: the P processes of the broadcast].
 *   rank_bufs  host array of P device pointers; rank r's buffer.  Every pointer
 *              must be 16-byte aligned so that a copy at equal offsets in two
 *              buffers is equally aligned on both sides.  Buffers must not
 *              overlap (not checked).  The array is copied; the buffers stay
 *              the caller's and must outlive the communicator's use.
 *   buf_bytes  usable size of every rank buffer.
 *   out        host pointer receiving the handle.
 * Errors: ARG (P < 1, P > VBCAST_MAX_RANKS, null), ALIGN, HIP, NOMEM.
 */
int vbcast_comm_create(int P, void *const *rank_bufs, size_t buf_bytes, vbcast_comm **out);

/* Destroy a communicator.  Plans made from it must be destroyed first. */
int vbcast_comm_destroy(vbcast_comm *comm);

/*
 * Generate the schedule of one broadcast on the GPU [Sec. IV, listing]:
 * chunk size ceil(n / P) and chunk extents in relative-rank order, every rank's
 * relative rank, ring neighbours and tuned switch point (step, flag), the
 * scatter-level tables [Sec. III-A, Figs. 1-2], the ring-step tables
 * [Sec. III-A Fig. 3 for NATIVE; Sec. IV Figs. 4-5 for TUNED], and for every
 * step the map from copy tiles to rows.  Where bcast_run is to go step by step
 * (VBCAST_RING_STEPS, and the algorithms that have no other way), then record
 * one graph that holds the table-generation kernels followed by the copy
 * kernels.
 *   comm        communicator; must outlive the plan.  The device that was current
 *               when it was created must be current now (ARG otherwise).
 *   count, dtype_size   message = count * dtype_size bytes; 0 is valid.
 *   root        absolute rank in [0, P).
 *   algo        VBCAST_NATIVE, VBCAST_TUNED, VBCAST_BINOMIAL or VBCAST_SCATTER_RDB
 *               (the last one needs a power-of-two P: ARG otherwise).
 *   hip_stream  stream the generation kernels run on; the call synchronises
 *               this stream before it returns (it reads per-step counts back).
 *   out         host pointer receiving the handle.
 * Errors: ARG, ROOT, COUNT, HIP, NOMEM.  P = 1 and n = 0 give valid plans that
 * move nothing.
 */
int bcast_plan(const vbcast_comm *comm, size_t count, size_t dtype_size, int root, int algo,
               void *hip_stream, vbcast_plan **out);

/*
 * Run the whole broadcast [Sec. IV, listing: scatter, then ring] on hip_stream
 * and return without waiting (MPI's "blocking" is the caller's stream
 * synchronisation).  With the one-launch executor (VBCAST_RING_CHAINS; native
 * and tuned plans) these are plain kernel launches: one, where the kernel works
 * its schedule out itself - it derives every chunk's path through the scatter
 * tree and the ring from (P, root, n, schedule) while it copies, and no table is
 * read (VBCAST_CHAIN_INLINE, which VBCAST_CHAIN_AUTO picks for all but long
 * broadcasts) - or three, the two table kernels and then the copy kernel that
 * looks the schedule up.  Otherwise it launches the plan's graph, which
 * regenerates the tables on the device, then executes the scatter levels in
 * order and then the ring steps, one kernel per step (see
 * vbcast_set_ring_executor and vbcast_set_chain_schedule).
 * Errors: ARG (null), HIP.
 */
int bcast_run(const vbcast_plan *plan, void *hip_stream);

/* Largest communicator bcast_run_static accepts. */
#define VBCAST_STATIC_MAX_RANKS 513

/*
 * One whole broadcast without any allocation: for callers that cannot allocate
 * device memory at the point of the call (code under stream capture into a graph,
 * tight serving loops, harnesses that forbid allocation).  It does what
 * bcast_plan followed by bcast_run does with the one-launch executor
 * (VBCAST_RING_CHAINS) - table generation on the device, then scatter and ring
 * in one launch - but keeps the tables in a fixed 10 MiB array that is part of
 * the library's device code (every GPU the library runs on holds its own copy
 * until the process ends) instead of a per-plan allocation, and creates no plan
 * object, graph, stream or event.  The call makes no hipMalloc, hipFree or other
 * allocating call; it enqueues three kernels on hip_stream and returns without
 * waiting.  Afterwards the rank buffers hold what bcast_run leaves.
 *   comm        communicator (created beforehand; vbcast_comm_create is the set-up
 *               step that allocates and that looks up the table array's address on
 *               the device); its device must be current.  At most
 *               VBCAST_STATIC_MAX_RANKS ranks.
 *   count, dtype_size, root   as in bcast_plan; any message size the rank buffers
 *               hold (the tables grow with the number of ranks only).
 *   algo        VBCAST_NATIVE or VBCAST_TUNED.
 * All calls on one GPU share the one table array, which keeps the previous call's
 * contents (every entry a call reads it has written itself first): calls on the
 * same stream are ordered and safe; calls that overlap in time on one GPU (other
 * streams, other threads) race.  The chain-slab and workgroups-per-CU settings
 * apply as they do to plans.
 * Errors: ARG (null, other algo, other device current), LIMIT (more than
 * VBCAST_STATIC_MAX_RANKS ranks), ROOT, COUNT, HIP.
 */
int bcast_run_static(const vbcast_comm *comm, size_t count, size_t dtype_size, int root, int algo,
                     void *hip_stream);

/*
 * Run steps [first, last) only, as plain kernel launches on hip_stream (no
 * graph, tables as they are in device memory), asynchronously.  Used to look at
 * the state between steps.  Steps count scatter levels first [Sec. III-A: one
 * level of the binomial tree], then ring steps [Sec. IV, listing: one iteration
 * i of the loop over comm_size - 1 exchanges, i.e. one send to the right
 * neighbour and one receive from the left per rank, or only one of the two for a
 * rank past its switch point].
 * Errors: ARG (null, first < 0, first > last, last > n_steps), HIP.
 */
int bcast_run_steps(const vbcast_plan *plan, int first, int last, void *hip_stream);

/*
 * Steps [first, last) executed by the kernel of the one-launch executor
 * (VBCAST_RING_CHAINS) in a single launch on hip_stream, asynchronously: every
 * piece of every chunk is carried through the transfers the tables hold for it
 * in those steps, in order [Sec. III-A: a rank passes on what it received one
 * step earlier].  The state of the rank buffers after step first - 1 must be in
 * place (the root's message for first = 0); afterwards they hold the state after
 * step last - 1, the same as after bcast_run_steps(first, last).  With first = 0
 * and last = n_steps this is the launch bcast_run makes (the plan's schedule
 * source, see vbcast_set_chain_schedule, applies here too).  VBCAST_NATIVE and
 * VBCAST_TUNED plans only.
 * Errors: ARG (null, other algorithm, first < 0, first > last, last > n_steps),
 * HIP.
 */
int bcast_run_chain_steps(const vbcast_plan *plan, int first, int last, void *hip_stream);

/*
 * As bcast_run_steps, but brackets every step's kernel with events recorded on
 * hip_stream, waits for the last one and writes the elapsed milliseconds of
 * step first + i to step_ms[i] (host array of last - first floats; 0 for a step
 * that moves nothing).  Synchronous.
 */
int bcast_run_steps_timed(const vbcast_plan *plan, int first, int last, void *hip_stream,
                          float *step_ms);

/*
 * Run the whole broadcast once as plain launches (no graph) with events recorded
 * on hip_stream between its three phases, wait, and write the elapsed
 * milliseconds to phase_ms[0..2] (host array): table generation, scatter levels,
 * the steps after the scatter - executed the way bcast_run executes them: with
 * VBCAST_RING_CHAINS the scatter is part of the one launch, so phase_ms[1] is
 * (close to) 0 and phase_ms[2] covers scatter and ring, and with
 * VBCAST_CHAIN_INLINE no table kernel runs either, so phase_ms[0] is (close to)
 * 0 too.  Synchronous.
 * Errors: ARG (null), HIP.
 */
int bcast_run_timed(const vbcast_plan *plan, void *hip_stream, float *phase_ms);

typedef struct vbcast_plan_info {
    int32_t P, root, algo;
    int32_t n_scatter_steps; /* ceil(log2 P); 0 for VBCAST_BINOMIAL */
    int32_t n_steps;         /* scatter steps + P - 1 ring steps (or log2 P exchanges, or
                                ceil(log2 P) tree levels); 0 for P = 1 */
    int32_t tile_bytes;      /* copy tile size the plan was built for */
    uint64_t n;              /* message bytes */
    uint64_t ss;             /* chunk size ceil(n / P) */
    uint64_t scatter_rows, ring_rows;   /* stored rows (length > 0); "ring" = every step
                                           after the scatter, whatever the algorithm */
    uint64_t scatter_bytes, ring_bytes; /* bytes moved, one direction */
    uint64_t bytes_moved;               /* scatter_bytes + ring_bytes */
    uint64_t ring_msgs_issued; /* sends the ranks post after the scatter, zero-length ones included
                                  [Sec. III-A: P (P - 1) native; Sec. IV: fewer tuned] */
    uint64_t pairing_mismatches; /* ring (step, rank) pairs where the sender's and the
                                    receiver's own decisions disagree; always 0 */
    uint64_t n_tiles;            /* copy tiles over all steps */
    uint64_t run_launches;       /* kernels one bcast_run runs: 1 when the one-launch executor
                                    works its schedule out itself, 3 when it looks it up, else
                                    the table kernels plus one copy kernel per step (a graph) */
} vbcast_plan_info;

/* Fill *info (host pointer) from the counts read back at plan time. */
int bcast_plan_info(const vbcast_plan *plan, vbcast_plan_info *info);

/*
 * Copy the step tables to the host (synchronous copies; the caller makes sure no
 * launch of this plan is still running).  Any output may be NULL.  A row is one
 * message of the schedule: for a ring step the sender, its right neighbour, and
 * the displacement and count the sender computes for that iteration [Sec. IV,
 * listing: right_disp / right_count, equal to the receiver's left_disp /
 * left_count]; for a scatter level the subtree root, the rank it hands the upper
 * half of its chunks to, and that range as one extent [Sec. III-A].
 *   step_ptr    n_steps + 1 entries; rows of step s are [step_ptr[s], step_ptr[s+1])
 *   src, dst    one entry per row: absolute ranks
 *   off, len    one entry per row: byte offset and length
 *   step_bytes  n_steps entries: bytes moved by the step
 * Row arrays need room for scatter_rows + ring_rows entries.
 */
int bcast_plan_export(const vbcast_plan *plan, uint64_t *step_ptr, uint32_t *src, uint32_t *dst,
                      uint64_t *off, uint64_t *len, uint64_t *step_bytes);

/*
 * Copy the chunk and rank descriptors to the host (synchronous); any output may
 * be NULL [Sec. IV, listing].
 *   chunk_off  P + 1 entries: running sum of the chunk lengths (entry P = n)
 *   chunk_len  P entries: clamp(n - c * ss, 0, ss) for relative chunk index c
 *   rel, left, right   P entries each, by absolute rank: relative rank and ring
 *                      neighbours
 *   sw_step, sw_flag   P entries each, by absolute rank: the tuned ring's switch
 *                      point; flag 1 = receive-only tail, 0 = send-only tail;
 *                      both -1 when P = 1
 */
int bcast_plan_export_desc(const vbcast_plan *plan, uint64_t *chunk_off, uint64_t *chunk_len,
                           int32_t *rel, int32_t *left, int32_t *right, int32_t *sw_step,
                           int32_t *sw_flag);

/*
 * Copy one step's tile map to the host (synchronous): tile t of the step copies
 * the part of row tile_row[t] that lies in the tile_idx[t]-th tile_bytes-aligned
 * window the row touches.  Arrays need *n_tiles entries; call with NULL arrays to
 * get the count first.
 */
int bcast_plan_export_tiles(const vbcast_plan *plan, int step, uint32_t *n_tiles,
                            uint32_t *tile_row, uint32_t *tile_idx);

/*
 * Copy the chunk-major "chain" view to the host (VBCAST_NATIVE / VBCAST_TUNED
 * plans only; ARG otherwise): for the chunk with relative index c and step s,
 * holder[c * n_steps + s] is the absolute rank whose buffer holds the chunk
 * after step s on the chunk's own path (down the scatter tree, then round the
 * ring), and moves[c * n_steps + s] is 1 if step s has a row that copies the
 * chunk there, 0 if not (the chunk is not on a tree edge at that level, the
 * tuned ring dropped the transfer, or the chunk is empty).  This is the table
 * the one-launch executor walks.  Arrays need P * n_steps entries; either may be
 * NULL.  Synchronous.
 */
int bcast_plan_export_chain(const vbcast_plan *plan, int32_t *holder, uint8_t *moves);

typedef struct vbcast_census {
    uint64_t scatter_inter_msgs, scatter_inter_bytes; /* scatter rows between nodes   */
    uint64_t scatter_intra_msgs, scatter_intra_bytes; /* scatter rows inside a node   */
    uint64_t ring_inter_msgs, ring_inter_bytes;       /* later steps, between nodes   */
    uint64_t ring_intra_msgs, ring_intra_bytes;       /* later steps, inside a node   */
} vbcast_census;

/*
 * Count, on the GPU, the stored rows (length > 0) of the plan that would cross a
 * node boundary, and their bytes, if the P ranks were MPI processes placed on
 * nodes in blocks of ranks_per_node (rank r on node r / ranks_per_node) - the
 * placement of the paper's measurements, 24 processes per node [Sec. V, V-A]; the
 * paper explains its gains at 64 and 256 processes by the smaller number of
 * inter-node messages.  Runs on hip_stream and waits for it.  *out is a host
 * pointer.  Errors: ARG (null, ranks_per_node < 1), HIP.
 */
int bcast_plan_census(const vbcast_plan *plan, int ranks_per_node, void *hip_stream,
                      vbcast_census *out);

int bcast_plan_destroy(vbcast_plan *plan);

/*
 * The multi-core-aware broadcast the paper describes for medium messages on a
 * non-power-of-two process count [Sec. I]: (1) a binomial broadcast among the
 * ranks of the root's node, (2) the scatter-ring-allgather among one rank per
 * node, (3) a binomial broadcast inside every other node.  The paper describes
 * it in one sentence and does not implement it; where that sentence is silent:
 * ranks sit on nodes in blocks of ranks_per_node [Sec. V-A], a node's
 * representative is its lowest rank, and phase 2 starts from the root node's
 * representative.  The plan is a sequence of ordinary plans over
 * sub-communicators (subsets of comm's rank buffers), chained in one graph.
 *   ring_algo   VBCAST_NATIVE or VBCAST_TUNED for phase 2.
 * Errors: ARG (null, ranks_per_node < 1, other ring_algo), ROOT, COUNT, HIP, NOMEM.
 */
typedef struct vbcast_smp_plan vbcast_smp_plan;
int bcast_plan_smp(const vbcast_comm *comm, size_t count, size_t dtype_size, int root,
                   int ranks_per_node, int ring_algo, void *hip_stream, vbcast_smp_plan **out);

/* Launch the whole three-phase broadcast (one graph) on hip_stream; asynchronous. */
int bcast_run_smp(const vbcast_smp_plan *plan, void *hip_stream);

/* Run the sub-plans of one phase (1, 2 or 3) as plain launches on hip_stream,
 * asynchronously; used to look at the state between phases.  ARG for other phases. */
int bcast_run_smp_phase(const vbcast_smp_plan *plan, int phase, void *hip_stream);

/*
 * The sub-plans in execution order: *count (host pointer) receives their number
 * when sub is NULL; otherwise sub-plan `index` is returned in *sub (owned by the
 * three-phase plan; valid until it is destroyed), its phase in *phase, and the
 * absolute ranks of its sub-communicator, in that communicator's rank order, in
 * members[0 .. *n_members) (host array with room for P entries; may be NULL).
 */
int bcast_smp_subplan(const vbcast_smp_plan *plan, int index, int *count, const vbcast_plan **sub,
                      int *phase, int *n_members, int *members);

int bcast_plan_smp_destroy(vbcast_smp_plan *plan);

/*
 * The algorithm MPICH's broadcast takes for nbytes on P processes, as the paper
 * states it [Abstract; Sec. I; thresholds in Sec. V]: short messages (below
 * VBCAST_SHORT_MSG_BYTES) -> VBCAST_BINOMIAL; medium messages on a power-of-two P
 * -> VBCAST_SCATTER_RDB; long messages (from VBCAST_LONG_MSG_BYTES) and medium
 * messages on any other P -> scatter + ring allgather: VBCAST_TUNED if `tuned` is
 * non-zero, else VBCAST_NATIVE.  Host only, no GPU call.  *algo is a host pointer.
 * Errors: ARG (null, P < 1).
 */
int vbcast_select_algo(size_t nbytes, int P, int tuned, int *algo);

/*
 * Copy-tile size of the per-step executor (and of the tile maps) used by plans
 * created afterwards: a power of two between 4096 and 65536 bytes (default
 * 16384).  Process-wide; returns ARG for other values.
 */
int vbcast_set_tile_bytes(size_t tile_bytes);

/*
 * Slab size of the one-launch executor (VBCAST_RING_CHAINS) for plans created
 * afterwards: a power of two between 4096 and 65536 bytes (default 16384).  The
 * launch uses a smaller slab (down to 1024 bytes) when chunks are shorter than
 * this, or hold fewer than four slabs without being a whole number of them, and
 * down to 4096 bytes when the message has fewer slabs than there are resident
 * workgroups.  Process-wide; returns ARG for other values.
 */
int vbcast_set_chain_slab_bytes(size_t slab_bytes);

/*
 * How bcast_run of plans created afterwards executes the scatter levels and the
 * P-1 ring steps [Sec. III-A: a subtree root passes on part of what it received;
 * a rank forwards in ring step i+1 the chunk it received in step i]:
 *   VBCAST_RING_STEPS   one copy kernel per step, in step order, all in one graph;
 *                       every step is complete before the next starts.
 *   VBCAST_RING_CHAINS  (default) one launch for the scatter and the ring together:
 *                       every piece of every chunk is carried down its path in the
 *                       scatter tree and then through its P-1 ring transfers, in
 *                       order and independently of the other pieces - the ordering
 *                       MPI's blocking point-to-point calls impose, without a
 *                       barrier between steps.  The same rows are copied, source
 *                       to destination through memory, and the final state is
 *                       the same; there is no global "state after step i" while
 *                       it runs.  (Applies to VBCAST_NATIVE and VBCAST_TUNED; the
 *                       other algorithms always run step by step.)
 * bcast_run_steps always runs whole steps.  Process-wide; ARG for other values.
 */
int vbcast_set_ring_executor(int mode);

/*
 * Where the one-launch executor (VBCAST_RING_CHAINS) of plans created afterwards
 * learns which buffer a chunk is copied to in each step, and which steps skip it:
 *   VBCAST_CHAIN_INLINE  the copy kernel computes it from the chunk index: the
 *                        chunk's path down the binomial tree [Sec. III-A], its P-1
 *                        ring transfers, and for the tuned schedule the step from
 *                        which the receiving rank no longer receives [Sec. IV].
 *                        No table is read; bcast_run is that one kernel launch.
 *                        Up to 1024 ranks (the kernel keeps the
 *                        hops of the chunks it is busy with in LDS); larger
 *                        communicators use VBCAST_CHAIN_TABLES whatever is set.
 *   VBCAST_CHAIN_TABLES  the kernel looks it up in the chunk-major view of the step
 *                        tables; bcast_run launches the two table kernels and then
 *                        the copy kernel.  bcast_run_static always works this way.
 *   VBCAST_CHAIN_AUTO    (default) INLINE, except for long broadcasts - slabs of
 *                        16 KiB or more, and a resident workgroup has 4096 or more
 *                        steps to go through (its share of the message's slabs
 *                        times the steps of the schedule) -
 *                        which use TABLES: the two table kernels no longer count
 *                        there, and the lookups - scalar loads that miss their
 *                        cache and come back after one trip to the L2 - keep a
 *                        workgroup from issuing steps faster than the L2 answers,
 *                        which measures a few per cent faster once every compute
 *                        unit has been streaming for a while.
 * All copy the same rows.  Process-wide; ARG for other values.
 */
int vbcast_set_chain_schedule(int mode);

/* Resident workgroups per compute unit for VBCAST_RING_CHAINS (1..16, default 1);
 * together with the slab size this sets how many bytes are in flight at once. */
int vbcast_set_chain_workgroups_per_cu(int k);

/*
 * Number of accelerator dies (XCDs) the copy kernels assume when they map
 * workgroups to pieces of the message, for communicators created afterwards:
 * the hardware deals workgroup b to die b mod n_xcd, and the kernels give every
 * die a contiguous share of the work so that its addresses spread over all
 * channels of its own L2.  0 (default) = ask the device (8 on the unpartitioned
 * part; 8 is also assumed when the device does not say).  Any value gives the
 * same results - the mapping is a permutation of the pieces - only the speed
 * differs.  1..64 or 0; ARG otherwise.  Process-wide.
 */
int vbcast_set_xcd_count(int n_xcd);

/* Text for an error code; never NULL.  The pointer is valid until the calling
 * thread's next library call. */
const char *bcast_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* VBCAST_H */
