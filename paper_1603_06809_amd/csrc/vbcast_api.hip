// Host side of libvbcast: argument checks, device allocations for the plan,
// the graph that chains table generation and the per-step copy kernels, and
// the exports.  See include/vbcast.h for the contract of every entry point.

#include "../../include/vbcast.h"
#include "vbcast_internal.h"

#include <atomic>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <type_traits>
#include <unordered_map>
#include <vector>

using vbcast::PlanArrays;
using vbcast::Row;
using vbcast::Tile;

struct vbcast_comm {
    int P = 0;
    size_t buf_bytes = 0;
    int device = 0;
    int compute_units = 256;  // of `device`, read once at creation
    int n_xcd = 8;            // accelerator dies of `device` (workgroups are dealt to them round-robin)
    std::vector<void *> host_bases;
    uint8_t **dev_bases = nullptr;
};

struct vbcast_plan {
    const vbcast_comm *comm = nullptr;
    PlanArrays pa{};
    void *arena = nullptr;  // one device allocation holding every plan array
    // per-step counts, read back once at plan time
    std::vector<uint32_t> step_rows, step_tiles, step_posted, step_mismatch;
    std::vector<uint64_t> step_bytes;
    int ring_executor = VBCAST_RING_CHAINS;  // what bcast_run uses for the ring phase
    bool chain_from_tables = false;          // one-launch executor: hops looked up, not derived
    uint32_t chain_grid = 0;                 // workgroups of the one-launch ring
    hipGraph_t graph = nullptr;
    hipGraphExec_t exec = nullptr;
};

struct vbcast_smp_plan {
    struct Sub {
        int phase = 0;
        std::vector<int> members;       // absolute ranks, in the sub-communicator's order
        vbcast_comm *comm = nullptr;
        vbcast_plan *plan = nullptr;
    };
    std::vector<Sub> subs;              // execution order
    hipGraph_t graph = nullptr;
    hipGraphExec_t exec = nullptr;
};

static_assert(vbcast::kAlgoNative == VBCAST_NATIVE && vbcast::kAlgoTuned == VBCAST_TUNED &&
                  vbcast::kAlgoBinomial == VBCAST_BINOMIAL &&
                  vbcast::kAlgoScatterRdb == VBCAST_SCATTER_RDB,
              "kernel-side algorithm codes must match the public header");

namespace {

thread_local std::string g_hip_msg;
thread_local std::string g_text;
std::atomic<int> g_tile_log2{14};
std::atomic<int> g_slab_log2{14};
std::atomic<int> g_ring_executor{VBCAST_RING_CHAINS};
std::atomic<int> g_chain_schedule{VBCAST_CHAIN_AUTO};
std::atomic<int> g_chain_wgs_per_cu{1};
std::atomic<int> g_xcd_override{0};  // 0 = ask the device

int hip_fail(hipError_t e, const char *what) {
    g_hip_msg = std::string(what) + ": " + hipGetErrorString(e);
    (void)hipGetLastError();  // clear the sticky slot
    return VBCAST_ERR_HIP;
}

#define HIP_TRY(call)                                        \
    do {                                                     \
        hipError_t e_ = (call);                              \
        if (e_ != hipSuccess) return hip_fail(e_, #call);    \
    } while (0)

int ceil_log2_int(int P) {
    int k = 0;
    while ((1 << k) < P) ++k;
    return k;
}

struct ArenaLayout {
    size_t total = 0;
    size_t take(size_t bytes) {
        const size_t at = total;
        total += (bytes + 255) & ~size_t(255);
        return at;
    }
};

// Places every plan array of `pa` (P, L, n_steps, algo and tile_cap already set)
// one after the other from `base`, each on a 256-byte boundary, and returns the
// bytes they take together; with base == nullptr it only measures.  Without
// `tile_maps` the tile maps and the census sums (needed by the per-step executor
// and bcast_plan_census only) get no room and stay null.
size_t bind_plan_arrays(PlanArrays &pa, char *base, bool tile_maps) {
    const size_t S = (size_t)pa.n_steps, Pz = (size_t)pa.P;
    const bool ring_algo = pa.algo == VBCAST_NATIVE || pa.algo == VBCAST_TUNED;
    ArenaLayout lay;
    auto place = [&](auto *&field, size_t bytes) {
        const size_t at = lay.take(bytes);
        using T = std::remove_reference_t<decltype(field)>;
        field = (base && bytes) ? reinterpret_cast<T>(base + at) : nullptr;
    };
    place(pa.chunk_off, sizeof(uint64_t) * (Pz + 1));
    place(pa.chunk_len, sizeof(uint64_t) * Pz);
    place(pa.rel, sizeof(int32_t) * Pz);
    place(pa.left, sizeof(int32_t) * Pz);
    place(pa.right, sizeof(int32_t) * Pz);
    place(pa.sw_step, sizeof(int32_t) * Pz);
    place(pa.sw_flag, sizeof(int32_t) * Pz);
    place(pa.rows, sizeof(Row) * S * Pz);
    place(pa.chain, ring_algo ? sizeof(uint64_t) * Pz * ((size_t)pa.L + Pz - 1) : 0);
    place(pa.tile_ptr, sizeof(uint32_t) * S * (Pz + 1));
    place(pa.tiles, tile_maps ? sizeof(Tile) * S * (size_t)pa.tile_cap : 0);
    place(pa.step_rows, sizeof(uint32_t) * S);
    place(pa.step_tiles, sizeof(uint32_t) * S);
    place(pa.step_posted, sizeof(uint32_t) * S);
    place(pa.step_mismatch, sizeof(uint32_t) * S);
    place(pa.step_bytes, sizeof(uint64_t) * S);
    place(pa.census, tile_maps ? sizeof(uint64_t) * 4 * S : 0);
    return lay.total;
}

// ---------------------------------------------------------------------------
// bcast_run_static: the tables of one broadcast in memory that exists without any
// allocation - a file-scope device array, present on every GPU the library runs
// on from the moment its code is loaded until the process ends.
//
// In host code the array's name stands for the symbol, not for a device address:
// the address on a given GPU comes from hipGetSymbolAddress, asked once per
// device with that device current (every GPU has its own copy at its own
// address), and only that pointer is ever handed to a kernel.
// ---------------------------------------------------------------------------
constexpr size_t kScratchBytes = size_t(10) << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};

// The address of `scratch` on `device`, which must be the current device.
int scratch_on_device(int device, void **out) {
    if (device < 0 || device >= kMaxDevices) return VBCAST_ERR_ARG;
    std::lock_guard<std::mutex> hold(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        void *p = nullptr;
        hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return hip_fail(e, "hipGetSymbolAddress(scratch)");
        if (!p) {
            g_hip_msg = "hipGetSymbolAddress(scratch) gave no address";
            return VBCAST_ERR_HIP;
        }
        g_scratch_ptr[device] = p;
    }
    *out = g_scratch_ptr[device];
    return VBCAST_SUCCESS;
}

void describe_plan(PlanArrays &pa, int P, int root, int algo, uint64_t n, int tile_log2,
                   uint32_t tile_cap) {
    pa.P = P;
    pa.root = root;
    pa.algo = algo;
    pa.L = ceil_log2_int(P);
    pa.n_scatter = algo == VBCAST_BINOMIAL ? 0 : pa.L;
    pa.n_steps = P <= 1 ? 0
                 : algo == VBCAST_BINOMIAL ? pa.L
                 : algo == VBCAST_SCATTER_RDB ? 2 * pa.L
                                              : pa.L + P - 1;
    pa.tile_log2 = tile_log2;
    pa.slab_log2 = g_slab_log2.load();
    pa.tile_cap = tile_cap;
    pa.n = n;
    pa.ss = (n + (uint64_t)P - 1) / (uint64_t)P;
}

int launch_steps(const vbcast_plan *plan, int first, int last, hipStream_t stream,
                 hipEvent_t *marks) {
    const PlanArrays &pa = plan->pa;
    for (int s = first; s < last; ++s) {
        if (marks) HIP_TRY(hipEventRecord(marks[s - first], stream));
        const uint32_t nt = plan->step_tiles[s];
        if (nt == 0) continue;
        HIP_TRY(vbcast::launch_step_copy(pa.rows + (size_t)s * pa.P,
                                         pa.tiles + (size_t)s * pa.tile_cap,
                                         plan->comm->dev_bases, nt, pa.tile_log2, pa.n_xcd, stream));
    }
    if (marks) HIP_TRY(hipEventRecord(marks[last - first], stream));
    return VBCAST_SUCCESS;
}

bool one_launch(const vbcast_plan *plan) {
    const int a = plan->pa.algo;
    return (a == VBCAST_NATIVE || a == VBCAST_TUNED) && plan->ring_executor == VBCAST_RING_CHAINS;
}

// The whole broadcast is one kernel that reads no table.
bool single_kernel(const vbcast_plan *plan) { return one_launch(plan) && !plan->chain_from_tables; }

// The scatter levels, the way bcast_run runs them: step by step, or not at all
// when the one-launch executor carries them together with the ring.
int launch_scatter(const vbcast_plan *plan, hipStream_t stream) {
    const PlanArrays &pa = plan->pa;
    if (pa.n_steps == 0 || one_launch(plan)) return VBCAST_SUCCESS;
    return launch_steps(plan, 0, pa.n_scatter, stream, nullptr);
}

// The steps after the scatter (with the one-launch executor: all steps), the way
// bcast_run runs them.
int launch_ring(const vbcast_plan *plan, hipStream_t stream) {
    const PlanArrays &pa = plan->pa;
    if (pa.n_steps == 0) return VBCAST_SUCCESS;
    if (one_launch(plan)) {
        hipError_t e = vbcast::launch_ring_chain(pa, plan->chain_grid, 0, pa.n_steps,
                                                 plan->chain_from_tables, stream);
        if (e != hipSuccess) return hip_fail(e, "ring chain kernel");
        return VBCAST_SUCCESS;
    }
    return launch_steps(plan, pa.n_scatter, pa.n_steps, stream, nullptr);
}

// Steps whose tile maps a broadcast rebuilds: all of them for the per-step executor;
// none for the one-launch executor, which reads the chain view if anything (the tile
// maps were built at plan time and serve bcast_run_steps).
int tile_map_steps(const vbcast_plan *plan) {
    const PlanArrays &pa = plan->pa;
    if (pa.n_steps == 0) return 0;
    return one_launch(plan) ? 0 : pa.n_steps;
}

// Everything one broadcast enqueues, in order: the table kernels (unless the copy
// kernel works the schedule out itself), the scatter levels, the ring phase.
int enqueue_broadcast(const vbcast_plan *plan, hipStream_t stream) {
    if (!single_kernel(plan)) {
        hipError_t e = vbcast::launch_plan_kernels(plan->pa, tile_map_steps(plan), stream);
        if (e != hipSuccess) return hip_fail(e, "plan kernels");
    }
    int rc = launch_scatter(plan, stream);
    if (rc == VBCAST_SUCCESS) rc = launch_ring(plan, stream);
    return rc;
}

int build_graph(vbcast_plan *plan) {
    // One to three launches are cheaper made directly than through a graph (about
    // 20 us per graph launch against 5 us per kernel launch, which overlap with the
    // kernels already queued): the one-launch executor has no graph.
    if (one_launch(plan)) return VBCAST_SUCCESS;
    hipStream_t cap = nullptr;
    HIP_TRY(hipStreamCreateWithFlags(&cap, hipStreamNonBlocking));
    hipError_t e = hipStreamBeginCapture(cap, hipStreamCaptureModeRelaxed);
    if (e != hipSuccess) {
        (void)hipStreamDestroy(cap);
        return hip_fail(e, "hipStreamBeginCapture");
    }
    const int rc = enqueue_broadcast(plan, cap);
    hipGraph_t graph = nullptr;
    e = hipStreamEndCapture(cap, &graph);
    (void)hipStreamDestroy(cap);
    if (rc != VBCAST_SUCCESS) {
        if (graph) (void)hipGraphDestroy(graph);
        return rc;
    }
    if (e != hipSuccess) return hip_fail(e, "hipStreamEndCapture");
    plan->graph = graph;
    HIP_TRY(hipGraphInstantiate(&plan->exec, graph, nullptr, nullptr, 0));
    return VBCAST_SUCCESS;
}

void free_plan(vbcast_plan *plan) {
    if (!plan) return;
    if (plan->exec) (void)hipGraphExecDestroy(plan->exec);
    if (plan->graph) (void)hipGraphDestroy(plan->graph);
    if (plan->arena) (void)hipFree(plan->arena);
    delete plan;
}

}  // namespace

extern "C" {

int vbcast_set_tile_bytes(size_t tile_bytes) {
    for (int k = 12; k <= 16; ++k)
        if (tile_bytes == (size_t(1) << k)) {
            g_tile_log2.store(k);
            return VBCAST_SUCCESS;
        }
    return VBCAST_ERR_ARG;
}

int vbcast_set_chain_slab_bytes(size_t slab_bytes) {
    for (int k = 12; k <= 16; ++k)
        if (slab_bytes == (size_t(1) << k)) {
            g_slab_log2.store(k);
            return VBCAST_SUCCESS;
        }
    return VBCAST_ERR_ARG;
}

int vbcast_set_ring_executor(int mode) {
    if (mode != VBCAST_RING_STEPS && mode != VBCAST_RING_CHAINS) return VBCAST_ERR_ARG;
    g_ring_executor.store(mode);
    return VBCAST_SUCCESS;
}

int vbcast_set_chain_schedule(int mode) {
    if (mode != VBCAST_CHAIN_AUTO && mode != VBCAST_CHAIN_INLINE && mode != VBCAST_CHAIN_TABLES)
        return VBCAST_ERR_ARG;
    g_chain_schedule.store(mode);
    return VBCAST_SUCCESS;
}

int vbcast_set_chain_workgroups_per_cu(int k) {
    if (k < 1 || k > 16) return VBCAST_ERR_ARG;
    g_chain_wgs_per_cu.store(k);
    return VBCAST_SUCCESS;
}

int vbcast_set_xcd_count(int n_xcd) {
    if (n_xcd < 0 || n_xcd > 64) return VBCAST_ERR_ARG;
    g_xcd_override.store(n_xcd);
    return VBCAST_SUCCESS;
}

int vbcast_comm_create(int P, void *const *rank_bufs, size_t buf_bytes, vbcast_comm **out) {
    if (!out) return VBCAST_ERR_ARG;
    *out = nullptr;
    if (!rank_bufs || P < 1 || P > VBCAST_MAX_RANKS) return VBCAST_ERR_ARG;
    for (int r = 0; r < P; ++r) {
        if (!rank_bufs[r]) return VBCAST_ERR_ARG;
        if (reinterpret_cast<uintptr_t>(rank_bufs[r]) & 15u) return VBCAST_ERR_ALIGN;
    }
    vbcast_comm *c = new (std::nothrow) vbcast_comm;
    if (!c) return VBCAST_ERR_NOMEM;
    c->P = P;
    c->buf_bytes = buf_bytes;
    c->host_bases.assign(rank_bufs, rank_bufs + P);
    hipError_t e = hipGetDevice(&c->device);
    if (e == hipSuccess) {
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, c->device) == hipSuccess &&
            cus > 0)
            c->compute_units = cus;
        else
            (void)hipGetLastError();
        int xcds = 0;
        if (g_xcd_override.load() > 0)
            c->n_xcd = g_xcd_override.load();
        else if (hipDeviceGetAttribute(&xcds, hipDeviceAttributeNumberOfXccs, c->device) == hipSuccess &&
                 xcds > 0 && c->compute_units % xcds == 0)
            c->n_xcd = xcds;
        else
            (void)hipGetLastError();   // not reported: keep 8, the full part's count
    }
    if (e == hipSuccess) {
        // set-up is also where the address of the static table memory on this device
        // is asked for, so that bcast_run_static itself only looks it up
        void *unused = nullptr;
        const int rc = scratch_on_device(c->device, &unused);
        if (rc != VBCAST_SUCCESS) {
            delete c;
            return rc;
        }
    }
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&c->dev_bases), sizeof(void *) * P);
    if (e == hipSuccess)
        e = hipMemcpy(c->dev_bases, c->host_bases.data(), sizeof(void *) * P, hipMemcpyHostToDevice);
    if (e != hipSuccess) {
        if (c->dev_bases) (void)hipFree(c->dev_bases);
        delete c;
        return e == hipErrorOutOfMemory ? VBCAST_ERR_NOMEM : hip_fail(e, "vbcast_comm_create");
    }
    *out = c;
    return VBCAST_SUCCESS;
}

int vbcast_comm_destroy(vbcast_comm *comm) {
    if (!comm) return VBCAST_ERR_ARG;
    hipError_t e = comm->dev_bases ? hipFree(comm->dev_bases) : hipSuccess;
    delete comm;
    if (e != hipSuccess) return hip_fail(e, "hipFree");
    return VBCAST_SUCCESS;
}

int bcast_plan(const vbcast_comm *comm, size_t count, size_t dtype_size, int root, int algo,
               void *hip_stream, vbcast_plan **out) {
    if (!out) return VBCAST_ERR_ARG;
    *out = nullptr;
    if (!comm) return VBCAST_ERR_ARG;
    if (algo < VBCAST_NATIVE || algo > VBCAST_SCATTER_RDB) return VBCAST_ERR_ARG;
    const int P = comm->P;
    if (algo == VBCAST_SCATTER_RDB && (P & (P - 1)) != 0) return VBCAST_ERR_ARG;
    if (root < 0 || root >= P) return VBCAST_ERR_ROOT;
    if (dtype_size != 0 && count > SIZE_MAX / dtype_size) return VBCAST_ERR_COUNT;
    const uint64_t n = (uint64_t)count * (uint64_t)dtype_size;
    if (n > comm->buf_bytes) return VBCAST_ERR_COUNT;
    const int tile_log2 = g_tile_log2.load();
    // Most bytes any one step moves: n for scatter levels and ring steps; the last
    // tree level of the binomial broadcast and the last recursive-doubling
    // exchange move P/2 messages' worth.
    const bool ring_algo = algo == VBCAST_NATIVE || algo == VBCAST_TUNED;
    const uint64_t per_step = ring_algo ? 1ull : (uint64_t)(P / 2 > 0 ? P / 2 : 1);
    if (n != 0 && per_step > (~0ull >> 1) / n) return VBCAST_ERR_COUNT;
    const uint64_t tile_cap64 = ((n * per_step) >> tile_log2) + 2ull * (uint64_t)P + 1ull;
    if (tile_cap64 >= (1ull << 31)) return VBCAST_ERR_COUNT;

    {
        // tables go next to the rank buffers: the communicator's device must be current
        int dev = -1;
        hipError_t de = hipGetDevice(&dev);
        if (de != hipSuccess) return hip_fail(de, "hipGetDevice");
        if (dev != comm->device) return VBCAST_ERR_ARG;
    }
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    vbcast_plan *plan = new (std::nothrow) vbcast_plan;
    if (!plan) return VBCAST_ERR_NOMEM;
    plan->comm = comm;
    PlanArrays &pa = plan->pa;
    describe_plan(pa, P, root, algo, n, tile_log2, (uint32_t)tile_cap64);
    pa.n_xcd = comm->n_xcd;

    const size_t S = (size_t)pa.n_steps;
    const size_t arena_bytes = bind_plan_arrays(pa, nullptr, /*tile_maps=*/true);

    hipError_t e = hipMalloc(&plan->arena, arena_bytes);
    if (e != hipSuccess) {
        delete plan;
        if (e == hipErrorOutOfMemory) {
            (void)hipGetLastError();
            return VBCAST_ERR_NOMEM;
        }
        return hip_fail(e, "hipMalloc(plan)");
    }
    (void)bind_plan_arrays(pa, static_cast<char *>(plan->arena), /*tile_maps=*/true);
    pa.bases = comm->dev_bases;
    plan->ring_executor = g_ring_executor.load();
    plan->chain_grid = (uint32_t)comm->compute_units * (uint32_t)g_chain_wgs_per_cu.load();
    {
        // AUTO: look the hops up when the launch walks slabs of 16 KiB or more (the
        // wavefronts of a workgroup then take turns, and the lookups pace them) and a
        // workgroup has 4096 or more steps to go through (its share of the slabs times
        // the steps of a slab; see vbcast_set_chain_schedule), else work them out
        const int mode = g_chain_schedule.load();
        uint64_t wgs = 0;
        const int tl = vbcast::chain_slab_log2(pa, plan->chain_grid, &wgs);
        const uint64_t slabs = (n + (uint64_t(1) << tl) - 1) >> tl;
        const uint64_t share = wgs ? (slabs + wgs - 1) / wgs : 0;
        const bool long_run = tl >= 14 && share * (uint64_t)pa.n_steps >= 4096;
        plan->chain_from_tables = mode == VBCAST_CHAIN_TABLES || P > vbcast::kInlineMaxRanks ||
                                  (mode == VBCAST_CHAIN_AUTO && long_run);
    }

    int rc = VBCAST_SUCCESS;
    e = vbcast::launch_plan_kernels(pa, pa.n_steps, stream);
    if (e != hipSuccess) rc = hip_fail(e, "plan kernels");

    plan->step_rows.resize(S);
    plan->step_tiles.resize(S);
    plan->step_posted.resize(S);
    plan->step_mismatch.resize(S);
    plan->step_bytes.resize(S);
    auto pull = [&](void *dst, const void *src, size_t bytes) {
        if (rc != VBCAST_SUCCESS || bytes == 0) return;
        hipError_t ee = hipMemcpyAsync(dst, src, bytes, hipMemcpyDeviceToHost, stream);
        if (ee != hipSuccess) rc = hip_fail(ee, "hipMemcpyAsync(step counts)");
    };
    pull(plan->step_rows.data(), pa.step_rows, sizeof(uint32_t) * S);
    pull(plan->step_tiles.data(), pa.step_tiles, sizeof(uint32_t) * S);
    pull(plan->step_posted.data(), pa.step_posted, sizeof(uint32_t) * S);
    pull(plan->step_mismatch.data(), pa.step_mismatch, sizeof(uint32_t) * S);
    pull(plan->step_bytes.data(), pa.step_bytes, sizeof(uint64_t) * S);
    if (rc == VBCAST_SUCCESS) {
        e = hipStreamSynchronize(stream);
        if (e != hipSuccess) rc = hip_fail(e, "hipStreamSynchronize(plan)");
    }
    if (rc == VBCAST_SUCCESS) {
        for (size_t s = 0; s < S; ++s)
            if (plan->step_tiles[s] > pa.tile_cap || plan->step_rows[s] > (uint32_t)P) {
                g_hip_msg = "internal: per-step counts exceed table capacity";
                rc = VBCAST_ERR_HIP;
            }
    }
    if (rc == VBCAST_SUCCESS) rc = build_graph(plan);
    if (rc != VBCAST_SUCCESS) {
        free_plan(plan);
        return rc;
    }
    *out = plan;
    return VBCAST_SUCCESS;
}

int bcast_run(const vbcast_plan *plan, void *hip_stream) {
    if (!plan) return VBCAST_ERR_ARG;
    // the copy kernel alone, or behind the two table kernels whose chain view it reads
    if (one_launch(plan)) return enqueue_broadcast(plan, static_cast<hipStream_t>(hip_stream));
    if (!plan->exec) return VBCAST_ERR_ARG;
    HIP_TRY(hipGraphLaunch(plan->exec, static_cast<hipStream_t>(hip_stream)));
    return VBCAST_SUCCESS;
}

int bcast_run_static(const vbcast_comm *comm, size_t count, size_t dtype_size, int root, int algo,
                     void *hip_stream) {
    if (!comm) return VBCAST_ERR_ARG;
    if (algo != VBCAST_NATIVE && algo != VBCAST_TUNED) return VBCAST_ERR_ARG;
    const int P = comm->P;
    if (P > VBCAST_STATIC_MAX_RANKS) return VBCAST_ERR_LIMIT;
    if (root < 0 || root >= P) return VBCAST_ERR_ROOT;
    if (dtype_size != 0 && count > SIZE_MAX / dtype_size) return VBCAST_ERR_COUNT;
    const uint64_t n = (uint64_t)count * (uint64_t)dtype_size;
    if (n > comm->buf_bytes) return VBCAST_ERR_COUNT;
    int dev = -1;
    hipError_t de = hipGetDevice(&dev);
    if (de != hipSuccess) return hip_fail(de, "hipGetDevice");
    if (dev != comm->device) return VBCAST_ERR_ARG;

    PlanArrays pa{};
    describe_plan(pa, P, root, algo, n, g_tile_log2.load(), 0);
    pa.n_xcd = comm->n_xcd;
    if (bind_plan_arrays(pa, nullptr, /*tile_maps=*/false) > kScratchBytes) return VBCAST_ERR_LIMIT;
    void *tables = nullptr;
    const int rc = scratch_on_device(dev, &tables);   // looked up at vbcast_comm_create
    if (rc != VBCAST_SUCCESS) return rc;
    (void)bind_plan_arrays(pa, static_cast<char *>(tables), /*tile_maps=*/false);
    pa.bases = comm->dev_bases;

    // Every table entry the copy kernel reads is written by the table kernels of
    // this same call first, so nothing of an earlier call's tables has to be cleared.
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    hipError_t e = vbcast::launch_plan_kernels(pa, 0, stream);
    if (e != hipSuccess) return hip_fail(e, "plan kernels");
    if (pa.n_steps == 0) return VBCAST_SUCCESS;
    const uint32_t grid = (uint32_t)comm->compute_units * (uint32_t)g_chain_wgs_per_cu.load();
    e = vbcast::launch_ring_chain(pa, grid, 0, pa.n_steps, /*from_tables=*/true, stream);
    if (e != hipSuccess) return hip_fail(e, "ring chain kernel");
    return VBCAST_SUCCESS;
}

int bcast_run_steps(const vbcast_plan *plan, int first, int last, void *hip_stream) {
    if (!plan) return VBCAST_ERR_ARG;
    if (first < 0 || first > last || last > plan->pa.n_steps) return VBCAST_ERR_ARG;
    return launch_steps(plan, first, last, static_cast<hipStream_t>(hip_stream), nullptr);
}

int bcast_run_chain_steps(const vbcast_plan *plan, int first, int last, void *hip_stream) {
    if (!plan) return VBCAST_ERR_ARG;
    const PlanArrays &pa = plan->pa;
    if (pa.algo != VBCAST_NATIVE && pa.algo != VBCAST_TUNED) return VBCAST_ERR_ARG;
    if (first < 0 || first > last || last > pa.n_steps) return VBCAST_ERR_ARG;
    hipError_t e = vbcast::launch_ring_chain(pa, plan->chain_grid, first, last,
                                             plan->chain_from_tables,
                                             static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return hip_fail(e, "ring chain kernel");
    return VBCAST_SUCCESS;
}

int bcast_run_steps_timed(const vbcast_plan *plan, int first, int last, void *hip_stream,
                          float *step_ms) {
    if (!plan || !step_ms) return VBCAST_ERR_ARG;
    if (first < 0 || first > last || last > plan->pa.n_steps) return VBCAST_ERR_ARG;
    const int k = last - first;
    if (k == 0) return VBCAST_SUCCESS;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    std::vector<hipEvent_t> marks((size_t)k + 1, nullptr);
    int rc = VBCAST_SUCCESS;
    for (auto &m : marks) {
        hipError_t e = hipEventCreate(&m);
        if (e != hipSuccess) {
            rc = hip_fail(e, "hipEventCreate");
            break;
        }
    }
    if (rc == VBCAST_SUCCESS) rc = launch_steps(plan, first, last, stream, marks.data());
    if (rc == VBCAST_SUCCESS) {
        hipError_t e = hipEventSynchronize(marks[k]);
        if (e != hipSuccess) rc = hip_fail(e, "hipEventSynchronize");
    }
    if (rc == VBCAST_SUCCESS) {
        for (int i = 0; i < k; ++i) {
            step_ms[i] = 0.f;
            if (plan->step_tiles[first + i] == 0) continue;
            hipError_t e = hipEventElapsedTime(&step_ms[i], marks[i], marks[i + 1]);
            if (e != hipSuccess) {
                rc = hip_fail(e, "hipEventElapsedTime");
                break;
            }
        }
    }
    for (auto &m : marks)
        if (m) (void)hipEventDestroy(m);
    return rc;
}

int bcast_run_timed(const vbcast_plan *plan, void *hip_stream, float *phase_ms) {
    if (!plan || !phase_ms) return VBCAST_ERR_ARG;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    hipEvent_t marks[4] = {nullptr, nullptr, nullptr, nullptr};
    int rc = VBCAST_SUCCESS;
    for (auto &m : marks) {
        hipError_t e = hipEventCreate(&m);
        if (e != hipSuccess) {
            rc = hip_fail(e, "hipEventCreate");
            break;
        }
    }
    auto mark = [&](int k) {
        if (rc != VBCAST_SUCCESS) return;
        hipError_t e = hipEventRecord(marks[k], stream);
        if (e != hipSuccess) rc = hip_fail(e, "hipEventRecord");
    };
    mark(0);
    if (rc == VBCAST_SUCCESS && !single_kernel(plan)) {
        hipError_t e = vbcast::launch_plan_kernels(plan->pa, tile_map_steps(plan), stream);
        if (e != hipSuccess) rc = hip_fail(e, "plan kernels");
    }
    mark(1);
    if (rc == VBCAST_SUCCESS)
        rc = launch_scatter(plan, stream);
    mark(2);
    if (rc == VBCAST_SUCCESS) rc = launch_ring(plan, stream);
    mark(3);
    if (rc == VBCAST_SUCCESS) {
        hipError_t e = hipEventSynchronize(marks[3]);
        if (e != hipSuccess) rc = hip_fail(e, "hipEventSynchronize");
    }
    for (int k = 0; k < 3 && rc == VBCAST_SUCCESS; ++k) {
        hipError_t e = hipEventElapsedTime(&phase_ms[k], marks[k], marks[k + 1]);
        if (e != hipSuccess) rc = hip_fail(e, "hipEventElapsedTime");
    }
    for (auto &m : marks)
        if (m) (void)hipEventDestroy(m);
    return rc;
}

int bcast_plan_info(const vbcast_plan *plan, vbcast_plan_info *info) {
    if (!plan || !info) return VBCAST_ERR_ARG;
    const PlanArrays &pa = plan->pa;
    std::memset(info, 0, sizeof(*info));
    info->P = pa.P;
    info->root = pa.root;
    info->algo = pa.algo;
    info->n_scatter_steps = pa.n_steps ? pa.n_scatter : 0;
    info->n_steps = pa.n_steps;
    info->tile_bytes = 1 << pa.tile_log2;
    info->n = pa.n;
    info->ss = pa.ss;
    for (int s = 0; s < pa.n_steps; ++s) {
        const bool scatter = s < pa.n_scatter;
        (scatter ? info->scatter_rows : info->ring_rows) += plan->step_rows[s];
        (scatter ? info->scatter_bytes : info->ring_bytes) += plan->step_bytes[s];
        if (!scatter) info->ring_msgs_issued += plan->step_posted[s];
        info->pairing_mismatches += plan->step_mismatch[s];
        info->n_tiles += plan->step_tiles[s];
    }
    info->bytes_moved = info->scatter_bytes + info->ring_bytes;
    const bool copies = pa.n_steps > 0 && pa.n > 0;
    if (single_kernel(plan)) {
        info->run_launches = copies ? 1 : 0;
    } else if (one_launch(plan)) {
        info->run_launches = pa.n_steps > 0 ? 2 + (copies ? 1 : 0) : 1;   // descriptors, rows, copy
    } else {
        info->run_launches = pa.n_steps > 0 ? 3 : 1;                      // descriptors, rows, tile maps
        for (int s = 0; s < pa.n_steps; ++s) info->run_launches += plan->step_tiles[s] > 0 ? 1 : 0;
    }
    return VBCAST_SUCCESS;
}

int bcast_plan_export(const vbcast_plan *plan, uint64_t *step_ptr, uint32_t *src, uint32_t *dst,
                      uint64_t *off, uint64_t *len, uint64_t *step_bytes) {
    if (!plan) return VBCAST_ERR_ARG;
    const PlanArrays &pa = plan->pa;
    uint64_t at = 0;
    std::vector<Row> tmp;
    for (int s = 0; s < pa.n_steps; ++s) {
        const uint32_t nr = plan->step_rows[s];
        if (step_ptr) step_ptr[s] = at;
        if (step_bytes) step_bytes[s] = plan->step_bytes[s];
        if (nr && (src || dst || off || len)) {
            tmp.resize(nr);
            HIP_TRY(hipMemcpy(tmp.data(), pa.rows + (size_t)s * pa.P, sizeof(Row) * nr,
                              hipMemcpyDeviceToHost));
            for (uint32_t k = 0; k < nr; ++k) {
                if (src) src[at + k] = tmp[k].src;
                if (dst) dst[at + k] = tmp[k].dst;
                if (off) off[at + k] = tmp[k].off;
                if (len) len[at + k] = tmp[k].len;
            }
        }
        at += nr;
    }
    if (step_ptr) step_ptr[pa.n_steps] = at;
    return VBCAST_SUCCESS;
}

int bcast_plan_export_desc(const vbcast_plan *plan, uint64_t *chunk_off, uint64_t *chunk_len,
                           int32_t *rel, int32_t *left, int32_t *right, int32_t *sw_step,
                           int32_t *sw_flag) {
    if (!plan) return VBCAST_ERR_ARG;
    const PlanArrays &pa = plan->pa;
    const size_t P = (size_t)pa.P;
    if (chunk_off)
        HIP_TRY(hipMemcpy(chunk_off, pa.chunk_off, sizeof(uint64_t) * (P + 1), hipMemcpyDeviceToHost));
    if (chunk_len)
        HIP_TRY(hipMemcpy(chunk_len, pa.chunk_len, sizeof(uint64_t) * P, hipMemcpyDeviceToHost));
    if (rel) HIP_TRY(hipMemcpy(rel, pa.rel, sizeof(int32_t) * P, hipMemcpyDeviceToHost));
    if (left) HIP_TRY(hipMemcpy(left, pa.left, sizeof(int32_t) * P, hipMemcpyDeviceToHost));
    if (right) HIP_TRY(hipMemcpy(right, pa.right, sizeof(int32_t) * P, hipMemcpyDeviceToHost));
    if (sw_step) HIP_TRY(hipMemcpy(sw_step, pa.sw_step, sizeof(int32_t) * P, hipMemcpyDeviceToHost));
    if (sw_flag) HIP_TRY(hipMemcpy(sw_flag, pa.sw_flag, sizeof(int32_t) * P, hipMemcpyDeviceToHost));
    return VBCAST_SUCCESS;
}

int bcast_plan_export_tiles(const vbcast_plan *plan, int step, uint32_t *n_tiles,
                            uint32_t *tile_row, uint32_t *tile_idx) {
    if (!plan || !n_tiles) return VBCAST_ERR_ARG;
    const PlanArrays &pa = plan->pa;
    if (step < 0 || step >= pa.n_steps) return VBCAST_ERR_ARG;
    const uint32_t nt = plan->step_tiles[step];
    *n_tiles = nt;
    if (nt && (tile_row || tile_idx)) {
        std::vector<Tile> tmp(nt);
        HIP_TRY(hipMemcpy(tmp.data(), pa.tiles + (size_t)step * pa.tile_cap, sizeof(Tile) * nt,
                          hipMemcpyDeviceToHost));
        for (uint32_t k = 0; k < nt; ++k) {
            if (tile_row) tile_row[k] = tmp[k].row;
            if (tile_idx) tile_idx[k] = tmp[k].idx;
        }
    }
    return VBCAST_SUCCESS;
}

int bcast_plan_export_chain(const vbcast_plan *plan, int32_t *holder, uint8_t *moves) {
    if (!plan) return VBCAST_ERR_ARG;
    const PlanArrays &pa = plan->pa;
    if (pa.algo != VBCAST_NATIVE && pa.algo != VBCAST_TUNED) return VBCAST_ERR_ARG;
    const size_t entries = (size_t)pa.P * (size_t)pa.n_steps;
    if (entries == 0 || (!holder && !moves)) return VBCAST_SUCCESS;
    std::vector<uint64_t> raw(entries);
    HIP_TRY(hipMemcpy(raw.data(), pa.chain, entries * sizeof(uint64_t), hipMemcpyDeviceToHost));
    std::unordered_map<uint64_t, int32_t> rank_of;
    for (int r = 0; r < pa.P; ++r)
        rank_of[reinterpret_cast<uint64_t>(plan->comm->host_bases[(size_t)r])] = r;
    for (size_t k = 0; k < entries; ++k) {
        if (holder) {
            auto it = rank_of.find(raw[k] & ~15ull);
            holder[k] = it == rank_of.end() ? -1 : it->second;
        }
        if (moves) moves[k] = (raw[k] & 1ull) ? 0 : 1;
    }
    return VBCAST_SUCCESS;
}

int bcast_plan_census(const vbcast_plan *plan, int ranks_per_node, void *hip_stream,
                      vbcast_census *out) {
    if (!plan || !out || ranks_per_node < 1) return VBCAST_ERR_ARG;
    std::memset(out, 0, sizeof(*out));
    const PlanArrays &pa = plan->pa;
    if (pa.n_steps == 0) return VBCAST_SUCCESS;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    hipError_t e = vbcast::launch_plan_census(pa, ranks_per_node, stream);
    if (e != hipSuccess) return hip_fail(e, "census kernel");
    std::vector<uint64_t> host((size_t)pa.n_steps * 4);
    HIP_TRY(hipMemcpyAsync(host.data(), pa.census, host.size() * sizeof(uint64_t),
                           hipMemcpyDeviceToHost, stream));
    HIP_TRY(hipStreamSynchronize(stream));
    for (int s = 0; s < pa.n_steps; ++s) {
        const uint64_t *v = &host[(size_t)s * 4];
        if (s < pa.n_scatter) {
            out->scatter_inter_msgs += v[0];
            out->scatter_inter_bytes += v[1];
            out->scatter_intra_msgs += v[2];
            out->scatter_intra_bytes += v[3];
        } else {
            out->ring_inter_msgs += v[0];
            out->ring_inter_bytes += v[1];
            out->ring_intra_msgs += v[2];
            out->ring_intra_bytes += v[3];
        }
    }
    return VBCAST_SUCCESS;
}

int bcast_plan_smp_destroy(vbcast_smp_plan *plan) {
    if (!plan) return VBCAST_ERR_ARG;
    if (plan->exec) (void)hipGraphExecDestroy(plan->exec);
    if (plan->graph) (void)hipGraphDestroy(plan->graph);
    for (auto &sub : plan->subs) {
        if (sub.plan) (void)bcast_plan_destroy(sub.plan);
        if (sub.comm) (void)vbcast_comm_destroy(sub.comm);
    }
    delete plan;
    return VBCAST_SUCCESS;
}

int bcast_plan_smp(const vbcast_comm *comm, size_t count, size_t dtype_size, int root,
                   int ranks_per_node, int ring_algo, void *hip_stream, vbcast_smp_plan **out) {
    if (!out) return VBCAST_ERR_ARG;
    *out = nullptr;
    if (!comm || ranks_per_node < 1) return VBCAST_ERR_ARG;
    if (ring_algo != VBCAST_NATIVE && ring_algo != VBCAST_TUNED) return VBCAST_ERR_ARG;
    const int P = comm->P;
    if (root < 0 || root >= P) return VBCAST_ERR_ROOT;
    if (dtype_size != 0 && count > SIZE_MAX / dtype_size) return VBCAST_ERR_COUNT;
    if ((uint64_t)count * (uint64_t)dtype_size > comm->buf_bytes) return VBCAST_ERR_COUNT;

    vbcast_smp_plan *sp = new (std::nothrow) vbcast_smp_plan;
    if (!sp) return VBCAST_ERR_NOMEM;
    const int n_nodes = (P + ranks_per_node - 1) / ranks_per_node;
    const int root_node = root / ranks_per_node;
    auto node_ranks = [&](int j) {
        std::vector<int> m;
        for (int r = j * ranks_per_node; r < P && r < (j + 1) * ranks_per_node; ++r) m.push_back(r);
        return m;
    };
    int rc = VBCAST_SUCCESS;
    auto add = [&](int phase, std::vector<int> members, int sub_root, int algo) {
        if (rc != VBCAST_SUCCESS) return;
        vbcast_smp_plan::Sub sub;
        sub.phase = phase;
        sub.members = std::move(members);
        std::vector<void *> ptrs;
        for (int r : sub.members) ptrs.push_back(comm->host_bases[(size_t)r]);
        rc = vbcast_comm_create((int)ptrs.size(), ptrs.data(), comm->buf_bytes, &sub.comm);
        if (rc == VBCAST_SUCCESS)
            rc = bcast_plan(sub.comm, count, dtype_size, sub_root, algo, hip_stream, &sub.plan);
        sp->subs.push_back(std::move(sub));   // kept even on failure so it is cleaned up
    };
    add(1, node_ranks(root_node), root - root_node * ranks_per_node, VBCAST_BINOMIAL);
    {
        std::vector<int> leaders;
        for (int j = 0; j < n_nodes; ++j) leaders.push_back(j * ranks_per_node);
        add(2, std::move(leaders), root_node, ring_algo);
    }
    for (int j = 0; j < n_nodes; ++j)
        if (j != root_node) add(3, node_ranks(j), 0, VBCAST_BINOMIAL);

    // one graph: every sub-plan's table kernels (where its executor reads tables) and
    // steps, in order
    if (rc == VBCAST_SUCCESS) {
        hipStream_t cap = nullptr;
        hipError_t e = hipStreamCreateWithFlags(&cap, hipStreamNonBlocking);
        if (e != hipSuccess) rc = hip_fail(e, "hipStreamCreateWithFlags");
        if (rc == VBCAST_SUCCESS) {
            e = hipStreamBeginCapture(cap, hipStreamCaptureModeRelaxed);
            if (e != hipSuccess) rc = hip_fail(e, "hipStreamBeginCapture");
            if (rc == VBCAST_SUCCESS) {
                for (auto &sub : sp->subs) {
                    rc = enqueue_broadcast(sub.plan, cap);
                    if (rc != VBCAST_SUCCESS) break;
                }
                hipGraph_t graph = nullptr;
                e = hipStreamEndCapture(cap, &graph);
                if (rc == VBCAST_SUCCESS && e != hipSuccess) rc = hip_fail(e, "hipStreamEndCapture");
                sp->graph = graph;
            }
            (void)hipStreamDestroy(cap);
        }
        if (rc == VBCAST_SUCCESS) {
            e = hipGraphInstantiate(&sp->exec, sp->graph, nullptr, nullptr, 0);
            if (e != hipSuccess) rc = hip_fail(e, "hipGraphInstantiate");
        }
    }
    if (rc != VBCAST_SUCCESS) {
        (void)bcast_plan_smp_destroy(sp);
        return rc;
    }
    *out = sp;
    return VBCAST_SUCCESS;
}

int bcast_run_smp(const vbcast_smp_plan *plan, void *hip_stream) {
    if (!plan || !plan->exec) return VBCAST_ERR_ARG;
    HIP_TRY(hipGraphLaunch(plan->exec, static_cast<hipStream_t>(hip_stream)));
    return VBCAST_SUCCESS;
}

int bcast_run_smp_phase(const vbcast_smp_plan *plan, int phase, void *hip_stream) {
    if (!plan || phase < 1 || phase > 3) return VBCAST_ERR_ARG;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    for (const auto &sub : plan->subs) {
        if (sub.phase != phase) continue;
        const vbcast_plan *p = sub.plan;
        int rc = launch_scatter(p, stream);
        if (rc == VBCAST_SUCCESS) rc = launch_ring(p, stream);
        if (rc != VBCAST_SUCCESS) return rc;
    }
    return VBCAST_SUCCESS;
}

int bcast_smp_subplan(const vbcast_smp_plan *plan, int index, int *count, const vbcast_plan **sub,
                      int *phase, int *n_members, int *members) {
    if (!plan) return VBCAST_ERR_ARG;
    if (count) *count = (int)plan->subs.size();
    if (!sub) return count ? VBCAST_SUCCESS : VBCAST_ERR_ARG;
    if (index < 0 || index >= (int)plan->subs.size()) return VBCAST_ERR_ARG;
    const auto &s = plan->subs[(size_t)index];
    *sub = s.plan;
    if (phase) *phase = s.phase;
    if (n_members) *n_members = (int)s.members.size();
    if (members)
        for (size_t k = 0; k < s.members.size(); ++k) members[k] = s.members[k];
    return VBCAST_SUCCESS;
}

int vbcast_select_algo(size_t nbytes, int P, int tuned, int *algo) {
    if (!algo || P < 1) return VBCAST_ERR_ARG;
    if (nbytes < VBCAST_SHORT_MSG_BYTES)
        *algo = VBCAST_BINOMIAL;
    else if (nbytes < VBCAST_LONG_MSG_BYTES && (P & (P - 1)) == 0)
        *algo = VBCAST_SCATTER_RDB;
    else
        *algo = tuned ? VBCAST_TUNED : VBCAST_NATIVE;
    return VBCAST_SUCCESS;
}

int bcast_plan_destroy(vbcast_plan *plan) {
    if (!plan) return VBCAST_ERR_ARG;
    free_plan(plan);
    return VBCAST_SUCCESS;
}

const char *bcast_strerror(int code) {
    switch (code) {
        case VBCAST_SUCCESS: return "success";
        case VBCAST_ERR_ARG: return "invalid argument";
        case VBCAST_ERR_ROOT: return "root is not a rank of the communicator";
        case VBCAST_ERR_COUNT: return "message size overflows or exceeds the rank buffers";
        case VBCAST_ERR_ALIGN: return "rank buffer is not 16-byte aligned";
        case VBCAST_ERR_NOMEM: return "out of memory";
        case VBCAST_ERR_LIMIT:
            return "communicator too large for the static tables of bcast_run_static";
        case VBCAST_ERR_HIP:
            g_text = "HIP runtime failure: " + g_hip_msg;
            return g_text.c_str();
        default: return "unknown error code";
    }
}

}  // extern "C"
