"""GPU path vs CPU oracle, bit for bit: tables, descriptors, byte counts, the
state after every step and the final state.  Everything goes through the C-ABI
library (via the ctypes binding)."""

import numpy as np
import pytest

from oracle import bcast_oracle as O
from paper_1603_06809_amd import inputs as I
import harness as H

pytestmark = pytest.mark.gpu

ALGOS = [O.NATIVE, O.TUNED]
DEFAULT_TILE = 16384
DEFAULT_SLAB = 16384


@pytest.fixture(scope="module")
def V():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_1603_06809_amd import vbcast
    vbcast.lib()
    vbcast.vbcast_set_tile_bytes(DEFAULT_TILE)
    vbcast.vbcast_set_chain_slab_bytes(DEFAULT_SLAB)
    vbcast.vbcast_set_ring_executor(vbcast.RING_CHAINS)
    vbcast.vbcast_set_chain_schedule(vbcast.CHAIN_AUTO)
    return vbcast


# "chains": the one-launch executor as it comes (it works its hops out itself for
# short broadcasts and looks them up for long ones); "inline" / "tables": the same
# kernel held to one of the two; "steps": one launch per step over the step tables.
EXECUTORS = ["chains", "steps"]
ALL_EXECUTORS = ["inline", "tables", "steps"]


def set_executor(V, name):
    V.vbcast_set_ring_executor(V.RING_STEPS if name == "steps" else V.RING_CHAINS)
    V.vbcast_set_chain_schedule({"inline": V.CHAIN_INLINE, "tables": V.CHAIN_TABLES}.get(name, V.CHAIN_AUTO))


def sync():
    import torch
    torch.cuda.synchronize()


def stepper(plan, executor):
    """Runs steps [first, last): one launch per step, or the one-launch executor's
    kernel held to that range of steps."""
    return plan.run_steps if executor == "steps" else plan.run_chain_steps


def make(V, w, algo, pad=64, executor="chains"):
    state = H.device_buffers(w, pad)
    comm = V.Comm([state[r].data_ptr() for r in range(w.P)], state.shape[1])
    set_executor(V, executor)
    plan = V.bcast_plan(comm, w.n, 1, w.root, algo)
    set_executor(V, "chains")
    return state, comm, plan


def check_tables(plan, sched):
    info = plan.info()
    assert (info.P, info.root, info.n) == (sched.P, sched.root, sched.n)
    assert info.ss == sched.ss
    assert info.n_steps == sched.n_steps
    assert info.n_scatter_steps == (sched.n_scatter_steps if sched.P > 1 else 0)
    rows = sched.step_rows()
    nsc = sched.n_scatter_steps
    assert info.scatter_rows == sum(rows[:nsc]) and info.ring_rows == sum(rows[nsc:])
    assert info.scatter_bytes == sched.scatter_bytes
    assert info.ring_bytes == sched.ring_bytes
    assert info.bytes_moved == sched.bytes_moved
    assert info.ring_msgs_issued == sched.ring_msgs_issued
    assert info.pairing_mismatches == 0
    t = plan.export()
    want_ptr = np.concatenate([[0], np.cumsum(rows)]).astype(np.uint64)
    assert np.array_equal(t.step_ptr, want_ptr)
    assert np.array_equal(t.step_bytes, np.array(sched.step_bytes(), dtype=np.uint64))
    flat = [r for step in sched.steps for r in step]
    want = np.array(flat, dtype=np.uint64).reshape(-1, 4)
    assert np.array_equal(t.src.astype(np.uint64), want[:, 0])
    assert np.array_equal(t.dst.astype(np.uint64), want[:, 1])
    assert np.array_equal(t.off, want[:, 2])
    assert np.array_equal(t.len, want[:, 3])
    return t


def check_desc(plan, w):
    d = plan.export_desc()
    P, root, n = w.P, w.root, w.n
    ext = [O.chunk_extent(c, n, P) for c in range(P)]
    assert [int(x) for x in d["chunk_len"]] == [e[1] for e in ext]
    run = 0
    for c in range(P):
        assert int(d["chunk_off"][c]) == run
        if ext[c][1] > 0:
            assert run == ext[c][0]
        run += ext[c][1]
    assert int(d["chunk_off"][P]) == n
    for r in range(P):
        rel = O.relative_rank(r, root, P)
        assert d["rel"][r] == rel
        assert d["left"][r] == (P + r - 1) % P and d["right"][r] == (r + 1) % P
        sw = O.tuned_switch(rel, P)
        assert (d["sw_step"][r], d["sw_flag"][r]) == (sw if sw else (-1, -1))


def check_chain(plan, sched):
    """The chunk-major view the one-launch executor walks, against the oracle's
    rows: a chunk moves in a step iff a row of that step covers it, and then it
    lands in that row's destination; where it does not move it stays with its
    holder during the scatter, and in ring step i it is looked for at the rank i
    places above its own."""
    P, root, n = sched.P, sched.root, sched.n
    holder, moves = plan.export_chain()
    ss = sched.ss
    want_h = np.zeros((P, sched.n_steps), np.int32)
    want_m = np.zeros((P, sched.n_steps), np.uint8)
    cur = [root] * P
    for s, rows in enumerate(sched.steps):
        landed = {}
        for (_src, dst, off, ln) in rows:
            for c in range(off // ss, (off + ln + ss - 1) // ss):
                landed[c] = dst
        for c in range(P):
            if c in landed:
                cur[c] = landed[c]
                want_m[c, s] = 1
            elif s >= sched.n_scatter_steps:
                cur[c] = (root + c + (s - sched.n_scatter_steps + 1)) % P
            elif O.chunk_extent(c, n, P)[1] == 0:
                # an empty chunk still has a place in the tree; nothing is copied for it
                m = O.ceil_pow2(P) >> (s + 1)
                cur[c] = (root + (c & ~(m - 1))) % P
            want_h[c, s] = cur[c]
    assert np.array_equal(moves, want_m)
    assert np.array_equal(holder, want_h)


def check_tiles(plan, t, steps):
    tb = plan.info().tile_bytes
    for s in steps:
        row, idx = plan.export_tiles(s)
        rows = t.rows_of(s)
        want = []
        for k, (_s, _d, off, ln) in enumerate(rows):
            nt = (off + ln - 1) // tb - off // tb + 1
            want += [(k, j) for j in range(nt)]
        assert list(zip(row.tolist(), idx.tolist())) == want


# ------------------------------------------------------------------ small and edge cases

EDGE = [(P, root, n)
        for P in (1, 2, 3, 5, 7, 8, 13, 16, 33)
        for root in sorted({0, P - 1})
        for n in sorted({0, 1, 15, 16, 17, P - 1, P + 1, 1000, 4097, 70_001})]


@pytest.mark.parametrize("algo", ALGOS)
def test_edge_cases_every_step(V, algo):
    """Tiny and degenerate shapes: one rank, empty message, fewer bytes than
    ranks (empty chunks), lengths around the 16-byte word."""
    for (P, root, n) in EDGE:
        w = I.Workload(f"edge_{P}_{root}_{n}", P, root, n, seed=1000 + P * 131 + n)
        state, comm, plan = make(V, w, algo, pad=40)
        sched = O.build_schedule(P, root, n, algo)
        check_tables(plan, sched)
        check_desc(plan, w)
        check_chain(plan, sched)
        plan.destroy()
        for ex in ALL_EXECUTORS:
            set_executor(V, ex)
            plan = V.bcast_plan(comm, n, 1, root, algo)
            set_executor(V, "chains")
            H.refill(state, w)
            ref = H.host_buffers(w, pad=40)
            for s in range(sched.n_steps):
                stepper(plan, ex)(s, s + 1)
                O.apply_step(ref, sched.steps[s])
                got = state.cpu().numpy()
                assert np.array_equal(got, np.stack(ref)), (P, root, n, algo, ex, s)
            plan.destroy()
        # and the whole broadcast from a fresh state, every way of running it
        want = np.stack(O.broadcast_definition(H.host_buffers(w, pad=40), root, n))
        for ex in ALL_EXECUTORS:
            set_executor(V, ex)
            plan = V.bcast_plan(comm, n, 1, root, algo)
            set_executor(V, "chains")
            H.refill(state, w)
            plan.run()
            sync()
            assert np.array_equal(state.cpu().numpy(), want), (P, root, n, algo, ex)
            plan.destroy()
        comm.destroy()


# ------------------------------------------------------------------ the workloads

@pytest.mark.parametrize("executor", ALL_EXECUTORS)
@pytest.mark.parametrize("algo", ALGOS)
@pytest.mark.parametrize("name", ["P10_n512K", "P24_n4M"])
def test_state_after_every_step(V, name, algo, executor):
    """State of every rank buffer after every step, with the per-step kernel and
    with the one-launch executor's kernel held to one step at a time (hops worked
    out in the kernel, or looked up)."""
    w = I.workload(name)
    state, comm, plan = make(V, w, algo, executor=executor)
    sched = O.build_schedule(w.P, w.root, w.n, algo)
    # kernels per bcast_run: the copy kernel alone; behind the two table kernels; or
    # three table kernels and one copy kernel per step that moves something
    assert plan.info().run_launches == {"inline": 1, "tables": 3}.get(
        executor, 3 + sum(1 for rows in sched.steps if rows))
    t = check_tables(plan, sched)
    check_desc(plan, w)
    check_chain(plan, sched)
    check_tiles(plan, t, range(sched.n_steps))
    ref = H.host_buffers(w)
    for s in range(sched.n_steps):
        stepper(plan, executor)(s, s + 1)
        O.apply_step(ref, sched.steps[s])
        assert np.array_equal(state.cpu().numpy(), np.stack(ref)), (name, algo, executor, s)
    want = O.broadcast_definition(H.host_buffers(w), w.root, w.n)
    assert np.array_equal(np.stack(ref), np.stack(want))
    plan.destroy()
    comm.destroy()


@pytest.mark.parametrize("executor", EXECUTORS)
@pytest.mark.parametrize("algo", ALGOS)
@pytest.mark.parametrize("name", ["P64_n16M", "P96_n12M_ragged"])
def test_state_at_sampled_steps(V, name, algo, executor):
    w = I.workload(name)
    state, comm, plan = make(V, w, algo)
    sched = O.build_schedule(w.P, w.root, w.n, algo)
    t = check_tables(plan, sched)
    check_desc(plan, w)
    nsc, S = sched.n_scatter_steps, sched.n_steps
    check_tiles(plan, t, [0, nsc - 1, nsc, S - 1])
    ref = H.host_buffers(w)
    stops = sorted({1, nsc, nsc + 1, nsc + 2, nsc + (w.P - 1) // 2, S - 1, S})
    done = 0
    for stop in stops:
        stepper(plan, executor)(done, stop)
        O.run_steps(ref, sched, done, stop)
        done = stop
        got = state.cpu().numpy()
        for r in range(w.P):
            assert np.array_equal(got[r], ref[r]), (name, algo, executor, stop, r)
    plan.destroy()
    comm.destroy()


@pytest.mark.parametrize("executor", ALL_EXECUTORS)
@pytest.mark.parametrize("algo", ALGOS)
@pytest.mark.parametrize("name", ["P10_n512K", "P24_n4M", "P64_n16M", "P96_n12M_ragged"])
def test_graph_run_final_state(V, name, algo, executor):
    """bcast_run from a fresh state, twice (the one kernel, or the graph, whose
    second launch regenerates the tables and must give the same result).  Every
    way of running the ring phase."""
    w = I.workload(name)
    state, comm, plan = make(V, w, algo, executor=executor)
    want = np.stack(O.broadcast_definition(H.host_buffers(w), w.root, w.n))
    for _ in range(2):
        H.refill(state, w)
        V.bcast_run(plan)
        sync()
        assert np.array_equal(state.cpu().numpy(), want)
    sched = O.build_schedule(w.P, w.root, w.n, algo)
    check_tables(plan, sched)   # tables after regeneration inside the graph
    plan.destroy()
    comm.destroy()


LAYOUTS_EVERY_STEP = [("P10_n512K", 16), ("P10_n512K", 48), ("P24_n4M", 112), ("P24_n4M", "mixed"),
                      ("P24_n4M", "per_rank")]


@pytest.mark.parametrize("executor", EXECUTORS)
@pytest.mark.parametrize("name,layout", LAYOUTS_EVERY_STEP)
def test_other_buffer_layouts_every_step(V, name, layout, executor):
    """Rank buffers whose bases are 16-byte aligned but sit 16, 48 or 112 bytes
    past a 256-byte boundary, or at different places inside their 256-byte
    windows, or in one allocation per rank in shuffled address order: the state
    after every step, both kernels, both schedules."""
    w = I.workload(name)
    rows, _keep = H.device_rows(w, layout)
    stride = rows[0].numel()
    assert len({r.data_ptr() % 16 for r in rows}) == 1
    if layout != "per_rank":
        assert any(r.data_ptr() % 256 for r in rows)
    comm = V.Comm([r.data_ptr() for r in rows], stride)
    for algo in ALGOS:
        H.refill_rows(rows, w)
        set_executor(V, executor)
        plan = V.bcast_plan(comm, w.n, 1, w.root, algo)
        set_executor(V, "chains")
        sched = O.build_schedule(w.P, w.root, w.n, algo)
        check_tables(plan, sched)
        ref = H.host_rows(w, stride)
        for s in range(sched.n_steps):
            stepper(plan, executor)(s, s + 1)
            O.apply_step(ref, sched.steps[s])
            assert np.array_equal(H.rows_to_numpy(rows), np.stack(ref)), (name, layout, algo, executor, s)
        H.refill_rows(rows, w)
        V.bcast_run(plan)
        sync()
        want = np.stack(O.broadcast_definition(H.host_rows(w, stride), w.root, w.n))
        assert np.array_equal(H.rows_to_numpy(rows), want), (name, layout, algo, executor, "graph")
        plan.destroy()
    comm.destroy()


@pytest.mark.parametrize("executor", EXECUTORS)
@pytest.mark.parametrize("layout", [16, 48, 112, "mixed", "per_rank"])
def test_other_buffer_layouts_final_state(V, layout, executor):
    """The ragged workload (96 ranks, odd chunk size) on the same layouts: the
    state in mid-ring and at the end."""
    w = I.workload("P96_n12M_ragged")
    rows, _keep = H.device_rows(w, layout)
    stride = rows[0].numel()
    comm = V.Comm([r.data_ptr() for r in rows], stride)
    for algo in ALGOS:
        H.refill_rows(rows, w)
        set_executor(V, executor)
        plan = V.bcast_plan(comm, w.n, 1, w.root, algo)
        set_executor(V, "chains")
        sched = O.build_schedule(w.P, w.root, w.n, algo)
        ref = H.host_rows(w, stride)
        done = 0
        for stop in (sched.n_scatter_steps + 41, sched.n_steps):
            stepper(plan, executor)(done, stop)
            O.run_steps(ref, sched, done, stop)
            done = stop
            assert np.array_equal(H.rows_to_numpy(rows), np.stack(ref)), (layout, algo, executor, stop)
        H.refill_rows(rows, w)
        V.bcast_run(plan)
        sync()
        assert np.array_equal(H.rows_to_numpy(rows), np.stack(ref)), (layout, algo, executor, "graph")
        plan.destroy()
    comm.destroy()


@pytest.mark.parametrize("n_xcd", [1, 2, 3, 4, 16])
def test_other_xcd_counts(V, n_xcd):
    """The kernels' map from workgroups to pieces of the message for other numbers
    of accelerator dies than the device reports: still every piece exactly once."""
    V.vbcast_set_xcd_count(n_xcd)
    try:
        for name in ("P24_n4M", "P96_n12M_ragged"):
            w = I.workload(name)
            for ex in EXECUTORS:
                state, comm, plan = make(V, w, O.TUNED, executor=ex)
                want = np.stack(O.broadcast_definition(H.host_buffers(w), w.root, w.n))
                plan.run()
                sync()
                assert np.array_equal(state.cpu().numpy(), want), (name, n_xcd, ex)
                plan.destroy()
                comm.destroy()
    finally:
        V.vbcast_set_xcd_count(0)


@pytest.mark.parametrize("tile", [4096, 8192, 32768, 65536])
def test_other_tile_sizes(V, tile):
    w = I.workload("P24_n4M")
    V.vbcast_set_tile_bytes(tile)
    V.vbcast_set_chain_slab_bytes(tile)
    try:
        for algo in ALGOS:
            state, comm, plan = make(V, w, algo)
            assert plan.info().tile_bytes == tile
            want = np.stack(O.broadcast_definition(H.host_buffers(w), w.root, w.n))
            plan.run()          # the one-launch ring with this tile size
            sync()
            assert np.array_equal(state.cpu().numpy(), want)
            H.refill(state, w)
            sched = O.build_schedule(w.P, w.root, w.n, algo)
            t = check_tables(plan, sched)
            check_tiles(plan, t, [0, sched.n_scatter_steps, sched.n_steps - 1])
            ref = H.host_buffers(w)
            nsc = sched.n_scatter_steps
            for (a, b) in [(0, nsc), (nsc, nsc + 3), (nsc + 3, sched.n_steps)]:
                plan.run_steps(a, b)
                O.run_steps(ref, sched, a, b)
                assert np.array_equal(state.cpu().numpy(), np.stack(ref))
            plan.destroy()
            comm.destroy()
    finally:
        V.vbcast_set_tile_bytes(DEFAULT_TILE)
        V.vbcast_set_chain_slab_bytes(DEFAULT_SLAB)


@pytest.mark.parametrize("wgs", [2, 3, 5, 16])
def test_other_numbers_of_chain_workgroups(V, wgs):
    """The one-launch executor with other numbers of resident workgroups per
    compute unit (the grid and the runs of slabs per XCD follow from it)."""
    V.vbcast_set_chain_workgroups_per_cu(wgs)
    try:
        for name in ("P24_n4M", "P96_n12M_ragged"):
            w = I.workload(name)
            state, comm, plan = make(V, w, O.TUNED)
            want = np.stack(O.broadcast_definition(H.host_buffers(w), w.root, w.n))
            plan.run()
            sync()
            assert np.array_equal(state.cpu().numpy(), want), (name, wgs)
            plan.destroy()
            comm.destroy()
    finally:
        V.vbcast_set_chain_workgroups_per_cu(1)


def test_plans_give_their_device_memory_back(V):
    """Two hundred plans (and a three-phase plan each tenth time) created, run and
    destroyed: the device's free memory ends where it started."""
    import torch
    w = I.workload("P24_n4M")
    state = H.device_buffers(w)
    comm = V.Comm([state[r].data_ptr() for r in range(w.P)], state.shape[1])
    # the runtime sets up a pool of its own on the first plan: not ours, not counted
    for warm in (V.bcast_plan(comm, w.n, 1, w.root, V.TUNED), V.bcast_plan_smp(comm, w.n, 1, w.root, 5, "tuned")):
        warm.run()
        sync()
        warm.destroy()
    sync()
    free0 = torch.cuda.mem_get_info()[0]
    for k in range(200):
        plan = V.bcast_plan(comm, w.n, 1, w.root, ALGOS[k % 2])
        plan.run()
        if k % 10 == 0:
            smp = V.bcast_plan_smp(comm, w.n, 1, w.root, 5, "tuned")
            smp.run()
            sync()
            smp.destroy()
        sync()
        plan.destroy()
    sync()
    free1 = torch.cuda.mem_get_info()[0]
    assert free0 - free1 < (4 << 20), (free0, free1)
    comm.destroy()


def test_timed_steps_report_a_time_per_step(V):
    w = I.workload("P24_n4M")
    state, comm, plan = make(V, w, O.TUNED)
    ms = plan.run_steps_timed(0, plan.info().n_steps)
    assert ms.shape == (plan.info().n_steps,) and (ms > 0).all()
    want = np.stack(O.broadcast_definition(H.host_buffers(w), w.root, w.n))
    assert np.array_equal(state.cpu().numpy(), want)
    H.refill(state, w)
    phases = plan.run_timed()
    # with the one-launch executor the scatter phase launches nothing: its slot is
    # the gap between two event records, which may read as zero
    assert phases.shape == (3,) and phases[0] > 0 and phases[1] >= 0 and phases[2] > 0
    assert np.array_equal(state.cpu().numpy(), want)
    plan.destroy()
    comm.destroy()


def test_errors_on_device(V):
    import torch
    bufs = [torch.zeros(256, dtype=torch.uint8, device="cuda") for _ in range(4)]
    comm = V.Comm.from_tensors(bufs)
    for args, code in [((16, 1, 4, V.NATIVE), V.ERR_ROOT), ((16, 1, -1, V.NATIVE), V.ERR_ROOT),
                       ((257, 1, 0, V.NATIVE), V.ERR_COUNT), ((1 << 62, 8, 0, V.TUNED), V.ERR_COUNT),
                       ((16, 1, 0, 4), V.ERR_ARG), ((16, 1, 0, -1), V.ERR_ARG)]:
        with pytest.raises(V.VbcastError) as e:
            V.bcast_plan(comm, *args)
        assert e.value.code == code
    plan = V.bcast_plan(comm, 256, 1, 0, V.TUNED)
    for (a, b) in [(-1, 2), (3, 2), (0, plan.info().n_steps + 1)]:
        for run in (plan.run_steps, plan.run_chain_steps):
            with pytest.raises(V.VbcastError) as e:
                run(a, b)
            assert e.value.code == V.ERR_ARG
    plan.destroy()
    tree = V.bcast_plan(comm, 256, 1, 0, V.BINOMIAL)   # no chains in a tree broadcast
    with pytest.raises(V.VbcastError) as e:
        tree.run_chain_steps(0, 1)
    assert e.value.code == V.ERR_ARG
    tree.destroy()
    comm.destroy()


# ------------------------------------------------------------------ the neighbouring algorithms

OTHER_SHAPES = [(P, root, n)
                for P in (1, 2, 3, 4, 7, 8, 13, 16, 32, 33, 64)
                for root in sorted({0, P - 1})
                for n in sorted({0, 1, 17, P + 1, 1000, 12_287, 70_001})]


@pytest.mark.parametrize("algo", [O.BINOMIAL, O.SCATTER_RDB])
def test_neighbouring_algorithms_every_step(V, algo):
    """Binomial-tree broadcast and scatter + recursive doubling: tables exact,
    state exact after every step, graph run exact."""
    for (P, root, n) in OTHER_SHAPES:
        if algo == O.SCATTER_RDB and P & (P - 1):
            continue
        w = I.Workload(f"other_{P}_{root}_{n}", P, root, n, seed=5000 + P * 17 + n)
        state, comm, plan = make(V, w, algo, pad=40)
        sched = O.build_schedule(P, root, n, algo)
        check_tables(plan, sched)
        ref = H.host_buffers(w, pad=40)
        for s in range(sched.n_steps):
            plan.run_steps(s, s + 1)
            O.apply_step(ref, sched.steps[s])
            assert np.array_equal(state.cpu().numpy(), np.stack(ref)), (P, root, n, algo, s)
        H.refill(state, w)
        plan.run()
        sync()
        want = np.stack(O.broadcast_definition(H.host_buffers(w, pad=40), root, n))
        assert np.array_equal(state.cpu().numpy(), want), (P, root, n, algo)
        plan.destroy()
        comm.destroy()


def test_recursive_doubling_rejects_other_process_counts(V):
    import torch
    bufs = [torch.zeros(256, dtype=torch.uint8, device="cuda") for _ in range(6)]
    comm = V.Comm.from_tensors(bufs)
    with pytest.raises(V.VbcastError) as e:
        V.bcast_plan(comm, 64, 1, 0, V.SCATTER_RDB)
    assert e.value.code == V.ERR_ARG
    comm.destroy()


@pytest.mark.parametrize("P,n", [(16, 4096), (16, 12_288), (16, 524_287), (64, 100_000), (256, 12_288),
                                 (129, 4096), (9, 12_287), (513, 8192), (64, 524_288)])
def test_selected_algorithm_runs(V, P, n):
    """MPI_Bcast as a whole: pick the algorithm by the size / process-count rule
    (the library's choice must be the oracle's), run it, compare."""
    for tuned in (False, True):
        code = V.vbcast_select_algo(n, P, tuned)
        algo = V.ALGO_NAMES[code]
        assert algo == O.select_algorithm(n, P, tuned)
        w = I.Workload(f"auto_{P}_{n}", P, P // 2, n, seed=9000 + P)
        state, comm, plan = make(V, w, algo)
        sched = O.build_schedule(P, w.root, n, algo)
        check_tables(plan, sched)
        plan.run()
        sync()
        want = np.stack(O.broadcast_definition(H.host_buffers(w), w.root, n))
        assert np.array_equal(state.cpu().numpy(), want), (P, n, algo)
        plan.destroy()
        comm.destroy()


@pytest.mark.parametrize("P,root,n,rpn", [(16, 0, 524_288, 24), (64, 17, 999_983, 24), (256, 5, 524_288, 24),
                                          (129, 128, 12_288, 24), (10, 3, 1000, 4), (50, 0, 77, 7),
                                          (513, 256, 8192, 24), (64, 0, 100_000, 24)])
def test_node_census(V, P, root, n, rpn):
    """Inter-/intra-node census counted on the GPU vs the oracle's, every algorithm."""
    import torch
    bufs = [torch.zeros(n + 16, dtype=torch.uint8, device="cuda") for _ in range(P)]
    comm = V.Comm.from_tensors(bufs)
    for algo in (O.NATIVE, O.TUNED, O.BINOMIAL, O.SCATTER_RDB):
        if algo == O.SCATTER_RDB and P & (P - 1):
            continue
        plan = V.bcast_plan(comm, n, 1, root, algo)
        want = O.node_census(O.build_schedule(P, root, n, algo), rpn)
        assert plan.census(rpn) == want, (P, root, n, rpn, algo)
        plan.destroy()
    plan = V.bcast_plan(comm, n, 1, root, V.TUNED)
    with pytest.raises(V.VbcastError):
        plan.census(0)
    plan.destroy()
    comm.destroy()


SMP_CASES = [(9, 4, 12_288, 4), (17, 16, 100_001, 4), (25, 12, 12_288, 24), (33, 0, 524_287, 8),
             (65, 40, 1_048_576, 24), (129, 5, 12_288, 24), (129, 128, 524_287, 24), (7, 6, 5, 3),
             (24, 23, 4096, 24), (1, 0, 100, 24), (10, 3, 0, 4)]


@pytest.mark.parametrize("P,root,n,rpn", SMP_CASES)
def test_three_phase_broadcast(V, P, root, n, rpn):
    """The multi-core-aware three-phase broadcast [Sec. I]: sub-communicators and
    their tables exact, state exact at the phase boundaries, graph run exact."""
    w = I.Workload(f"smp_{P}_{root}_{n}", P, root, n, seed=31_000 + P)
    state = H.device_buffers(w, pad=40)
    comm = V.Comm([state[r].data_ptr() for r in range(P)], state.shape[1])
    for ring in (O.NATIVE, O.TUNED):
        subs = O.smp_schedule(P, root, n, rpn, ring)
        plan = V.bcast_plan_smp(comm, n, 1, root, rpn, ring)
        got = plan.subplans()
        assert [(ph, m) for (ph, m, _p) in got] == [(s.phase, s.members) for s in subs]
        for (_ph, _m, view), sub in zip(got, subs):
            check_tables(view, sub.sched)
        H.refill(state, w)
        ref = H.host_buffers(w, pad=40)
        for phase in (1, 2, 3):
            plan.run_phase(phase)
            O.run_smp(ref, subs, phases=(phase,))
            assert np.array_equal(state.cpu().numpy(), np.stack(ref)), (P, root, n, rpn, ring, phase)
        H.refill(state, w)
        plan.run()
        sync()
        want = np.stack(O.broadcast_definition(H.host_buffers(w, pad=40), root, n))
        assert np.array_equal(state.cpu().numpy(), want), (P, root, n, rpn, ring)
        plan.destroy()
    for bad in [dict(root=P), dict(rpn=0), dict(ring=V.BINOMIAL)]:
        args = dict(root=root, rpn=rpn, ring=V.TUNED)
        args.update(bad)
        with pytest.raises(V.VbcastError):
            V.bcast_plan_smp(comm, n, 1, args["root"], args["rpn"], args["ring"])
    comm.destroy()


# ------------------------------------------------------------------ the paper's own shapes

PAPER_SHAPES = (
    [(P, n) for P in (9, 17, 33, 65, 129) for n in (12_288, 524_287, 1_048_576)]   # Sec. V-B
    + [(129, 2_560_000)]
    + [(16, 524_288), (16, 30_000_000), (64, 3_000_000), (64, 30_000_000),       # Sec. V-A
       (256, 524_288), (256, 3_000_000)]
)


@pytest.mark.parametrize("P,n", PAPER_SHAPES)
def test_paper_sweep_shapes(V, P, n):
    """Process counts and message sizes of the paper's experiments (Sec. V):
    tables exact, final state exact, both schedules, both ring executors."""
    w = I.Workload(f"paper_P{P}_n{n}", P, P // 3, n, seed=77_000 + P)
    init = H.host_buffers(w)
    want = np.stack(O.broadcast_definition(init, w.root, w.n))
    state = H.device_buffers(w)
    comm = V.Comm([state[r].data_ptr() for r in range(w.P)], state.shape[1])
    for algo in ALGOS:
        sched = O.build_schedule(P, w.root, n, algo)
        for ex in EXECUTORS:
            set_executor(V, ex)
            plan = V.bcast_plan(comm, n, 1, w.root, algo)
            set_executor(V, "chains")
            if ex == "chains":
                check_tables(plan, sched)
            H.refill(state, w)
            V.bcast_run(plan)
            sync()
            assert np.array_equal(state.cpu().numpy(), want), (P, n, algo, ex)
            plan.destroy()
    comm.destroy()


@pytest.mark.parametrize("P", [5, 16, 33])
def test_chunk_sizes_around_the_slab_sizes(V, P):
    """The one-launch executor picks its slab (1, 2, 4, 8 KiB) and its kernel from
    the chunk size: chunk sizes one below, at and one above every switch
    (and where a chunk holds one and four of the largest slab), with a
    last chunk P - 1 bytes short and with an exact fit."""
    for ss in (1023, 1024, 1025, 2047, 2048, 2049, 4095, 4096, 4097, 8191, 8192, 8193, 16383, 16384,
               16385, 65535, 65536, 65537):
        for n in (P * ss, P * ss - (P - 1)):
            w = I.Workload(f"slab_P{P}_n{n}", P, P - 2, n, seed=99_000 + P + ss)
            assert -(-n // P) == ss
            init = H.host_buffers(w)
            want = np.stack(O.broadcast_definition(init, w.root, w.n))
            state = H.device_buffers(w)
            comm = V.Comm([state[r].data_ptr() for r in range(P)], state.shape[1])
            for algo in ALGOS:
                for ex in ("inline", "tables"):
                    set_executor(V, ex)
                    plan = V.bcast_plan(comm, n, 1, w.root, algo)
                    set_executor(V, "chains")
                    H.refill(state, w)
                    plan.run()
                    sync()
                    assert np.array_equal(state.cpu().numpy(), want), (P, n, ss, algo, ex)
                    plan.destroy()
            comm.destroy()


@pytest.mark.parametrize("P", [257, 258])
def test_chunk_boundary_lines_around_the_rank_limit(V, P):
    """Up to 257 ranks on a 256-unit device the one-launch executor walks the cache
    line in which two chunks meet in a workgroup of its own, beyond that with the
    slab it lies in: both sides of the limit, chunks of 5000 bytes (every boundary
    inside a line), the broadcast in three pieces cut at steps 7 and n_steps - 3,
    hops worked out and looked up, both schedules."""
    n = P * 5000 - 7
    w = I.Workload(f"cutline_P{P}", P, 11, n, seed=31_000 + P)
    for algo in ALGOS:
        sched = O.build_schedule(P, w.root, n, algo)
        assert sched.ss == 5000
        for ex in ("inline", "tables"):
            state, comm, plan = make(V, w, algo, pad=24, executor=ex)
            ref = [H.host_row(w, r, state.shape[1]) for r in range(P)]
            for (first, last) in ((0, 7), (7, sched.n_steps - 3), (sched.n_steps - 3, sched.n_steps)):
                plan.run_chain_steps(first, last)
                O.run_steps(ref, sched, first, last)
                assert np.array_equal(state.cpu().numpy(), np.stack(ref)), (P, algo, ex, first, last)
            want = np.stack(O.broadcast_definition([H.host_row(w, r, state.shape[1]) for r in range(P)], w.root, n))
            assert np.array_equal(np.stack(ref), want)
            plan.destroy()
            comm.destroy()


def test_sweep_modes_run_and_check_their_results(V, capsys):
    """The two side sweeps (every algorithm around the size thresholds; flat
    against three-phase) return 0 only if every broadcast they timed left every
    rank equal to the root."""
    import torch
    from paper_1603_06809_amd import sweep
    assert sweep.selection(V, torch, 2, True) == 0
    assert sweep.smp(V, torch, 2, 24, True) == 0
    out = capsys.readouterr().out
    assert out.count("\n| ") >= 27 + 7


# ------------------------------------------------------------------ random shapes, streams, many ranks

def test_random_shapes_final_state(V):
    """A seeded random walk over (P, root, n, algorithm): tables and final state."""
    import random
    rnd = random.Random(20160306)
    for _ in range(60):
        P = rnd.choice([2, 3, 5, 6, 11, 12, 20, 31, 48, 100, 127, 200])
        root = rnd.randrange(P)
        n = rnd.choice([rnd.randrange(0, 64), rnd.randrange(64, 20_000), rnd.randrange(20_000, 3_000_000)])
        algo = rnd.choice([O.NATIVE, O.TUNED, O.TUNED, O.BINOMIAL])
        w = I.Workload(f"rnd_{P}_{root}_{n}", P, root, n, seed=rnd.randrange(1 << 30))
        V.vbcast_set_tile_bytes(rnd.choice([4096, 8192, 16384]))
        V.vbcast_set_chain_slab_bytes(rnd.choice([4096, 8192, 16384, 65536]))
        try:
            state, comm, plan = make(V, w, algo, pad=rnd.choice([0, 1, 40, 300]),
                                     executor=rnd.choice(ALL_EXECUTORS))
        finally:
            V.vbcast_set_tile_bytes(DEFAULT_TILE)
            V.vbcast_set_chain_slab_bytes(DEFAULT_SLAB)
        sched = O.build_schedule(P, root, n, algo)
        check_tables(plan, sched)
        plan.run()
        sync()
        want = np.stack(O.broadcast_definition(
            [H.host_row(w, r, state.shape[1]) for r in range(P)], root, n))
        assert np.array_equal(state.cpu().numpy(), want), (P, root, n, algo)
        if algo != O.BINOMIAL and sched.n_steps > 0:
            # the same broadcast in three pieces cut at random steps, each piece one
            # launch of the one-launch executor's kernel
            H.refill(state, w)
            ref = [H.host_row(w, r, state.shape[1]) for r in range(P)]
            a = rnd.randrange(sched.n_steps + 1)
            b = rnd.randrange(a, sched.n_steps + 1)
            for (first, last) in ((0, a), (a, b), (b, sched.n_steps)):
                plan.run_chain_steps(first, last)
                O.run_steps(ref, sched, first, last)
                assert np.array_equal(state.cpu().numpy(), np.stack(ref)), (P, root, n, algo, first, last)
        plan.destroy()
        comm.destroy()


def test_runs_on_a_side_stream_and_back_to_back(V):
    """bcast_run on a stream of the caller's choice; two plans on the same
    buffers one after the other on that stream."""
    import torch
    w = I.workload("P24_n4M")
    state = H.device_buffers(w)
    comm = V.Comm([state[r].data_ptr() for r in range(w.P)], state.shape[1])
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        tuned = V.bcast_plan(comm, w.n, 1, w.root, V.TUNED, stream=side)
        native = V.bcast_plan(comm, w.n, 1, w.root, V.NATIVE, stream=side)
        V.bcast_run(tuned, stream=side)
        V.bcast_run(native, stream=side)
        V.bcast_run(tuned, stream=side)
    side.synchronize()
    want = np.stack(O.broadcast_definition(H.host_buffers(w), w.root, w.n))
    assert np.array_equal(state.cpu().numpy(), want)
    tuned.destroy()
    native.destroy()
    comm.destroy()


@pytest.mark.parametrize("executor", ["inline", "tables"])
def test_bcast_run_captured_into_a_callers_graph(V, executor):
    """The one-launch executor's bcast_run is one or three plain kernel launches, so
    a caller can capture it into a graph of their own (nothing in it allocates,
    synchronises or sets memory).  Three replays with the harness's eager work
    (re-poisoning, copies to the host, synchronisations) between them, each checked."""
    import torch
    w = I.workload("P24_n4M")
    state, comm, plan = make(V, w, O.TUNED, executor=executor)
    want = np.stack(O.broadcast_definition(H.host_buffers(w), w.root, w.n))
    V.bcast_run(plan)           # once outside, so that nothing is set up lazily under capture
    sync()
    assert np.array_equal(state.cpu().numpy(), want)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        V.bcast_run(plan)       # on the capturing stream (torch's current stream here)
    for replay in range(3):
        H.refill(state, w)
        sync()
        graph.replay()
        sync()
        assert np.array_equal(state.cpu().numpy(), want), (executor, replay)
    del graph
    plan.destroy()
    comm.destroy()


@pytest.mark.parametrize("executor", ALL_EXECUTORS)
@pytest.mark.parametrize("algo", ALGOS)
def test_graph_replays(V, algo, executor):
    """The same plan (its instantiated graph; for the default executor its one
    kernel) launched five times, with the harness's own
    eager work (re-poisoning, copies back to the host) and synchronisations
    between the launches: every replay must give the state the un-graphed steps
    give, which is the oracle's."""
    w = I.workload("P96_n12M_ragged")
    state, comm, plan = make(V, w, algo, executor=executor)
    want = np.stack(O.broadcast_definition(H.host_buffers(w), w.root, w.n))
    plan.run_steps(0, plan.info().n_steps)
    sync()
    assert np.array_equal(state.cpu().numpy(), want)
    for replay in range(5):
        H.refill(state, w)
        sync()
        plan.run()
        sync()
        assert np.array_equal(state.cpu().numpy(), want), (algo, executor, replay)
    plan.destroy()
    comm.destroy()


@pytest.mark.parametrize("P,n", [(1500, 3000), (2049, 40_000), (1024, 1_000_000)])
def test_many_ranks(V, P, n):
    """More ranks than one workgroup has lanes: the table kernels loop and carry."""
    w = I.Workload(f"many_{P}_{n}", P, P - 7, n, seed=4242 + P)
    state, comm, plan = make(V, w, O.TUNED, pad=0)
    sched = O.build_schedule(P, w.root, n, O.TUNED)
    check_tables(plan, sched)
    check_desc(plan, w)
    plan.run()
    sync()
    want = np.stack(O.broadcast_definition([H.host_row(w, r, state.shape[1]) for r in range(P)],
                                           w.root, n))
    assert np.array_equal(state.cpu().numpy(), want)
    plan.destroy()
    comm.destroy()


def test_largest_communicator(V):
    """VBCAST_MAX_RANKS ranks: too many rows for the oracle's Python loops to list in
    a test, so the counts are held to the closed forms the oracle is pinned to
    (bytes (P-1) n, messages P (P-1) minus the subtree savings, log2 P tree
    levels) and the final state to the definition of broadcast."""
    import torch
    P, n, root = 8192, 100_003, 8000
    w = I.Workload("max_ranks", P, root, n, seed=8192)
    stride = H.stride_of(n, 0)
    state = torch.zeros((P, stride), dtype=torch.uint8, device="cuda")
    msg = I.message_torch(w, "cuda")
    state[root, :n].copy_(msg)
    comm = V.Comm([state[r].data_ptr() for r in range(P)], stride)
    ss = -(-n // P)
    clen = [max(0, min(ss, n - c * ss)) for c in range(P)]
    span = lambda c: P if c == 0 else min(c & -c, P - c)
    scatter_bytes = sum(bin(c).count("1") * clen[c] for c in range(P))
    for algo, ex in ((V.TUNED, "chains"), (V.NATIVE, "chains"), (V.TUNED, "steps")):
        set_executor(V, ex)
        plan = V.bcast_plan(comm, n, 1, root, algo)
        set_executor(V, "chains")
        i = plan.info()
        assert (i.n_scatter_steps, i.n_steps, i.ss) == (13, 13 + P - 1, ss)
        assert i.scatter_bytes == scatter_bytes and i.pairing_mismatches == 0
        if algo == V.TUNED:
            assert i.bytes_moved == (P - 1) * n
        else:
            assert i.ring_bytes == (P - 1) * n and i.bytes_moved == (P - 1) * n + scatter_bytes
        # messages: empty chunks are never sent, so count the non-empty ones only
        if algo == V.NATIVE:
            empty = sum(1 for c in range(P) if clen[c] == 0)
            assert i.ring_msgs_issued == P * (P - 1)
            assert i.ring_rows == (P - empty) * (P - 1)
        else:
            assert i.ring_msgs_issued == P * (P - 1) - sum(span(c) - 1 for c in range(P))
        state.zero_()
        state[root, :n].copy_(msg)
        plan.run()
        sync()
        assert bool((state[:, :n] == msg).all()), (algo, ex)
        assert bool((state[:, n:] == 0).all())
        plan.destroy()
    comm.destroy()


@pytest.mark.parametrize("algo", ALGOS)
def test_offsets_beyond_4_GiB(V, algo):
    """Three ranks, a message of 6 GiB and a few bytes: the third chunk starts
    above 2^32, so offsets, tile and slab indices need their 64 bits.  Too large
    for host buffers: tables are compared in full; the state after the scatter,
    after the first ring step and at the end is compared on 8 KiB windows (at the
    start, around every chunk boundary, around 2^32, around the end of the message
    and at the end of the buffer) built from the oracle's chunk-ownership form;
    at the end every rank is also compared with the root on the device."""
    import torch
    P, root, n = 3, 1, 6 * 2**30 + 12_345
    w = I.Workload("beyond_4GiB", P, root, n, seed=4_294_967_296 + 7)
    state = H.device_buffers(w)
    stride = state.shape[1]
    comm = V.Comm([state[r].data_ptr() for r in range(P)], stride)
    sched = O.build_schedule(P, root, n, algo)
    ss = sched.ss
    assert 2 * ss > 2**32
    marks = [0, ss, 2 * ss, 2**32, n, stride]
    windows = sorted({(max(0, m - 4096), min(stride, m + 4096)) for m in marks})

    def check(k, where):
        has = O.ownership_after(sched, k)
        for r in range(P):
            for (a, b) in windows:
                want = I.bytes_numpy(w.seed, r + 1, b - a, start=a)
                for c in range(P):
                    d, cnt = O.chunk_extent(c, n, P)
                    lo, hi = max(a, d), min(b, d + cnt)
                    if lo < hi and (has[r, c] or r == root):
                        want[lo - a:hi - a] = I.bytes_numpy(w.seed, 0, hi - lo, start=lo)
                got = state[r, a:b].cpu().numpy()
                assert np.array_equal(got, want), (algo, where, r, a)

    plan = V.bcast_plan(comm, n, 1, root, algo)
    check_tables(plan, sched)
    check_desc(plan, w)
    check_chain(plan, sched)
    nsc, S = sched.n_scatter_steps, sched.n_steps
    for ex in EXECUTORS:
        H.refill(state, w)
        done = 0
        for stop in (nsc, nsc + 1, S):
            stepper(plan, ex)(done, stop)
            done = stop
            sync()
            check(stop, f"{ex}, after step {stop}")
    plan.destroy()
    for ex in EXECUTORS:
        set_executor(V, ex)
        plan = V.bcast_plan(comm, n, 1, root, algo)
        set_executor(V, "chains")
        H.refill(state, w)
        plan.run()
        sync()
        check(S, ex)
        for r in range(P):
            assert torch.equal(state[r, :n], state[root, :n]), (algo, ex, r)
        plan.destroy()
    comm.destroy()
    del state
    torch.cuda.empty_cache()


# ------------------------------------------------------------------ the large workload

@pytest.fixture(scope="module")
def big(V):
    """P = 513 ranks x 128 MiB: ~64 GiB of rank buffers, allocated once."""
    w = I.workload("P513_n128M")
    state = H.device_buffers(w, pad=64)
    yield w, state
    del state


@pytest.mark.parametrize("algo", ALGOS)
def test_large_workload_tables(V, big, algo):
    w, state = big
    comm = V.Comm([state[r].data_ptr() for r in range(w.P)], state.shape[1])
    plan = V.bcast_plan(comm, w.n, 1, w.root, algo)
    sched = O.build_schedule(w.P, w.root, w.n, algo)
    t = check_tables(plan, sched)
    check_desc(plan, w)
    check_chain(plan, sched)
    check_tiles(plan, t, [0, 9, 10, sched.n_steps - 1])
    plan.destroy()
    comm.destroy()


def expected_rows(w, sched, k, ranks, stride):
    """State of the given ranks after k steps, from the oracle's ownership form."""
    has = O.ownership_after(sched, k)
    msg = I.message_numpy(w)
    out = {}
    for r in ranks:
        row = H.host_row(w, r, stride)
        for c in range(w.P):
            if has[r, c]:
                d, cnt = O.chunk_extent(c, w.n, w.P)
                row[d:d + cnt] = msg[d:d + cnt]
        out[r] = row
    return out


@pytest.mark.parametrize("slab,hops", [(16384, "inline"), (32768, "inline"), (32768, "tables"), (65536, "chains")])
def test_large_slabs_on_a_large_message(V, slab, hops):
    """Slabs of 32 and 64 KiB are only kept for messages with enough of them (the
    launch halves them otherwise): 16 ranks, 96 MiB + 12345 bytes, so that the
    wavefront that has the turn copies its slab in several batches; with 16 KiB
    slabs the same message has the wavefronts take turns on whole slabs and meet
    slabs in which two chunks join.  The kernel works its hops out or looks them up
    (as it comes, a message of this length has it look them up).  Sampled ranks at
    sampled steps against the oracle's chunk-ownership form; then bcast_run, every
    rank against the message."""
    import torch
    w = I.Workload(f"slab_{slab}", 16, 5, (96 << 20) + 12345, seed=4242 + slab)
    V.vbcast_set_chain_slab_bytes(slab)
    set_executor(V, hops)
    try:
        state = H.device_buffers(w)
        stride = state.shape[1]
        comm = V.Comm([state[r].data_ptr() for r in range(w.P)], stride)
        msg_dev = I.message_torch(w, state.device)
        for algo in ALGOS:
            H.refill(state, w)
            tails_dev = state[:, w.n:].clone()
            plan = V.bcast_plan(comm, w.n, 1, w.root, algo)
            sched = O.build_schedule(w.P, w.root, w.n, algo)
            nsc, S = sched.n_scatter_steps, sched.n_steps
            done = 0
            ranks = [w.root, (w.root + 1) % w.P, (w.root + 8) % w.P, (w.root - 1) % w.P, 0]
            for stop in (nsc + 3, S - 2):
                plan.run_chain_steps(done, stop)
                done = stop
                sync()
                want = expected_rows(w, sched, stop, ranks, stride)
                for r in ranks:
                    assert np.array_equal(state[r].cpu().numpy(), want[r]), (slab, hops, algo, stop, r)
            H.refill(state, w)
            V.bcast_run(plan)
            sync()
            assert bool(torch.equal(state[:, w.n:], tails_dev)), (slab, algo)
            for r in range(w.P):
                assert bool(torch.equal(state[r, : w.n], msg_dev)), (slab, algo, r)
            plan.destroy()
        comm.destroy()
    finally:
        V.vbcast_set_chain_slab_bytes(DEFAULT_SLAB)
        set_executor(V, "chains")


@pytest.mark.parametrize("algo", ALGOS)
def test_large_workload_state(V, big, algo):
    """Sampled ranks compared whole at sampled steps (state from the oracle's
    chunk-ownership form), then every rank compared whole against the message
    after the graph run."""
    w, state = big
    H.refill(state, w)
    stride = state.shape[1]
    comm = V.Comm([state[r].data_ptr() for r in range(w.P)], stride)
    plan = V.bcast_plan(comm, w.n, 1, w.root, algo)
    # a broadcast this long looks its hops up: two table kernels, then the copy kernel
    assert plan.info().run_launches == 3
    sched = O.build_schedule(w.P, w.root, w.n, algo)
    nsc, S = sched.n_scatter_steps, sched.n_steps
    ranks = [w.root, (w.root + 1) % w.P, (w.root + 256) % w.P, (w.root + 384) % w.P,
             (w.root - 1) % w.P, 0, 300]
    for ex, stops in (("steps", [nsc, nsc + 1, nsc + 200, S - 1]), ("chains", [3, nsc + 2, S - 3])):
        H.refill(state, w)
        done = 0
        for stop in stops:
            stepper(plan, ex)(done, stop)
            done = stop
            sync()
            want = expected_rows(w, sched, stop, ranks, stride)
            for r in ranks:
                assert np.array_equal(state[r].cpu().numpy(), want[r]), (algo, ex, stop, r)
    plan.destroy()
    # the whole broadcast through the graph, from a fresh state, with either ring executor
    # Expected: the definition of broadcast - every rank's first n bytes are the
    # root's message, the bytes past it are still that rank's poison.  The 64 GiB
    # are compared where they are (torch, against the input generator's bytes on
    # the device); a sample of ranks also goes to the host and through numpy.
    import torch
    msg = I.message_numpy(w)
    msg_dev = I.message_torch(w, state.device)
    assert np.array_equal(msg_dev.cpu().numpy(), msg)
    on_host = sorted({w.root, 0, 1, 255, 257, 300, w.P - 1})
    for ex in EXECUTORS:
        set_executor(V, ex)
        plan = V.bcast_plan(comm, w.n, 1, w.root, algo)
        set_executor(V, "chains")
        H.refill(state, w)
        tails_dev = state[:, w.n:].clone()      # every rank's poison past the message, as filled
        V.bcast_run(plan)
        sync()
        assert bool(torch.equal(state[:, w.n:], tails_dev)), (algo, ex)
        for r in range(w.P):
            assert bool(torch.equal(state[r, : w.n], msg_dev)), (algo, ex, r)
        for r in on_host:
            got = state[r].cpu().numpy()
            assert np.array_equal(got[: w.n], msg), (algo, ex, r)
            assert np.array_equal(got[w.n:], H.host_tail(w, r, stride)), (algo, ex, r)
        plan.destroy()
    comm.destroy()
