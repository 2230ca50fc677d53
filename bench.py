#!/usr/bin/env python3
"""Benchmark: simulated large-message broadcast of P virtual ranks on one GPU.

One step = one whole broadcast of the tuned schedule (table generation on the
device, all scatter levels, all ring steps: one graph launch) over rank buffers
already resident in device memory.  The native schedule is timed the same way
and reported beside it, with the bytes-moved ratio.

Two rates are reported and kept apart:

  algorithmic GB/s   2 * bytes_moved / time: every row of every step read once
                     and written once, wherever the read is served from.  This
                     is the paper's way of counting (message bytes over time,
                     Sec. V) applied to every transfer; it is NOT an HBM rate.
  HBM GB/s           the bytes that have to cross the HBM interface, over time.
                     One-launch executor: every rank's copy is written once and
                     the message is read once, (P - 1) * n + n bytes (tuned; the
                     native schedule also rewrites what the scatter delivered),
                     because a row's source is what the same lane wrote one hop
                     earlier and is re-read from cache.  Per-step executor:
                     every row read from and written to HBM, 2 * bytes_moved.
                     `value`, `pct_of_hbm_peak` and `roofline.frac` are this
                     rate; it cannot exceed the peak.

Prints one JSON line.  Besides the headline it carries
  roofline      the dominant kernel timed alone with HIP events on the launch
                stream; `traffic` is the counter-measured HBM bytes per launch
                read from the committed profile, or null when that profile was
                taken with another build of the kernel or another configuration
  per_config    the other four workloads, both schedules, default executor
  cpu_baseline  the CPU oracle on a bounded sample: one core, and the rows of a
                step spread over all host cores
  plain_fill_of_the_rank_buffers
                the same buffers written once by torch's fill, for scale
"""

from __future__ import annotations

import argparse
import hashlib
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, vendor figure

PROFILES = {
    "chains": os.path.join(ROOT, "profiles", "ring_chain_P513_n128M.md"),
    "steps": os.path.join(ROOT, "profiles", "step_copy_P513_n128M.md"),
}
KERNEL_SOURCES = {
    "chains": os.path.join(ROOT, "paper_1603_06809_amd", "csrc", "chain_kernels.hip"),
    "steps": os.path.join(ROOT, "paper_1603_06809_amd", "csrc", "copy_kernels.hip"),
}


def say(text):
    print(f"[bench] {text}", file=sys.stderr, flush=True)


def measured_traffic(executor: str, workload: str, unit_bytes: int, wgs_per_cu: int):
    """HBM bytes per launch of the dominant kernel as the committed profile
    records them (rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE), or None when the
    profile was taken on another workload, slab / tile size or workgroup count, or
    with another version of the kernel's source (its SHA-256 is in the profile)."""
    path = PROFILES[executor]
    try:
        text = open(path).read()
        src = open(KERNEL_SOURCES[executor], "rb").read()
    except OSError:
        return None, None
    m = re.search(r"```traffic\n(.*?)```", text, re.S)
    if not m:
        return None, None
    rec = dict(line.split("=", 1) for line in m.group(1).strip().splitlines() if "=" in line)
    rec = {k.strip(): v.strip() for k, v in rec.items()}
    want = {"workload": workload, "unit_bytes": str(unit_bytes), "workgroups_per_cu": str(wgs_per_cu),
            "kernel_source_sha256": hashlib.sha256(src).hexdigest()}
    for k, v in want.items():
        if rec.get(k) != v:
            return None, f"{os.path.relpath(path, ROOT)}: {k} differs (profile {rec.get(k)}, this run {v})"
    try:
        return float(rec["hbm_bytes_per_launch"]), os.path.relpath(path, ROOT)
    except (KeyError, ValueError):
        return None, None


def mem_available():
    try:
        with open("/proc/meminfo") as f:
            for line in f:
                if line.startswith("MemAvailable:"):
                    return int(line.split()[1]) * 1024
    except OSError:
        pass
    return None


def host_threads() -> int:
    try:
        return len(os.sched_getaffinity(0))
    except AttributeError:
        return os.cpu_count() or 1


def oracle_buffers(w, n):
    import numpy as np

    rng = np.random.default_rng(w.seed)
    bufs = [np.zeros(n, dtype=np.uint8) for _ in range(w.P)]
    bufs[w.root][:] = rng.integers(0, 256, n, dtype=np.uint8)
    for b in bufs:          # touch every page before timing
        b[::4096] = b[::4096]
    return bufs


def time_oracle(w, n):
    """The oracle's tuned schedule for a message of n bytes on numpy buffers, as
    the oracle executes it (one core)."""
    import numpy as np
    from oracle import bcast_oracle as O

    sched = O.build_schedule(w.P, w.root, n, O.TUNED)
    bufs = oracle_buffers(w, n)
    t0 = time.perf_counter()
    O.run_steps(bufs, sched)
    dt = time.perf_counter() - t0
    ok = all(np.array_equal(b, bufs[w.root]) for b in bufs)
    return sched, dt, ok


def time_oracle_all_cores(w, n, sched):
    """The same rows, every step's rows spread over all host cores by the oracle's
    C byte execution (one memcpy per row; valid because no row of a step reads
    what another row of the step writes, which is checked first)."""
    import numpy as np
    from oracle import native_rows as N

    independent = N.rows_independent(sched.steps)
    threads = min(N.host_threads(), host_threads())
    bufs = oracle_buffers(w, n)
    t0 = time.perf_counter()
    N.run_rows(bufs, sched.steps, threads, staged=not independent)
    dt = time.perf_counter() - t0
    ok = all(np.array_equal(b, bufs[w.root]) for b in bufs)
    return dt, ok, threads


def cpu_baseline(w, wanted_shrink: int, budget_s: float = 12.0):
    """The oracle as it stands on a bounded sample of the workload: same P and
    root, tuned schedule, the message shrunk by a power of two chosen so that the
    host buffers fit in 40 % of the available memory and - judged from a small
    pilot run - the one-core run takes about `budget_s` seconds at most.  Timed
    twice on that sample: one core (the plain numpy form), and the rows of every
    step spread over all host cores (the oracle's C byte execution)."""
    pilot_n = max(w.P, w.n // 64)
    sched, dt, _ = time_oracle(w, pilot_n)
    rate = sched.bytes_moved / dt                       # bytes moved per second
    shrink = max(1, wanted_shrink)
    avail = mem_available()
    while shrink < 64 and ((avail is not None and w.P * (w.n // shrink) > 0.4 * avail)
                           or (w.P - 1) * (w.n // shrink) > rate * budget_s):
        shrink *= 2
    n = max(w.P, w.n // shrink)
    sched, dt, ok = (sched, dt, _) if n == pilot_n else time_oracle(w, n)
    moved = sched.bytes_moved
    dt_all, ok_all, cores = time_oracle_all_cores(w, n, sched)
    note = (f"same P={w.P}, root={w.root}, tuned schedule, message shrunk {w.n // n}x to {n} bytes "
            f"({moved} bytes moved); value = 2 * bytes moved / time, every row read and written "
            f"by the host; one core {dt:.2f} s, {cores} threads {dt_all:.2f} s; result "
            f"{'equals' if ok and ok_all else 'DIFFERS FROM'} the broadcast definition")
    return {
        "value": round(2.0 * moved / dt / 1e9, 3),
        "unit": "GB/s",
        "cores": 1,
        "kind": "oracle",
        "sample": note,
        "all_cores": {"value": round(2.0 * moved / dt_all / 1e9, 3), "unit": "GB/s", "cores": cores,
                      "kind": "oracle's rows, one memcpy per row, rows of a step over all host threads"},
    }


def hbm_floor_bytes(info, executor: str, algo: str) -> float:
    """Bytes one broadcast has to move across the HBM interface."""
    if executor == "steps":
        return 2.0 * float(info.bytes_moved)
    if info.P < 2 or info.n == 0:
        return 0.0
    # every written byte reaches HBM once; reads: the message once (the root's
    # buffer), everything else comes back from cache
    return float(info.bytes_moved) + float(info.n)


def time_runs(torch, V, plan, steps: int, each_launch: bool = True):
    """K bcast_run calls between two synchronisations, host clock.  With
    `each_launch` an event between consecutive calls (on the launch stream) also
    gives each one's own time; without, nothing but the calls is enqueued (an
    event costs a few microseconds, which shows on the short broadcasts)."""
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)] if each_launch else []
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(steps):
        if each_launch:
            marks[k].record()
        V.bcast_run(plan)
    if each_launch:
        marks[steps].record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    each = sorted(marks[k].elapsed_time(marks[k + 1]) for k in range(steps)) if each_launch else []
    return dt / steps * 1e3, each


def spot_check(torch, V, I, w, bufs, plan, msg, stride: int) -> bool:
    """Poison three ranks again (their whole buffer), run the plan once, and
    compare them with the message and their tails with the poison: a run that
    did nothing, or wrote past the message, fails here."""
    ranks = sorted({(w.root + 1) % w.P, (w.root + w.P // 2) % w.P, (w.root + w.P - 1) % w.P} - {w.root})
    for r in ranks:
        bufs[r].copy_(I.poison_torch(w, r, stride, "cuda"))
    V.bcast_run(plan)
    torch.cuda.synchronize()
    ok = True
    for r in ranks:
        ok &= bool(torch.equal(bufs[r][: w.n], msg))
        if stride > w.n:
            ok &= bool(torch.equal(bufs[r][w.n:], I.poison_torch(w, r, stride, "cuda")[w.n:]))
    return ok


def small_configs(torch, V, I, executor: str, steps: int, warmup: int):
    """The other workloads (parity-test cases, timed here for the per-(P, n)
    table): both schedules, bcast_run back to back, the default executor (which
    for broadcasts this short is one kernel launch each)."""
    out = []
    for w in I.WORKLOADS[:-1]:
        stride = (w.n + 255) // 256 * 256
        bufs = [torch.empty(stride, dtype=torch.uint8, device="cuda") for _ in range(w.P)]
        msg = I.message_torch(w, "cuda")
        rec = {"workload": w.name, "P": w.P, "root": w.root, "n": w.n}
        ok = True
        for algo in ("native", "tuned"):
            for r, b in enumerate(bufs):
                b.copy_(I.poison_torch(w, r, stride, "cuda"))
            bufs[w.root][: w.n].copy_(msg)
            comm = V.Comm([b.data_ptr() for b in bufs], stride)
            plan = V.bcast_plan(comm, w.n, 1, w.root, algo)
            info = plan.info()
            V.bcast_run(plan)
            torch.cuda.synchronize()
            ok &= all(bool(torch.equal(b[: w.n], msg)) for b in bufs)
            for _ in range(warmup):
                V.bcast_run(plan)
            torch.cuda.synchronize()
            ms, _ = time_runs(torch, V, plan, max(steps, 200), each_launch=False)
            floor = hbm_floor_bytes(info, executor, algo)
            rec[f"ms_{algo}"] = round(ms, 5)
            rec[f"bytes_moved_{algo}"] = int(info.bytes_moved)
            rec["launches_per_bcast"] = int(info.run_launches)
            rec[f"algorithmic_gbs_{algo}"] = round(2.0 * info.bytes_moved / (ms * 1e-3) / 1e9, 1)
            rec[f"hbm_floor_frac_{algo}"] = round(floor / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
            plan.destroy()
            comm.destroy()
        rec["bytes_tuned_over_native"] = round(rec["bytes_moved_tuned"] / rec["bytes_moved_native"], 5)
        rec["time_tuned_over_native"] = round(rec["ms_tuned"] / rec["ms_native"], 4)
        rec["result_ok"] = ok
        out.append(rec)
        del bufs
    torch.cuda.empty_cache()
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="P513_n128M")
    ap.add_argument("--tile-bytes", type=int, default=0,
                    help="copy tile of the per-step executor (0 = library default)")
    ap.add_argument("--slab-bytes", type=int, default=0,
                    help="slab of the one-launch executor (0 = library default)")
    ap.add_argument("--pad", type=int, default=0, help="extra bytes at the end of every rank buffer")
    ap.add_argument("--ring-executor", choices=["chains", "steps"], default="chains")
    ap.add_argument("--chain-wgs-per-cu", type=int, default=0)
    ap.add_argument("--cpu-shrink", type=int, default=2,
                    help="the CPU oracle is timed on the same P and root with the message shrunk by this")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-per-config", action="store_true")
    ap.add_argument("--init", choices=["seeded", "fast"], default="seeded",
                    help="fast: poison from one torch random fill (for profiler runs)")
    ap.add_argument("--calibration-copy", type=float, default=0.0, metavar="GIB",
                    help="instead of the benchmark: five plain elementwise passes by torch over "
                         "tensors of this many GiB (dst = src + 1, every byte read once and written "
                         "once), the copy of known size that the HBM byte counters are scaled by")
    ap.add_argument("--allocations", type=int, default=2,
                    help="the rank buffers are allocated this many times, released in between, and "
                         "the last set is used (1 = use the process's first allocation)")
    args = ap.parse_args()

    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; the P virtual ranks all live in that "
              "GPU's memory and there is no multi-GPU path (--gpus must be 1)", file=sys.stderr)
        return 2

    import torch
    from paper_1603_06809_amd import inputs as I
    from paper_1603_06809_amd import vbcast as V

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    if args.calibration_copy > 0:
        nbytes = int(args.calibration_copy * 2**30) // 256 * 256
        src = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        src.view(torch.int64).random_()
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(5):
            torch.add(src, 1, out=dst)
        torch.cuda.synchronize()
        print(json.dumps({"calibration_copy_bytes_read": nbytes, "calibration_copy_bytes_written": nbytes,
                          "passes": 5, "kernel": "torch elementwise add, uint8, out-of-place"}))
        return 0
    V.lib()
    if args.tile_bytes:
        V.vbcast_set_tile_bytes(args.tile_bytes)
    if args.slab_bytes:
        V.vbcast_set_chain_slab_bytes(args.slab_bytes)
    if args.chain_wgs_per_cu:
        V.vbcast_set_chain_workgroups_per_cu(args.chain_wgs_per_cu)
    executor = args.ring_executor
    V.vbcast_set_ring_executor(V.RING_CHAINS if executor == "chains" else V.RING_STEPS)

    w = I.workload(args.workload)
    stride = (w.n + args.pad + 255) // 256 * 256
    # One allocation per rank, as P processes would have.  How fast the same
    # kernel runs depends on which physical memory the driver hands out (a
    # write-only sweep of the buffers shows the same spread, so it is the memory,
    # not the broadcast); the first set the first process on a fresh machine gets
    # has been the slowest in every run, the set it gets after releasing that one
    # among the fastest.  So the buffers are allocated, probed, released and
    # allocated again, and the probe of every set is reported.
    placement = []
    bufs = None
    for attempt in range(max(1, args.allocations)):
        if bufs is not None:
            del bufs
            torch.cuda.empty_cache()
        say(f"allocating {w.P} rank buffers of {stride} bytes (set {attempt + 1})")
        bufs = [torch.empty(stride, dtype=torch.uint8, device="cuda") for _ in range(w.P)]
        bufs[w.root].random_()
        comm = V.Comm([b.data_ptr() for b in bufs], stride)
        probe = V.bcast_plan(comm, w.n, 1, w.root, "tuned")
        for _ in range(3):
            V.bcast_run(probe)
        torch.cuda.synchronize()
        ms, _ = time_runs(torch, V, probe, 4)
        placement.append(round(ms, 3))
        say(f"set {attempt + 1}: {ms:.3f} ms per tuned broadcast")
        probe.destroy()
        comm.destroy()

    msg = I.message_torch(w, "cuda")
    if args.init == "fast":
        torch.manual_seed(w.seed)
        for b in bufs:
            b.view(torch.int64).random_()
    else:
        for r, b in enumerate(bufs):
            b.copy_(I.poison_torch(w, r, stride, "cuda"))
    bufs[w.root][: w.n].copy_(msg)
    torch.cuda.synchronize()
    say("buffers filled")
    comm = V.Comm([b.data_ptr() for b in bufs], stride)

    results = {}
    plans = {}
    ok = True
    for algo in ("native", "tuned"):
        t0 = time.perf_counter()
        plan = V.bcast_plan(comm, w.n, 1, w.root, algo)
        plan_ms = (time.perf_counter() - t0) * 1e3
        plans[algo] = plan
        info = plan.info()
        # correctness of this plan on its own: from poisoned buffers to the message
        V.bcast_run(plan)
        torch.cuda.synchronize()
        first_ok = all(bool(torch.equal(b[: w.n], msg)) for b in bufs)
        for _ in range(args.warmup):
            V.bcast_run(plan)
        torch.cuda.synchronize()
        ms, each = time_runs(torch, V, plan, args.steps)
        again_ok = spot_check(torch, V, I, w, bufs, plan, msg, stride)
        ok &= first_ok and again_ok
        say(f"{algo}: {ms:.3f} ms per broadcast; result {'ok' if first_ok and again_ok else 'WRONG'}")
        floor = hbm_floor_bytes(info, executor, algo)
        results[algo] = {
            "ms_per_bcast": round(ms, 4),
            "ms_median": round(each[len(each) // 2], 4),
            "ms_min": round(each[0], 4),
            "bytes_moved": int(info.bytes_moved),
            "hbm_bytes_floor": int(floor),
            "hbm_gbs": round(floor / (ms * 1e-3) / 1e9, 2),
            "algorithmic_gbs": round(2.0 * info.bytes_moved / (ms * 1e-3) / 1e9, 2),
            "bcast_bandwidth_MBps": round(w.n / (ms * 1e-3) / 2**20, 1),
            "plan_ms": round(plan_ms, 2),
            "n_steps": int(info.n_steps),
            "rows": int(info.scatter_rows + info.ring_rows),
            "launches_per_bcast": int(info.run_launches),
            "result_ok": bool(first_ok and again_ok),
        }
        if algo == "native":
            # the native runs leave every rank complete: poison them again so that the
            # tuned plan starts from what a broadcast starts from
            for r, b in enumerate(bufs):
                if r != w.root:
                    b.copy_(I.poison_torch(w, r, stride, "cuda"))
            torch.cuda.synchronize()

    # per-launch timing of the dominant kernel (the copy work after table generation), tuned plan,
    # with HIP events recorded on the launch stream around plain (un-graphed) launches
    plan = plans["tuned"]
    info = plan.info()
    nsc, S = info.n_scatter_steps, info.n_steps
    roof = None
    if S > nsc and info.ring_bytes > 0:
        reps = max(3, min(args.steps, 10))
        plan.run_timed()                      # warm
        ring_ms = [float(plan.run_timed()[2]) for _ in range(reps)]
        if executor == "chains":
            avg_ms = sum(ring_ms) / len(ring_ms)
            launches = 1
            alg_bytes = 2.0 * float(info.bytes_moved)     # the launch carries scatter and ring
            floor = hbm_floor_bytes(info, executor, "tuned")
            kernel = "ring_chain (scatter + ring in one launch, tuned)"
            unit_bytes, wgs = (args.slab_bytes or 16384), (args.chain_wgs_per_cu or 1)
        else:
            # the ring steps launched back to back between two events (an event
            # around every launch would add about 5 us to each of them)
            ring_bytes = plan.export().step_bytes[nsc:].astype(float)
            launches = int((ring_bytes > 0).sum())
            avg_ms = sum(ring_ms) / len(ring_ms) / launches
            alg_bytes = 2.0 * float(ring_bytes.sum()) / launches
            floor = alg_bytes
            kernel = "step_copy (one launch per ring step, tuned)"
            unit_bytes, wgs = int(info.tile_bytes), 0
        traffic, source = (None, "no counters for a padded layout") if args.pad else \
            measured_traffic(executor, w.name, unit_bytes, wgs)
        achieved = floor / (avg_ms * 1e-3) / 1e9
        roof = {
            "bound": "hbm", "kernel": kernel,
            "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBS, 4),
            "traffic": traffic, "traffic_source": source,
            "traffic_gbs": None if traffic is None else round(traffic / (avg_ms * 1e-3) / 1e9, 1),
            "hbm_bytes_floor_per_launch": int(floor),
            "algorithmic_bytes_per_launch": int(alg_bytes),
            "algorithmic_gbs": round(alg_bytes / (avg_ms * 1e-3) / 1e9, 1),
            "launches_per_bcast": launches, "avg_launch_us": round(avg_ms * 1e3, 2),
            "note": "achieved = hbm_bytes_floor_per_launch / avg_launch_us; algorithmic_gbs counts "
                    "every row's read and write whether or not it reaches HBM and may exceed the peak",
        }

    # the same broadcast with the other executor, for the record
    other = "steps" if executor == "chains" else "chains"
    V.vbcast_set_ring_executor(V.RING_STEPS if other == "steps" else V.RING_CHAINS)
    oplan = V.bcast_plan(comm, w.n, 1, w.root, "tuned")
    V.vbcast_set_ring_executor(V.RING_CHAINS if executor == "chains" else V.RING_STEPS)
    reps = max(3, min(args.steps, 10))
    other_ok = spot_check(torch, V, I, w, bufs, oplan, msg, stride)
    V.bcast_run(oplan)
    torch.cuda.synchronize()
    oms, _ = time_runs(torch, V, oplan, reps)
    ofloor = hbm_floor_bytes(info, other, "tuned")
    other_result = {
        "ring_executor": other, "schedule": "tuned", "runs": reps, "ms_per_bcast": round(oms, 4),
        "hbm_bytes_floor": int(ofloor),
        "hbm_gbs": round(ofloor / (oms * 1e-3) / 1e9, 2),
        "pct_of_hbm_peak": round(100.0 * ofloor / (oms * 1e-3) / 1e9 / HBM_PEAK_GBS, 2),
        "algorithmic_gbs": round(2.0 * info.bytes_moved / (oms * 1e-3) / 1e9, 2),
        "result_ok": bool(other_ok),
    }
    ok &= other_ok
    oplan.destroy()
    say(f"{other} executor, tuned: {oms:.3f} ms per broadcast")

    tuned, native = results["tuned"], results["native"]
    out = {
        "metric": "simulated bcast HBM GB/s (% of peak) + bytes-moved tuned/native, per (P, n)",
        "value": tuned["hbm_gbs"],
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": tuned["ms_per_bcast"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u8",
        "data": "synthetic",
        "config": {
            "workload": f"{w.name}: P={w.P} virtual ranks, root={w.root}, n={w.n} bytes, "
                        "seeded uniform random bytes; step = one tuned broadcast = one bcast_run "
                        + ("(one kernel: scatter + ring, schedule worked out in the kernel)"
                           if tuned["launches_per_bcast"] == 1 else
                           f"({tuned['launches_per_bcast']} kernels: table generation, then scatter + ring)"),
            "tile_bytes": int(info.tile_bytes),
            "slab_bytes": args.slab_bytes or 16384,
            "ring_executor": executor,
            "rank_stride_bytes": stride,
        },
        "value_is": f"HBM bytes that have to move ({tuned['hbm_bytes_floor']} per tuned broadcast with the "
                    f"{executor} executor) / ms_per_step; the 70 % target is judged on pct_of_hbm_peak",
        "pct_of_hbm_peak": round(100.0 * tuned["hbm_gbs"] / HBM_PEAK_GBS, 2),
        "algorithmic_gbs": tuned["algorithmic_gbs"],
        "bytes_moved_tuned_over_native": round(tuned["bytes_moved"] / native["bytes_moved"], 5),
        "time_tuned_over_native": round(tuned["ms_per_bcast"] / native["ms_per_bcast"], 4),
        "tuned": tuned,
        "native": native,
        "result_ok": bool(ok),
        "rank_buffer_sets_probed_ms": placement,
        "paper_context": "paper reports 2-54% bandwidth gain of tuned over native on a Cray XC40 "
                         "(other hardware, MPI over a network); not comparable",
        "other_executor": other_result,
        "roofline": roof,
    }
    for p in plans.values():
        p.destroy()
    comm.destroy()
    # for scale: the same rank buffers written once, one after the other, by torch's fill
    # (everything that had to be checked has been; the buffers are not used again)
    fill_ms = []
    for _ in range(3):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for b in bufs:
            b.fill_(0)
        e1.record()
        torch.cuda.synchronize()
        fill_ms.append(e0.elapsed_time(e1))
    out["plain_fill_of_the_rank_buffers"] = {
        "ms": round(min(fill_ms), 3),
        "write_gbs": round(w.P * stride / (min(fill_ms) * 1e-3) / 1e9, 1),
        "note": "P fill launches writing every rank buffer once; no broadcast, for scale only",
    }
    del bufs
    torch.cuda.empty_cache()
    if not args.no_per_config:
        say("timing the other workloads")
        out["per_config"] = small_configs(torch, V, I, executor, args.steps, args.warmup)
        ok &= all(r["result_ok"] for r in out["per_config"])
        out["per_config"].append({
            "workload": w.name, "P": w.P, "root": w.root, "n": w.n,
            "ms_native": native["ms_per_bcast"], "ms_tuned": tuned["ms_per_bcast"],
            "bytes_moved_native": native["bytes_moved"], "bytes_moved_tuned": tuned["bytes_moved"],
            "algorithmic_gbs_native": native["algorithmic_gbs"], "algorithmic_gbs_tuned": tuned["algorithmic_gbs"],
            "hbm_floor_frac_native": round(native["hbm_gbs"] / HBM_PEAK_GBS, 4),
            "hbm_floor_frac_tuned": round(tuned["hbm_gbs"] / HBM_PEAK_GBS, 4),
            "bytes_tuned_over_native": out["bytes_moved_tuned_over_native"],
            "time_tuned_over_native": out["time_tuned_over_native"],
            "result_ok": bool(tuned["result_ok"] and native["result_ok"]),
        })
        out["result_ok"] = bool(ok)
    if not args.no_cpu:
        say("timing the CPU oracle on the bounded sample")
        out["cpu_baseline"] = cpu_baseline(w, args.cpu_shrink)
    print(json.dumps(out))
    return 0 if ok else 1


if __name__ == "__main__":
    sys.exit(main())
