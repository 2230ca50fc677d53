"""Sweep over the (process count, message size) points of the paper's three
experiments [Sec. V]: long messages on 16, 64 and 256 processes; 12288,
524287 and 1048576 bytes on 9, 17, 33, 65 and 129 processes; 12288 to 2560000
bytes on 129 processes.  For every point the native and the tuned broadcast
are timed as bcast_run calls on one GPU and set side by side.

    python -m paper_1603_06809_amd.sweep [--iters 100] [--markdown]
    python -m paper_1603_06809_amd.sweep --selection [--markdown]
    python -m paper_1603_06809_amd.sweep --smp [--ranks-per-node 24] [--markdown]
    python -m paper_1603_06809_amd.sweep --bandwidth-bound --iters 10 [--markdown]

``--selection`` times, on 16, 64 and 129 processes and sizes on both sides of
the two thresholds (12288 and 524288 bytes [Sec. V]), every broadcast algorithm
the library has - binomial tree, scatter + recursive doubling (power-of-two
process counts), scatter + ring native and tuned - and marks the one MPICH's
size / process-count rule selects [Abstract, Sec. I].  ``--smp`` sets the flat
tuned broadcast beside the multi-core-aware three-phase one [Sec. I] under the
blocked placement [Sec. V-A]: time, and messages and bytes between nodes.

Columns: bytes moved by each schedule and their ratio, the messages that would
cross a node boundary under the paper's blocked placement (24 per node), time per broadcast,
tuned/native time ratio, the paper's "bandwidth" figure - message bytes
per second of one broadcast, in MB/s with MB = 2**20 [Sec. V] - and two rates
for the tuned schedule: algorithmic (every row read once and written once,
wherever the read is served from; not an HBM rate) and HBM (the bytes that have
to cross the HBM interface over the time; small workloads that fit the 256 MB
Infinity Cache may not reach HBM at all, so for them this is an upper bound of
the traffic, not a measurement).  The paper's
protocol is a barrier followed by 100 iterations; here that is a stream
synchronisation followed by ``--iters`` bcast_run calls.
"""

from __future__ import annotations

import argparse
import json
import sys
import time


def points():
    long_sizes = [524_288, 1_048_576, 2_097_152, 4_194_304, 8_388_608, 16_777_216, 30_000_000]
    pts = [("lmsg-pof2", P, n) for P in (16, 64, 256) for n in long_sizes]
    pts += [("npof2", P, n) for n in (12_288, 524_287, 1_048_576) for P in (9, 17, 33, 65, 129)]
    pts += [("P129", 129, n) for n in (12_288, 49_152, 196_608, 524_288, 1_048_576, 2_560_000)]
    return pts


def selection(V, torch, iters: int, markdown: bool) -> int:
    sizes = [1024, 4096, 12_287, 12_288, 65_536, 262_144, 524_287, 524_288, 2_097_152]
    names = ["binomial", "scatter_rdb", "native", "tuned"]
    rows, all_ok = [], True
    for P in (16, 64, 129):
        for n in sizes:
            stride = (n + 255) // 256 * 256
            bufs = [torch.empty(stride, dtype=torch.uint8, device="cuda") for _ in range(P)]
            torch.manual_seed(P * 1_000_003 + n)
            bufs[0].random_()
            comm = V.Comm([b.data_ptr() for b in bufs], stride)
            chosen = V.ALGO_NAMES[V.vbcast_select_algo(n, P, True)]
            rec = {"P": P, "n": n, "selected": chosen}
            for name in names:
                if name == "scatter_rdb" and P & (P - 1):
                    rec[name] = None
                    continue
                for b in bufs[1:]:
                    b.zero_()
                plan = V.bcast_plan(comm, n, 1, 0, name)
                for _ in range(3):
                    V.bcast_run(plan)
                torch.cuda.synchronize()
                all_ok &= all(bool(torch.equal(b[:n], bufs[0][:n])) for b in bufs)
                t0 = time.perf_counter()
                for _ in range(iters):
                    V.bcast_run(plan)
                torch.cuda.synchronize()
                rec[name] = round((time.perf_counter() - t0) / iters * 1e6, 2)
                plan.destroy()
            comm.destroy()
            del bufs
            rows.append(rec)
            if not markdown:
                print(json.dumps(rec), flush=True)
    if markdown:
        print("| P | n | selected | binomial us | scatter + rec. doubling us | scatter + ring native us | tuned us |")
        print("|---|---|---|---|---|---|---|")
        for r in rows:
            cell = lambda k: "-" if r[k] is None else (f"**{r[k]}**" if r["selected"] == k else str(r[k]))
            print(f"| {r['P']} | {r['n']} | {r['selected']} | {cell('binomial')} | {cell('scatter_rdb')} | "
                  f"{cell('native')} | {cell('tuned')} |")
    return 0 if all_ok else 1


def smp(V, torch, iters: int, rpn: int, markdown: bool) -> int:
    rows, all_ok = [], True
    for (P, n) in [(48, 1_048_576), (64, 524_288), (64, 4_194_304), (129, 1_048_576), (256, 524_288),
                   (256, 4_194_304), (256, 30_000_000)]:
        stride = (n + 255) // 256 * 256
        bufs = [torch.empty(stride, dtype=torch.uint8, device="cuda") for _ in range(P)]
        torch.manual_seed(P * 1_000_003 + n)
        bufs[0].random_()
        comm = V.Comm([b.data_ptr() for b in bufs], stride)
        rec = {"P": P, "n": n, "ranks_per_node": rpn}
        for kind in ("flat", "three_phase"):
            for b in bufs[1:]:
                b.zero_()
            if kind == "flat":
                plan = V.bcast_plan(comm, n, 1, 0, "tuned")
                cens = [plan.census(rpn)]
            else:
                plan = V.bcast_plan_smp(comm, n, 1, 0, rpn, "tuned")
                # a sub-plan's ranks are positions in its sub-communicator: only the
                # second phase (one rank per node) crosses nodes, with every message
                cens = []
                for (phase, members, sub) in plan.subplans():
                    c = sub.census(1 if phase == 2 else len(members))
                    cens.append(c)
            for _ in range(3):
                plan.run()
            torch.cuda.synchronize()
            all_ok &= all(bool(torch.equal(b[:n], bufs[0][:n])) for b in bufs)
            t0 = time.perf_counter()
            for _ in range(iters):
                plan.run()
            torch.cuda.synchronize()
            rec[kind] = {
                "us": round((time.perf_counter() - t0) / iters * 1e6, 2),
                "inter_node_msgs": sum(c["scatter_inter_msgs"] + c["ring_inter_msgs"] for c in cens),
                "inter_node_bytes": sum(c["scatter_inter_bytes"] + c["ring_inter_bytes"] for c in cens),
            }
            plan.destroy()
        comm.destroy()
        del bufs
        rows.append(rec)
        if not markdown:
            print(json.dumps(rec), flush=True)
    if markdown:
        print("| P | n | flat tuned us | inter-node msgs | inter-node bytes | three-phase us | inter-node msgs | inter-node bytes |")
        print("|---|---|---|---|---|---|---|---|")
        for r in rows:
            f, t = r["flat"], r["three_phase"]
            print(f"| {r['P']} | {r['n']} | {f['us']} | {f['inter_node_msgs']} | {f['inter_node_bytes']} | "
                  f"{t['us']} | {t['inter_node_msgs']} | {t['inter_node_bytes']} |")
    return 0 if all_ok else 1


def bandwidth_bound(V, torch, iters: int, markdown: bool) -> int:
    """Few ranks, messages of 0.5-1 GiB: where the tuned schedule saves the largest
    share of the bytes [Sec. IV: the saving is (P/2) log2 P of P (P - 1) transfers]
    and the run is bound by bandwidth, not by the latency of dependent steps.  Both
    executors on the same buffers, native and tuned alternating."""
    rows, all_ok = [], True
    for (P, n) in [(10, 1 << 30), (24, 1 << 30), (64, 1 << 29)]:
        bufs = [torch.empty(n, dtype=torch.uint8, device="cuda") for _ in range(P)]
        bufs[0].random_()
        comm = V.Comm([b.data_ptr() for b in bufs], n)
        rec = {"P": P, "n": n}
        for ex in ("steps", "chains"):
            V.vbcast_set_ring_executor(V.RING_CHAINS if ex == "chains" else V.RING_STEPS)
            plans = {algo: V.bcast_plan(comm, n, 1, 0, algo) for algo in ("native", "tuned")}
            ms = {"native": [], "tuned": []}
            for algo, plan in plans.items():
                for b in bufs[1:]:
                    b.zero_()
                V.bcast_run(plan)
                torch.cuda.synchronize()
                all_ok &= all(bool(torch.equal(b, bufs[0])) for b in bufs)
            for rep in range(3):          # alternate, so that both see the same state of the device
                for algo, plan in plans.items():
                    V.bcast_run(plan)
                    torch.cuda.synchronize()
                    t0 = time.perf_counter()
                    for _ in range(iters):
                        V.bcast_run(plan)
                    torch.cuda.synchronize()
                    ms[algo].append((time.perf_counter() - t0) / iters * 1e3)
            rec[ex] = {algo: round(min(v), 4) for algo, v in ms.items()}
            rec["bytes_ratio"] = round(plans["tuned"].info().bytes_moved / plans["native"].info().bytes_moved, 4)
            rec[ex]["time_ratio"] = round(rec[ex]["tuned"] / rec[ex]["native"], 4)
            for plan in plans.values():
                plan.destroy()
        V.vbcast_set_ring_executor(V.RING_CHAINS)
        comm.destroy()
        del bufs
        torch.cuda.empty_cache()
        rows.append(rec)
        if not markdown:
            print(json.dumps(rec), flush=True)
    if markdown:
        print("| P | n | bytes tuned/native | steps executor: native ms | tuned ms | time ratio | "
              "chain executor: native ms | tuned ms | time ratio |")
        print("|---|---|---|---|---|---|---|---|---|")
        for r in rows:
            a, b = r["steps"], r["chains"]
            print(f"| {r['P']} | {r['n']} | {r['bytes_ratio']} | {a['native']} | {a['tuned']} | {a['time_ratio']} | "
                  f"{b['native']} | {b['tuned']} | {b['time_ratio']} |")
    return 0 if all_ok else 1


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--iters", type=int, default=100)
    ap.add_argument("--bandwidth-bound", action="store_true",
                    help="few ranks, messages of 0.5-1 GiB, both executors (use --iters 10)")
    ap.add_argument("--smp", action="store_true",
                    help="flat tuned broadcast against the three-phase one instead")
    ap.add_argument("--selection", action="store_true",
                    help="time every algorithm around the two size thresholds instead")
    ap.add_argument("--markdown", action="store_true")
    ap.add_argument("--ring-executor", choices=["chains", "steps"], default="chains")
    ap.add_argument("--ranks-per-node", type=int, default=24,
                    help="block size of the placement used for the inter-node census")
    args = ap.parse_args()

    import torch
    from . import vbcast as V

    if not torch.cuda.is_available():
        print("sweep: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    V.lib()
    V.vbcast_set_ring_executor(V.RING_CHAINS if args.ring_executor == "chains" else V.RING_STEPS)
    if args.bandwidth_bound:
        return bandwidth_bound(V, torch, args.iters, args.markdown)
    if args.selection:
        return selection(V, torch, args.iters, args.markdown)
    if args.smp:
        return smp(V, torch, args.iters, args.ranks_per_node, args.markdown)

    rows = []
    for (exp, P, n) in points():
        stride = (n + 255) // 256 * 256
        bufs = [torch.empty(stride, dtype=torch.uint8, device="cuda") for _ in range(P)]
        torch.manual_seed(P * 1_000_003 + n)
        bufs[0].random_()
        comm = V.Comm([b.data_ptr() for b in bufs], stride)
        rec = {"experiment": exp, "P": P, "n": n}
        ok = True
        for algo in ("native", "tuned"):
            plan = V.bcast_plan(comm, n, 1, 0, algo)
            for b in bufs[1:]:          # every schedule starts from buffers that lack the message
                b.random_()
            V.bcast_run(plan)
            torch.cuda.synchronize()
            ok &= all(bool(torch.equal(b[:n], bufs[0][:n])) for b in bufs)
            for _ in range(3):
                V.bcast_run(plan)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.iters):
                V.bcast_run(plan)
            torch.cuda.synchronize()
            us = (time.perf_counter() - t0) / args.iters * 1e6
            info = plan.info()
            cen = plan.census(args.ranks_per_node)
            # bytes that have to cross the HBM interface: with the one-launch executor the
            # writes and one read of the message (re-reads come from cache); with one
            # launch per step every row's read and write
            floor = (info.bytes_moved + n) if args.ring_executor == "chains" else 2 * info.bytes_moved
            rec[algo] = {"inter_node_msgs": cen["scatter_inter_msgs"] + cen["ring_inter_msgs"],
                         "inter_node_bytes": cen["scatter_inter_bytes"] + cen["ring_inter_bytes"],
                         "us": round(us, 2), "bytes_moved": int(info.bytes_moved),
                         "MBps": round(n / (us * 1e-6) / 2**20, 1),
                         "algorithmic_gbs": round(2.0 * info.bytes_moved / (us * 1e-6) / 1e9, 1),
                         "hbm_gbs": round(floor / (us * 1e-6) / 1e9, 1)}
            plan.destroy()
        rec["ok"] = ok
        rec["bytes_ratio"] = round(rec["tuned"]["bytes_moved"] / rec["native"]["bytes_moved"], 4)
        rec["time_ratio"] = round(rec["tuned"]["us"] / rec["native"]["us"], 4)
        rows.append(rec)
        comm.destroy()
        del bufs
        if not args.markdown:
            print(json.dumps(rec), flush=True)
    if args.markdown:
        print("| experiment | P | n | bytes tuned/native | inter-node msgs native | tuned | native us | "
              "tuned us | time tuned/native | native MB/s | tuned MB/s | tuned algorithmic GB/s | tuned HBM GB/s | ok |")
        print("|---|---|---|---|---|---|---|---|---|---|---|---|---|---|")
        for r in rows:
            print(f"| {r['experiment']} | {r['P']} | {r['n']} | {r['bytes_ratio']} | "
                  f"{r['native']['inter_node_msgs']} | {r['tuned']['inter_node_msgs']} | {r['native']['us']} | "
                  f"{r['tuned']['us']} | {r['time_ratio']} | {r['native']['MBps']} | {r['tuned']['MBps']} | "
                  f"{r['tuned']['algorithmic_gbs']} | {r['tuned']['hbm_gbs']} | {r['ok']} |")
    return 0 if all(r["ok"] for r in rows) else 1


if __name__ == "__main__":
    sys.exit(main())
