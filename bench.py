#!/usr/bin/env python3
"""Throughput of the whole prioritized-update step on one MI355X.

A "step" is one pass of the full hot path over one batch: dedup of the lookahead IDs, collision
split and class order, priority pass (gradient segment-reduce fused with row-wise Adagrad on the
collision rows), deferred pass (the same on the exclusive rows) on its own stream, and the jagged
gather of the lookahead batch.  The workload is
BASELINE configs[1] (one 4M x 128 fp32 table shard, batch 1024, power-law UIH lengths, Zipf(1.05)
IDs); its two consecutive iterations are stepped back and forth (t=0 with lookahead 1, then t=1
with lookahead 0, ...) so that every step consumes the layout and class order an earlier step's index half produced,
as in steady-state training (default schedule: the index half of iteration s+2 is enqueued on the
library's index streams before the pipelined call of iteration s).  Inputs are resident in HBM
before the timed region.

Prints ONE JSON line: rows/s, ms/step, the roofline of the dominant kernel (HIP events around it
inside the timed steps) and the CPU oracle timed on this machine's host cores.
"""
from __future__ import annotations

import argparse
import math
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E peak

# HBM bytes per launch measured with hardware counters (FETCH_SIZE, WRITE_SIZE, each scaled by what
# the same counter reads for a plain copy of known size) in separate counter runs of this file on
# the default workload; the runs and their figures are summarised under profiles/.
MEASURED_TRAFFIC_BYTES = {
    ("configs[1]", "class_pass_kernel (priority pass)"): 143.2e6,
    ("configs[1]", "class_pass_kernel (deferred pass)"): 109.5e6,
    ("configs[1]", "gather_kernel"): 202.2e6,
    # the eleven index kernels of one iteration (half of what a chain for two iterations moves)
    ("configs[1]", "index kernels"): 40.0e6,
}


def algorithmic_bytes(n_t, u_t, n_t1, u_t1, dim, w):
    """Compulsory bytes of one step (each distinct row counted once per pass; the sort's
    internal passes and the reduced-gradient round trip are NOT counted)."""
    unique = 8 * n_t1 + 8 * u_t1 + 4 * n_t1
    split = 16 * (u_t + u_t1)
    gather = 8 * n_t1 + u_t1 * dim * w + n_t1 * dim * w
    reduce_update = n_t * dim * 4 + 4 * n_t + 2 * u_t * dim * w + 8 * u_t + 8 * u_t
    return {"unique": unique, "split": split, "gather": gather, "reduce_update": reduce_update,
            "total": unique + split + gather + reduce_update}


def group_tables(tabs, G):
    """The tables of a shard in G groups (one context, stream and call sequence each).  Tables of one row width
    share the launches of their class passes and gathers inside a call, so a group should hold few widths, and
    the groups run side by side, so they should be about equally heavy: every assignment is tried (a shard has a
    handful of tables) and the one with the smallest (heaviest group / mean group + 0.05 x launch classes) kept."""
    import itertools
    if G == 1 or len(tabs) > 12:
        return [tabs[g::G] for g in range(G)]
    load = [sum(t.n) * t.dim * t.w for t in tabs]
    mean = sum(load) / G
    best, best_cost = None, None
    for assign in itertools.product(range(G), repeat=len(tabs)):
        if len(set(assign)) < G:
            continue
        heavy = max(sum(l for l, a in zip(load, assign) if a == g) for g in range(G))
        classes = len({(a, t.dim * t.w) for a, t in zip(assign, tabs)})
        cost = heavy / mean + 0.05 * classes
        if best_cost is None or cost < best_cost - 1e-12:
            best, best_cost = assign, cost
    return [[t for t, a in zip(tabs, best) if a == g] for g in range(G)]


def bench_tables(args, cfg) -> int:
    """Several tables per shard (BASELINE configs[2]): one independent problem per table (table-local IDs, own
    buffers), ONE context and stream for the shard: per step the index halves of all tables two iterations
    ahead in shared launches (fs_step_forward_ahead_batch) and one fs_prioritized_step_pipelined_multi."""
    import numpy as np
    import torch
    import paper_2604_24073_amd as fs
    from fs_workloads import make_iterations, hash_init_rows, compact_rows

    dev = torch.device("cuda:0")
    its_all = make_iterations(cfg, iterations=2)
    D = 2                                      # iterations between issuing the index halves and stepping them
    L, P = 1 + D + 3, 1 + D + 2
    period = math.lcm(L, P, 2)
    if len(cfg.tables) > min(fs.FS_MAX_AHEAD_BATCH, fs.FS_MAX_STEP_TABLES):
        print("bench.py: more tables per shard than one call takes", file=sys.stderr)
        return 4

    class T:
        pass

    tabs = []
    for ti, tab in enumerate(cfg.tables):
        t = T()
        t.tab, t.its = tab, [its_all[0][ti], its_all[1][ti]]
        t.dim, t.w = tab.dim, (4 if tab.dtype == "f32" else 2)
        t.n = [int(it.values.shape[0]) for it in t.its]
        tabs.append(t)
    # the tables of the shard in G groups, each with its own context and stream (G = 1: one call per step for all)
    G = max(1, min(args.table_groups, len(tabs)))
    groups = group_tables(tabs, G)
    ctxs = [fs.Context(max_ids=max(max(t.n) for t in grp), max_dim=max(t.dim for t in grp)) for grp in groups]
    streams = [torch.cuda.Stream() for _ in groups]
    ctx = ctxs[0]
    for t in tabs:
        tab = t.tab
        tdtype = torch.float32 if tab.dtype == "f32" else torch.bfloat16
        t.table = torch.empty((tab.num_rows, t.dim), dtype=tdtype, device=dev)
        fs.fs_init_table_hash(ctx, t.table)
        t.state = torch.zeros(tab.num_rows, dtype=torch.float32, device=dev)
        t.vals = [torch.from_numpy(it.values).to(dev) for it in t.its]
        t.offs = [torch.from_numpy(it.offsets).to(dev) for it in t.its]
        t.grads = [torch.from_numpy(it.grads).to(dev) for it in t.its]
        nmax = max(t.n)
        t.layouts = [fs.alloc_layout(nmax, dev, inverse=False) for _ in range(L)]
        t.splits = [fs.alloc_split(nmax, nmax, dev) for _ in range(P)]
        t.embs = [torch.empty((t.n[0], t.dim), dtype=tdtype, device=dev),
                  torch.empty((t.n[1], t.dim), dtype=tdtype, device=dev)]

        def args_for(s, t=t):
            lay = dict(t.layouts[s % L]); lay["n"] = t.n[s % 2]
            nb = (s + 1) % 2
            return fs.make_step_args(t.table, t.state, cfg.lr, cfg.eps, lay, t.grads[s % 2], t.vals[nb], t.offs[nb],
                                     t.layouts[(s + 1) % L], t.splits[s % P], None, t.embs[nb])

        t.args = [args_for(s) for s in range(period)]
    # one contiguous array of records per group and iteration of the period: what the two calls of a step take
    step_records = [[fs.step_args_array([t.args[s] for t in grp]) for s in range(period)] for grp in groups]
    torch.cuda.synchronize()
    stepped = [False]

    def ahead(s):
        for c, st, rec in zip(ctxs, streams, step_records):
            fs.fs_step_forward_ahead_batch(c, rec[s % period], stream=fs.FS_STREAM_LAST_STEP if stepped[0] else st)

    def run(k0, k):
        for s in range(k0, k0 + k):
            ahead(s + D)
            for c, st, rec in zip(ctxs, streams, step_records):
                fs.fs_prioritized_step_pipelined_multi(c, rec[s % period], rec[(s + 1) % period], stream=st)
            stepped[0] = True

    def join_all(check=False):
        for c, st in zip(ctxs, streams):
            if check:
                assert fs.fs_check_async(c, st) == fs.FS_OK, c.last_error()
            else:
                fs.fs_step_join(c, st)

    for c, st, grp in zip(ctxs, streams, groups):
        for t in grp:
            fs.fs_unique_ids(c, t.vals[0], t.tab.num_rows, out=t.layouts[0], stream=st)
    for s in range(D):
        ahead(s)
    run(0, 1)
    cpu_s, u_all = 0.0, []
    join_all(check=True)
    for ti, t in enumerate(tabs):
        t.u = [int(t.layouts[0]["n_unique"].item()), int(t.layouts[1]["n_unique"].item())]
        u_all.append(t.u)
        if not args.no_cpu_baseline:
            import oracle as O
            touched, (v0c, v1c) = compact_rows([t.its[0].values, t.its[1].values])
            w0 = hash_init_rows(touched, t.dim, t.tab.dtype)
            times = []
            for _ in range(3):
                t_ref, s_ref = w0.copy(), np.zeros(len(touched), np.float32)
                lay0 = O.unique_ids(v0c, len(touched))
                t0 = time.perf_counter()
                O.step(t_ref, s_ref, lay0, t.its[0].grads, v1c, t.its[1].offsets, cfg.lr, cfg.eps)
                times.append(time.perf_counter() - t0)
            got_rows = t.table[torch.from_numpy(touched).to(dev)].float().cpu().numpy()
            if not (t.u[0] == len(lay0["unique"]) and np.allclose(got_rows, t_ref, rtol=1e-5, atol=1e-6)):
                print(f"bench.py: GPU step of table {ti} does not match the oracle", file=sys.stderr)
                return 4
            cpu_s += statistics.median(times)
    run(1, args.warmup)
    join_all()
    torch.cuda.synchronize()
    k0 = 1 + args.warmup
    fs.fs_ctx_set_kernel_timing(ctx, args.steps, args.time_every)
    for c in ctxs:
        fs.fs_ctx_host_times(c, reset=True)
    t0 = time.perf_counter()
    run(k0, args.steps)
    t_enq = time.perf_counter() - t0
    join_all()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    names = ("wait_side_thread", "fork_and_post", "wait_side_stream", "priority_and_gather", "index_thread_enqueue",
             "side_thread_enqueue")
    host_phases = []
    for c in ctxs:
        ht = fs.fs_ctx_host_times(c)
        host_phases.append({k: ht[i] / ht[6] for i, k in enumerate(names)} if ht[6] > 0 else None)
    join_all(check=True)
    kinds = {"gather": fs.FS_TIME_GATHER, "priority_pass": fs.FS_TIME_UPDATE_CO, "deferred_pass": fs.FS_TIME_UPDATE_EX}
    kernel_ms = {}
    for name, kind in kinds.items():
        vals = fs.fs_ctx_get_kernel_timing(ctx, kind, args.steps)
        kernel_ms[name] = (sum(vals) / len(vals)) if vals else None
    rows = sum(t.u[s % 2] for t in tabs for s in range(k0, k0 + args.steps))
    step_bytes = 0.0
    for t in tabs:
        by = [algorithmic_bytes(t.n[0], t.u[0], t.n[1], t.u[1], t.dim, t.w),
              algorithmic_bytes(t.n[1], t.u[1], t.n[0], t.u[0], t.dim, t.w)]
        step_bytes += sum(by[s % 2]["total"] for s in range(k0, k0 + args.steps)) / args.steps
    ms_per_step = elapsed / args.steps * 1e3
    step_gbps = step_bytes / (ms_per_step * 1e-3) / 1e9
    # the event pairs of the first group's context bracket everything that call enqueues of one kind: the gathers
    # (or class passes of one class) of all its tables, one launch per row width
    grp0 = groups[0]
    roofline = None
    if kernel_ms.get("gather"):
        gbytes = sum((algorithmic_bytes(t.n[0], t.u[0], t.n[1], t.u[1], t.dim, t.w)["gather"] +
                      algorithmic_bytes(t.n[1], t.u[1], t.n[0], t.u[0], t.dim, t.w)["gather"]) / 2 for t in grp0)
        widths = len({t.dim * t.w for t in grp0})
        gb = gbytes / (kernel_ms["gather"] * 1e-3) / 1e9
        roofline = {"bound": "hbm", "kernel": f"gather_kernel (the {len(grp0)} tables of group 0: {widths} launch(es), "
                                              "bracketed together)",
                    "achieved": gb, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": gb / HBM_PEAK_GBPS, "traffic": None,
                    "avg_launch_us": kernel_ms["gather"] * 1e3, "algorithmic_bytes_per_launch": gbytes}
    out = {
        "metric": "unique embedding rows updated/sec + achieved HBM GB/s (% of peak), 1 GPU",
        "value": rows / elapsed, "unit": "rows/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"configs[{cfg.index}] {cfg.name}: {len(tabs)} tables per shard, rows "
                               f"{[t.tab.num_rows for t in tabs]}, dims {[t.dim for t in tabs]}, batch {cfg.batch}, "
                               f"{cfg.length_rule} UIH lengths [{cfg.length_lo},{cfg.length_hi}], a step = one "
                               "iteration of every table; 2 consecutive iterations stepped back and forth",
                   "ids_per_iteration": [t.n for t in tabs], "unique_rows": u_all},
        "schedule": f"the tables in {G} group(s), each with a context and a stream: per step and group one multi-table "
                    "pipelined call + the index halves of its tables two iterations ahead in shared launches",
        "table_groups": [[tabs.index(t) for t in grp] for grp in groups],
        "host_phase_us_per_step_and_group": host_phases,
        "host_enqueue_us_per_step": t_enq / args.steps * 1e6,
        "step_algorithmic_bytes": step_bytes, "step_algorithmic_GBps": step_gbps,
        "step_frac_of_hbm_peak": step_gbps / HBM_PEAK_GBPS,
        "kernel_avg_us": {k: (v * 1e3 if v is not None else None) for k, v in kernel_ms.items()},
        "roofline": roofline,
        "cpu_baseline": None if args.no_cpu_baseline else {
            "value": sum(t.u[0] for t in tabs) / cpu_s, "unit": "rows/s", "cores": 1, "kind": "oracle",
            "ms_per_step": cpu_s * 1e3,
            "sample": "the full step t=0 of every table, median of 3 runs each of the single-threaded C oracle on "
                      "tables holding only the touched rows", "host_cpus": os.cpu_count()},
    }
    print(json.dumps(out))
    for c in ctxs:
        c.close()
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=1, help="index into the workload configurations (default 1)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-isolated", action="store_true",
                    help="skip the extra launches that time every kernel alone on the chip after the timed steps")
    ap.add_argument("--time-every", type=int, default=16,
                    help="bracket the kernels of one timed step in this many with HIP event pairs")
    ap.add_argument("--calibration-copy", type=int, default=0, metavar="MiB",
                    help="also launch one plain copy of this many MiB before the steps: the known-size dispatch that "
                         "hardware byte counters are scaled by in a counter run")
    ap.add_argument("--ahead-order", choices=["last_step", "stream"], default="last_step",
                    help="what an ahead-of-time dedup is ordered after: the start of the most recent pipelined call "
                         "(no event on the caller's stream, six layout buffers) or the caller's stream as it stands "
                         "(one more event per step on it, five layout buffers)")
    ap.add_argument("--ahead", choices=["index", "dedup", "none"], default="index",
                    help="pipelined mode, what runs ahead of time on the index streams: the whole index half of an "
                         "iteration two iterations ahead (default), only the dedup of the lookahead IDs, or nothing "
                         "(the side stream of the step call does it all)")
    ap.add_argument("--ahead-batch", type=int, default=2, metavar="K",
                    help="with --ahead index: index halves of K consecutive iterations share their launches "
                         "(fs_step_forward_ahead_batch), issued K+1 iterations before the first of them is stepped; "
                         "1 = one chain of launches per iteration")
    ap.add_argument("--table-groups", type=int, default=2, metavar="G",
                    help="configurations with several tables per shard: the tables are stepped in G groups, each "
                         "with its own context and stream (1 = one call per step for all tables; 2 measured best: "
                         "two tables' passes side by side, and no more streams than the hardware has queues for)")
    ap.add_argument("--two-part", action="store_true",
                    help="the lookup in the two parts of Algorithm 2 (fs_prioritized_step_two_part_multi): exclusive "
                         "rows of the batch after next fetched on the side stream, collision rows after the priority pass")
    ap.add_argument("--no-widening", action="store_true",
                    help="skip the load balancer's data path (partitioner and jagged shuffles) timed after the step")
    ap.add_argument("--keep-reduced", action="store_true",
                    help="also write the summed gradients to memory in the timed steps (the step itself does not "
                         "need them there)")
    ap.add_argument("--mode", choices=["pipelined", "graph", "sequential"], default="pipelined",
                    help="pipelined (default): index half of step s+1 beside the gradient half of step s, "
                         "eager launches; graph: the same step replayed as a HIP graph (measured slower: the "
                         "replay serialises its cross-stream edges); sequential: every step self-contained")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (one embedding-table shard, no collectives); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    import paper_2604_24073_amd as fs
    from fs_workloads import CONFIGS, make_iterations, hash_init_rows, compact_rows

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    cfg = CONFIGS[args.config]
    if len(cfg.tables) != 1:
        return bench_tables(args, cfg)
    tab = cfg.tables[0]
    its = [x[0] for x in make_iterations(cfg, iterations=2)]
    dim, w = tab.dim, (4 if tab.dtype == "f32" else 2)
    tdtype = torch.float32 if tab.dtype == "f32" else torch.bfloat16

    n = [int(it.values.shape[0]) for it in its]
    ctx = fs.Context(max_ids=max(n), max_dim=dim)
    table = torch.empty((tab.num_rows, dim), dtype=tdtype, device=dev)
    fs.fs_init_table_hash(ctx, table)
    state = torch.zeros(tab.num_rows, dtype=torch.float32, device=dev)
    d_vals = [torch.from_numpy(it.values).to(dev) for it in its]
    d_offs = [torch.from_numpy(it.offsets).to(dev) for it in its]
    d_grads = [torch.from_numpy(it.grads).to(dev) for it in its]

    # Buffers.  The index half of step s+1 runs beside the gradient half of step s, and with
    # ahead-of-time dedups the layout of batch s+3 is being written meanwhile: five layout buffers
    # in rotation (six when the dedup is only ordered after the start of the previous call, three
    # without ahead-of-time dedups), three split/class buffers.  The two batches alternate, so the
    # argument records repeat with period lcm(L, 3, 2).
    pipelined = args.mode in ("pipelined", "graph")
    ahead = args.mode == "pipelined" and args.ahead != "none"
    index_ahead = ahead and args.ahead == "index"
    last_step_order = ahead and args.ahead_order == "last_step"
    K = max(1, min(args.ahead_batch, fs.FS_MAX_AHEAD_BATCH)) if index_ahead else 1
    D = K + 1                                  # iterations between issuing a batch and stepping its first record
    L = (K + D + 3 if index_ahead else (6 if last_step_order else 5)) if ahead else 3
    P = K + D + 2 if index_ahead else 3
    period = math.lcm(L, P, 2)
    nmax = max(n)
    layouts = [fs.alloc_layout(nmax, dev, inverse=args.two_part) for _ in range(L)]   # only the two-part lookup reads it
    splits = [fs.alloc_split(nmax, nmax, dev) for _ in range(P)]
    reduced = [torch.empty((nmax, dim), dtype=torch.float32, device=dev) for _ in range(2)]
    embs = [torch.empty((n[0], dim), dtype=tdtype, device=dev), torch.empty((n[1], dim), dtype=tdtype, device=dev)]

    def args_for(s, with_reduced):
        lay = dict(layouts[s % L]); lay["n"] = n[s % 2]
        nb = (s + 1) % 2
        return fs.make_step_args(table, state, cfg.lr, cfg.eps, lay, d_grads[s % 2], d_vals[nb], d_offs[nb],
                                 layouts[(s + 1) % L], splits[s % P], reduced[s % 2] if with_reduced else None,
                                 embs[nb])

    check_args = [args_for(s, True) for s in range(period)]
    step_args = check_args if args.keep_reduced else [args_for(s, False) for s in range(period)]
    fs.fs_unique_ids(ctx, d_vals[0], tab.num_rows, out=layouts[0])
    graphs = None
    arrays = {id(r): [fs.step_args_array([x]) for x in r] for r in (check_args, step_args)} if args.two_part else {}

    stepped = [False]

    def order():
        return fs.FS_STREAM_LAST_STEP if (last_step_order and stepped[0]) else None

    def dedup_ahead(s):
        if ahead and not index_ahead:
            fs.fs_unique_ids_ahead(ctx, d_vals[s % 2], tab.num_rows, layouts[s % L], stream=order())

    def index_half_ahead(first, records):
        # the index halves of iterations first .. first+K-1, when `first` starts a batch
        if index_ahead and first >= 0 and first % K == 0:
            fs.fs_step_forward_ahead_batch(ctx, [records[(first + k) % period] for k in range(K)], stream=order())

    def run(k0, k, records=None):
        records = records or step_args
        for s in range(k0, k0 + k):
            if graphs is not None:
                fs.fs_graph_launch(ctx, graphs[s % period])
            elif pipelined:
                dedup_ahead(s + 3)
                index_half_ahead(s + D, records)
                if args.two_part:
                    arr = arrays[id(records)]
                    fs.fs_prioritized_step_two_part_multi(ctx, arr[s % period], arr[(s + 1) % period])
                else:
                    fs.fs_prioritized_step_pipelined(ctx, records[s % period], records[(s + 1) % period])
                stepped[0] = True
            else:
                fs.fs_prioritized_step(ctx, records[s % period])

    if args.calibration_copy > 0:
        src = torch.empty(args.calibration_copy << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        fs.fs_stream_copy(ctx, src, dst)
        torch.cuda.synchronize()
        del src, dst

    # ---- one untimed step from the fresh table, checked against the oracle on the touched rows
    cpu_baseline = None
    if pipelined and index_ahead:
        for first in range(0, D):                      # the batches a loop that had run forever would have issued
            index_half_ahead(first, check_args)
    elif pipelined:
        dedup_ahead(1)
        fs.fs_step_forward(ctx, check_args[0])         # primes the pipeline: layout 1, split and class order 0
        dedup_ahead(2)
    run(0, 1, check_args)
    assert fs.fs_check_async(ctx) == fs.FS_OK, ctx.last_error()
    u = [int(layouts[0]["n_unique"].item()), int(layouts[1]["n_unique"].item())]
    counts0 = splits[0]["counts"].cpu().numpy().tolist()
    if not args.no_cpu_baseline:
        import oracle as O
        touched, (v0c, v1c) = compact_rows([its[0].values, its[1].values])
        w0 = hash_init_rows(touched, dim, tab.dtype)
        if tab.dtype == "bf16":
            w0 = (w0.view(np.uint32) >> np.uint32(16)).astype(np.uint16)
        reps, times, want = 0, [], None
        t_budget = time.perf_counter()
        while reps < 3 or (time.perf_counter() - t_budget < 10.0 and reps < 100):
            t_ref, s_ref = w0.copy(), np.zeros(len(touched), np.float32)
            lay0 = O.unique_ids(v0c, len(touched))          # produced by the previous step: not timed
            t0 = time.perf_counter()
            want = O.step(t_ref, s_ref, lay0, its[0].grads, v1c, its[1].offsets, cfg.lr, cfg.eps)
            times.append(time.perf_counter() - t0)
            reps += 1
        sp = want["split"]
        ok = counts0 == [len(sp["co"]), len(sp["ex"]), len(sp["ex_next"])] and u[0] == len(lay0["unique"]) \
            and u[1] == len(want["layout_next"]["unique"])
        got_rows = table[torch.from_numpy(touched).to(dev)].float().cpu().numpy()
        ref_rows = t_ref if tab.dtype == "f32" else O.bf16_bits_to_f32(t_ref)
        ok = ok and np.allclose(got_rows, ref_rows, rtol=1e-5 if tab.dtype == "f32" else 8e-3, atol=1e-6)
        ok = ok and np.allclose(reduced[0][:u[0]].cpu().numpy(), want["reduced"], rtol=1e-5, atol=1e-6)
        if not ok:
            print("bench.py: GPU step does not match the oracle", file=sys.stderr)
            return 4
        cpu_s = statistics.median(times)
        cpu_baseline = {"value": u[0] / cpu_s, "unit": "rows/s", "cores": 1, "kind": "oracle",
                        "ms_per_step": cpu_s * 1e3,
                        "sample": f"the full step t=0 of this workload (N={n[0]}, U={u[0]}), median of {reps} runs of "
                                  "the single-threaded C oracle on a table holding only the touched rows",
                        "host_cpus": os.cpu_count()}

    # the ping-pong continues with t=1 -> 0, then t=0 -> 1, ...
    if args.mode == "graph":
        graphs = [fs.fs_graph_capture_pipelined(ctx, step_args[s], step_args[(s + 1) % period])
                  for s in range(period)]
    run(1, args.warmup)
    torch.cuda.synchronize()
    k0 = 1 + args.warmup
    if graphs is None:
        fs.fs_ctx_set_kernel_timing(ctx, args.steps, args.time_every)
    torch.cuda.synchronize()
    fs.fs_ctx_host_times(ctx, reset=True)
    # ten marks on the caller's stream inside the timed region (an event record each, no wait): the spread of
    # the step time over the run
    nblk = 10 if args.steps >= 100 else 1
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(nblk + 1)]
    bounds = [k0 + args.steps * b // nblk for b in range(nblk + 1)]
    t0 = time.perf_counter()
    for b in range(nblk):
        marks[b].record()
        run(bounds[b], bounds[b + 1] - bounds[b])
    marks[nblk].record()
    t_enq = time.perf_counter() - t0
    fs.fs_step_join(ctx)                      # the index half of the last step is part of the timed work
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    assert fs.fs_check_async(ctx) == fs.FS_OK, ctx.last_error()
    blk_us = sorted(marks[b].elapsed_time(marks[b + 1]) * 1e3 / (bounds[b + 1] - bounds[b]) for b in range(nblk))
    step_spread = {"blocks": nblk, "min_us": blk_us[0], "median_us": blk_us[len(blk_us) // 2], "max_us": blk_us[-1],
                   "note": "step time of each tenth of the timed region, from events on the caller's stream"}
    ht = fs.fs_ctx_host_times(ctx)
    host_phases = None
    if ht[6] > 0:
        names = ("wait_side_thread", "fork_and_post", "wait_side_stream", "priority_and_gather",
                 "index_thread_enqueue", "side_thread_enqueue")
        host_phases = {k: ht[i] / ht[6] for i, k in enumerate(names)}
    if graphs is not None:
        # Per-kernel durations cannot be bracketed inside a replayed graph: the same kernels are
        # timed with event pairs over as many eager pipelined steps right after the timed region.
        k1 = k0 + args.steps
        saved, graphs = graphs, None
        fs.fs_ctx_set_kernel_timing(ctx, args.steps)
        run(k1, args.steps)
        fs.fs_step_join(ctx)
        torch.cuda.synchronize()
        graphs = saved
        s_executed = k1 + args.steps - 1
    else:
        s_executed = k0 + args.steps - 1

    kinds = {"gather": fs.FS_TIME_GATHER, "priority_pass": fs.FS_TIME_UPDATE_CO, "deferred_pass": fs.FS_TIME_UPDATE_EX}
    kernel_ms = {}
    for name, kind in kinds.items():
        vals = fs.fs_ctx_get_kernel_timing(ctx, kind, args.steps)
        kernel_ms[name] = (sum(vals) / len(vals)) if vals else None
    fs.fs_ctx_set_kernel_timing(ctx, 0)
    if graphs is not None:
        for g in graphs:
            fs.fs_graph_destroy(ctx, g)

    # rows updated over the timed steps: step s updates U_{s%2}
    rows = sum(u[s % 2] for s in range(k0, k0 + args.steps))
    ms_per_step = elapsed / args.steps * 1e3
    by = [algorithmic_bytes(n[0], u[0], n[1], u[1], dim, w), algorithmic_bytes(n[1], u[1], n[0], u[0], dim, w)]
    step_bytes = sum(by[s % 2]["total"] for s in range(k0, k0 + args.steps)) / args.steps
    step_gbps = step_bytes / (ms_per_step * 1e-3) / 1e9

    # Occurrences and rows per class of the two alternating iterations: from the layout of each batch
    # and the split buffers of two consecutive iterations that are still in place (pipelined: the last
    # step and the iteration whose index half it ran; self-contained steps: the last two).
    s_last = s_executed
    cls_pos, cls_rows = {}, {}
    for s in ((s_last, s_last + 1) if pipelined else (s_last - 1, s_last)):
        lay, sp = layouts[s % L], splits[s % P]
        cn = sp["counts"].cpu().numpy().tolist()
        uu = int(lay["n_unique"].item())
        assert uu == u[s % 2] and cn[0] + cn[1] == uu, (s, uu, u, cn)
        seg = lay["seg_offsets"][:uu + 1].cpu().numpy().astype(np.int64)
        lens = seg[1:] - seg[:-1]
        co_pos = int(lens[sp["co_slot"][:cn[0]].cpu().numpy()].sum())
        cls_pos[s % 2] = (co_pos, n[s % 2] - co_pos)
        cls_rows[s % 2] = (cn[0], cn[1])

    def class_pass_bytes(b, c):
        # gradient rows + two index words per occurrence; row read+write, state read+write, row id per row
        return cls_pos[b][c] * (dim * 4 + 8) + cls_rows[b][c] * (2 * dim * w + 8 + 8)

    # Dominant kernel = the kernel that takes the most GPU time per step: class_pass_kernel, launched
    # twice per step (priority pass on the caller's stream, deferred pass on the side stream, usually
    # side by side), against the gather.  For class_pass_kernel the figures are per launch, averaged
    # over both launches; the two passes are also listed on their own.
    avg = lambda f: sum(f(s % 2) for s in range(k0, k0 + args.steps)) / args.steps
    per_kernel = {}
    if kernel_ms.get("gather"):
        per_kernel["gather_kernel"] = (kernel_ms["gather"], avg(lambda b: by[b]["gather"]), 1)
    if kernel_ms.get("priority_pass"):
        per_kernel["class_pass_kernel (priority pass)"] = (kernel_ms["priority_pass"],
                                                           avg(lambda b: class_pass_bytes(b, 0)), 1)
    if kernel_ms.get("deferred_pass"):
        per_kernel["class_pass_kernel (deferred pass)"] = (kernel_ms["deferred_pass"],
                                                           avg(lambda b: class_pass_bytes(b, 1)), 1)
    cand = dict(per_kernel)
    both = [v for k, v in per_kernel.items() if k.startswith("class_pass_kernel")]
    if len(both) == 2:
        cand = {k: v for k, v in per_kernel.items() if not k.startswith("class_pass_kernel")}
        cand["class_pass_kernel"] = ((both[0][0] + both[1][0]) / 2, (both[0][1] + both[1][1]) / 2, 2)
    roofline = None
    if cand:
        name = max(cand, key=lambda k: cand[k][0] * cand[k][2])
        ms, nbytes, launches = cand[name]
        achieved = nbytes / (ms * 1e-3) / 1e9
        traffic = None
        if pipelined and ahead:
            key = f"configs[{cfg.index}]"
            if name == "class_pass_kernel":
                t2 = [MEASURED_TRAFFIC_BYTES.get((key, name + sfx)) for sfx in (" (priority pass)", " (deferred pass)")]
                traffic = (t2[0] + t2[1]) / 2 if all(t2) else None
            else:
                traffic = MEASURED_TRAFFIC_BYTES.get((key, name))
        roofline = {"bound": "hbm", "kernel": name, "launches_per_step": launches, "achieved": achieved,
                    "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS, "traffic": traffic,
                    "avg_launch_us": ms * 1e3, "algorithmic_bytes_per_launch": nbytes,
                    "all_kernels": {nm: {"avg_launch_us": m * 1e3, "algorithmic_bytes": nb,
                                         "GBps": nb / (m * 1e-3) / 1e9} for nm, (m, nb, _) in per_kernel.items()}}

    # what the counters say the whole step moves (all kernels of one iteration), where they were read
    step_traffic = None
    if pipelined and ahead:
        parts = [MEASURED_TRAFFIC_BYTES.get((f"configs[{cfg.index}]", k)) for k in
                 ("class_pass_kernel (priority pass)", "class_pass_kernel (deferred pass)", "gather_kernel",
                  "index kernels")]
        step_traffic = sum(parts) if all(parts) else None

    # ---- beside the metric: the chip's own copy rate (the achievable ceiling) and the step with the caches
    # scrubbed between iterations (a 1 GiB -> 1 GiB copy, eight times the memory-side cache, before every step)
    copy_ceiling = None
    if not args.no_isolated and pipelined:
        fs.fs_step_join(ctx)
        torch.cuda.synchronize()
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)

        def timed_loop(f, reps):
            f(0)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for i in range(reps):
                f(i + 1)
            fs.fs_step_join(ctx)
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) / reps

        def scrub(i):
            fs.fs_stream_copy(ctx, src, dst)

        t_copy = timed_loop(scrub, 20)
        k1 = [k0 + args.steps]

        def step_and_scrub(i):
            fs.fs_stream_copy(ctx, src, dst)
            run(k1[0], 1)
            k1[0] += 1

        if graphs is None:
            t_both = timed_loop(step_and_scrub, 20)
            cold_us = (t_both - t_copy) * 1e6
        else:
            cold_us = None
        copy_gbps = 2 * src.numel() / t_copy / 1e9
        copy_ceiling = {"stream_copy_GBps": copy_gbps, "stream_copy_frac_of_hbm_peak": copy_gbps / HBM_PEAK_GBPS,
                        "bytes": 2 * src.numel(),
                        "step_algorithmic_frac_of_stream_copy": step_gbps / copy_gbps,
                        "cold_step_us": cold_us,
                        "cold_step_note": "20 steps, each behind a 1 GiB -> 1 GiB copy on the same stream, minus the "
                                          "time of the copies alone; the steady-state loop does not flush anything"}
        del src, dst

    # ---- the same kernels alone on the chip: each operation launched 20 times back to back on one
    # stream with nothing beside it (after the timed region; the table keeps being updated, which
    # does not change what the kernels move)
    isolated = None
    if not args.no_isolated:
        def alone(f, reps=20):
            for _ in range(3):
                f()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                f()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / reps * 1e3

        fs.fs_step_join(ctx)
        torch.cuda.synchronize()
        lay_a = fs.fs_unique_ids(ctx, d_vals[0], tab.num_rows)
        lay_b = fs.fs_unique_ids(ctx, d_vals[1], tab.num_rows)
        sp_a = fs.fs_collision_split_classes(ctx, lay_a, lay_b["unique"], lay_b["n_unique"], n[1])
        iso = {
            "class_pass_kernel (priority pass)": (alone(lambda: fs.fs_reduce_update_class(
                ctx, 0, table, state, cfg.lr, cfg.eps, d_grads[0], lay_a, sp_a)), class_pass_bytes(0, 0)),
            "class_pass_kernel (deferred pass)": (alone(lambda: fs.fs_reduce_update_class(
                ctx, 1, table, state, cfg.lr, cfg.eps, d_grads[0], lay_a, sp_a)), class_pass_bytes(0, 1)),
            "gather_kernel": (alone(lambda: fs.fs_gather_jagged(ctx, table, d_vals[1], d_offs[1], out=embs[1])),
                              by[0]["gather"]),
            "dedup (8 launches)": (alone(lambda: fs.fs_unique_ids(ctx, d_vals[1], tab.num_rows, out=lay_b)),
                                   by[0]["unique"]),
            "split + class order + records (3 launches)": (alone(lambda: fs.fs_collision_split_classes(
                ctx, lay_a, lay_b["unique"], lay_b["n_unique"], n[1], out=sp_a)), by[0]["split"]),
        }
        assert fs.fs_check_async(ctx) == fs.FS_OK, ctx.last_error()
        isolated = {k: {"us": t, "algorithmic_bytes": nb, "GBps": nb / (t * 1e-6) / 1e9,
                        "frac_of_hbm_peak": nb / (t * 1e-6) / 1e9 / HBM_PEAK_GBPS} for k, (t, nb) in iso.items()}

    # ---- beside the metric: the load balancer's data path (Sections 4.1 and 4.2 of the paper) on the batch a
    # job of 64 ranks with this configuration's local batch would balance; each operation alone on the chip
    balancer = None
    if not args.no_widening and tab.dtype == "f32" and cfg.batch * 64 <= nmax:
        from fs_workloads.generators import powerlaw_lengths
        fs.fs_step_join(ctx)
        torch.cuda.synchronize()
        ranks, keys = 64, 4
        Bg = cfg.batch * ranks
        rng = np.random.default_rng(20240)
        lens = powerlaw_lengths(rng, Bg, 1.5, cfg.length_lo, cfg.length_hi)
        offs = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
        ng = int(offs[-1])
        d_len, d_off = torch.from_numpy(lens).to(dev), torch.from_numpy(offs).to(dev)
        d_ids = torch.randint(0, tab.num_rows, (ng,), dtype=torch.int64, device=dev)

        def timed(f, reps=10):
            for _ in range(2):
                f()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                f()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / reps * 1e3

        sample_of, rank_off = fs.fs_partition_fbs(ctx, d_len, cfg.length_hi, ranks)
        Bk = Bg // keys                                   # the same segments read as keys x samples
        _, rank_off_k = fs.fs_partition_fbs(ctx, d_len[:Bk], cfg.length_hi, ranks)
        disp, disp_off, _ = fs.fs_jagged_ranged_dispatch(ctx, d_ids, d_off, keys, Bk, rank_off_k)
        emb_rows, emb_off = embs[1], d_offs[1]            # the gathered rows of one local batch, 512 bytes each
        local_of, _ = fs.fs_partition_fbs(ctx, (emb_off[1:] - emb_off[:-1]).contiguous(), cfg.length_hi, 8)
        seg_bytes = 3 * 8 * Bg
        ops = {
            f"fs_partition_fbs ({Bg} samples, {ranks} ranks)":
                (timed(lambda: fs.fs_partition_fbs(ctx, d_len, cfg.length_hi, ranks)), 8 * Bg + 4 * Bg),
            f"fs_jagged_indexed_permute ({ng} IDs of {Bg} samples, FBS order)":
                (timed(lambda: fs.fs_jagged_indexed_permute(ctx, d_ids, d_off, sample_of, ng)), 16 * ng + seg_bytes),
            f"fs_jagged_ranged_dispatch ({ng} IDs, {keys} keys x {Bk} samples, {ranks} ranks)":
                (timed(lambda: fs.fs_jagged_ranged_dispatch(ctx, d_ids, d_off, keys, Bk, rank_off_k)), 16 * ng + seg_bytes),
            f"fs_jagged_ranged_combine (the same, back)":
                (timed(lambda: fs.fs_jagged_ranged_combine(ctx, disp, disp_off, keys, Bk, rank_off_k)), 16 * ng + seg_bytes),
            f"fs_jagged_keyed_transpose ({ng} IDs, {keys} keys x {Bk} samples)":
                (timed(lambda: fs.fs_jagged_keyed_transpose(ctx, d_ids, d_off, keys, Bk)), 16 * ng + seg_bytes),
            f"fs_jagged_indexed_permute ({n[1]} embedding rows of {dim * 4} bytes, {cfg.batch} samples)":
                (timed(lambda: fs.fs_jagged_indexed_permute(ctx, emb_rows, emb_off, local_of, n[1])), 2 * n[1] * dim * 4),
        }
        assert fs.fs_check_async(ctx) == fs.FS_OK, ctx.last_error()
        balancer = {k: {"us": t, "algorithmic_bytes": nb, "GBps": nb / (t * 1e-6) / 1e9,
                        "frac_of_hbm_peak": nb / (t * 1e-6) / 1e9 / HBM_PEAK_GBPS} for k, (t, nb) in ops.items()}
        del d_ids, disp

    out = {
        "metric": "unique embedding rows updated/sec + achieved HBM GB/s (% of peak), 1 GPU",
        "value": rows / elapsed, "unit": "rows/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": tab.dtype, "data": "synthetic",
        "config": {"workload": f"configs[{cfg.index}] {cfg.name}: 1 table shard {tab.num_rows} rows x dim {dim} "
                               f"{tab.dtype} + fp32 row-wise Adagrad state, batch {cfg.batch}, "
                               f"{cfg.length_rule} UIH lengths [{cfg.length_lo},{cfg.length_hi}], Zipf({tab.zipf_alpha}) IDs, "
                               "2 consecutive iterations stepped back and forth",
                   "ids_per_iteration": n, "unique_rows": u, "collision_rows_first_step": counts0[0]},
        "schedule": args.mode + ((f"+index_half_ahead(batches of {K})" if index_ahead else "+dedup_ahead") if ahead else "") + ("+two_part_lookup" if args.two_part else ""), "reduced_gradients_in_memory": bool(args.keep_reduced),
        "class_occurrences": cls_pos, "class_rows": cls_rows, "host_enqueue_us_per_step": t_enq / args.steps * 1e6,
        "host_phase_us_per_step": host_phases,
        "step_time_spread": step_spread,
        "step_algorithmic_bytes": step_bytes, "step_algorithmic_GBps": step_gbps,
        "step_frac_of_hbm_peak": step_gbps / HBM_PEAK_GBPS,
        "step_measured_traffic_bytes": step_traffic,
        "step_measured_traffic_frac_of_hbm_peak": (step_traffic / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS
                                                   if step_traffic else None),
        "kernel_avg_us": {k: (v * 1e3 if v is not None else None) for k, v in kernel_ms.items()},
        "roofline": roofline,
        "achievable_ceiling": copy_ceiling,
        "isolated_kernels": isolated,
        "load_balancer_path": balancer,
        "cpu_baseline": cpu_baseline,
    }
    print(json.dumps(out))
    ctx.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
