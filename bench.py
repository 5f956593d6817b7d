#!/usr/bin/env python3
"""Throughput of the whole prioritized-update step on one MI355X, on every full-size workload.

A "step" is one pass of the full hot path over one batch of every table of the shard: dedup of the lookahead
IDs, collision split and class order, priority pass (gradient segment-reduce fused with row-wise Adagrad on the
collision rows), deferred pass (the same on the exclusive rows) on its own stream, and the jagged gather of the
lookahead batch.  One invocation times the workload configurations [1], [2], [3] and [4]; the headline (`value`,
`ms_per_step`, `config.workload`) is the largest single-GPU configuration, configs[2] (eight tables per shard,
2 GB per step); the others are in `per_config`.  Every configuration cycles through ALL its batches (two, or
the ten of the streaming configuration with its drifting hot set): step s works on batch s mod T with batch
(s + 1) mod T as lookahead, so every step consumes the layout and class order that earlier index work produced,
as in steady-state training.  The call sequence is paper_2604_24073_amd.schedule.StepLoop, the same object the
full-size parity tests drive.  Inputs are resident in HBM before the timed region.

Timing: after W warm-up steps, `blocks` (default 10) blocks of K steps are enqueued back to back with an event
mark between blocks on every stream that carries steps (no wait anywhere); the region is bracketed by a
synchronisation on both sides.  `ms_per_step` is the MEDIAN block / K; `ms_per_step_whole_region` is the wall
clock of all blocks / (blocks * K).

Prints ONE JSON line.  `python bench.py --summarize-counters DIR [DIR ...]` instead prints the per-kernel means
of rocprofv3 counter CSVs (the rows of profiles/hbm_traffic_per_launch.txt).
"""
from __future__ import annotations

import argparse
import csv
import glob
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E peak
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic_per_launch.txt")
METRIC = "unique embedding rows updated/sec + achieved HBM GB/s (% of peak), 1 GPU"


def algorithmic_bytes(n_t, u_t, n_t1, u_t1, dim, w):
    """Compulsory bytes of one step (each distinct row counted once per pass; the sort's
    internal passes and the reduced-gradient round trip are NOT counted)."""
    unique = 8 * n_t1 + 8 * u_t1 + 4 * n_t1
    split = 16 * (u_t + u_t1)
    gather = 8 * n_t1 + u_t1 * dim * w + n_t1 * dim * w
    reduce_update = n_t * dim * 4 + 4 * n_t + 2 * u_t * dim * w + 8 * u_t + 8 * u_t
    return {"unique": unique, "split": split, "gather": gather, "reduce_update": reduce_update,
            "total": unique + split + gather + reduce_update}


def device_info():
    """What the runtime says about the chip the figures were taken on (as found: nothing is set or locked)."""
    import torch
    p = torch.cuda.get_device_properties(0)
    info = {"name": p.name, "compute_units": p.multi_processor_count, "memory_GiB": p.total_memory / 2 ** 30,
            "hbm_peak_GBps_used": HBM_PEAK_GBPS}
    for field in ("gcnArchName", "clock_rate", "memory_clock_rate", "memory_bus_width", "L2_cache_size"):
        v = getattr(p, field, None)
        if v is not None:
            info[field] = v
    return info


def read_traffic(path=TRAFFIC_FILE):
    """profiles/hbm_traffic_per_launch.txt -> {(workload, kernel): HBM bytes per launch, launches per step}.
    Columns (blanks; '#' starts a comment): workload, kernel (no blanks; "/LPRnn" marks the launch of one row
    width), dispatches averaged over, launches per step, FETCH_SIZE KiB, WRITE_SIZE KiB, the two calibration
    factors.  Bytes = (FETCH * f_fetch + WRITE * f_write) * 1024 per launch."""
    out = {}
    if not os.path.exists(path):
        return out
    for line in open(path):
        line = line.split("#", 1)[0].strip()
        if not line:
            continue
        f = line.split()
        if len(f) < 8:
            continue
        out[(f[0], f[1])] = {"bytes": (float(f[4]) * float(f[6]) + float(f[5]) * float(f[7])) * 1024.0,
                             "launches_per_step": float(f[3])}
    return out


def summarize_counters(dirs) -> int:
    """Mean counter value per kernel over the dispatches of rocprofv3 --pmc runs (CSV output); for a
    --kernel-trace --stats run the per-kernel durations of its kernel_stats CSV."""
    import collections
    agg = collections.defaultdict(lambda: collections.defaultdict(list))
    for d in dirs:
        for path in glob.glob(os.path.join(d, "**", "*kernel_stats.csv"), recursive=True):
            print(f"# {path}: kernel, calls, avg us, min us, max us, % of kernel time")
            for r in csv.DictReader(open(path)):
                if not r["Name"].replace("void ", "").startswith("fs::"):
                    continue
                name = r["Name"].replace("void ", "").replace("fs::", "").split("(")[0].strip().replace(" ", "")
                print(f"{name:60s} {int(r['Calls']):6d} {float(r['AverageNs']) / 1e3:8.1f} {float(r['MinNs']) / 1e3:8.1f} "
                      f"{float(r['MaxNs']) / 1e3:8.1f} {float(r['Percentage']):6.1f}")
        for path in glob.glob(os.path.join(d, "**", "*counter_collection.csv"), recursive=True):
            for r in csv.DictReader(open(path)):
                name = r["Kernel_Name"].replace("void ", "").replace("fs::", "").split("(")[0].strip()
                if not r["Kernel_Name"].replace("void ", "").startswith("fs::"):
                    continue
                agg[name][r["Counter_Name"]].append(float(r["Counter_Value"]))
    for name in sorted(agg):
        cols = "  ".join(f"{c}={sum(v) / len(v):.1f}" for c, v in sorted(agg[name].items()))
        n = len(next(iter(agg[name].values())))
        print(f"{name.replace(' ', ''):70s} dispatches={n}  {cols}")
    return 0


def class_stats(vals):
    """Per batch of one table: distinct rows, and (occurrences, rows) of collision and exclusive rows against the
    next batch of the cycle.  Plain torch on the device: a statistic for the byte counts, not part of the path."""
    import torch
    T = len(vals)
    uniq = [torch.unique(v, return_counts=True) for v in vals]
    out = []
    for b in range(T):
        u, c = uniq[b]
        is_co = torch.isin(u, uniq[(b + 1) % T][0])
        co_pos, co_rows = int(c[is_co].sum().item()), int(is_co.sum().item())
        out.append({"u": int(u.numel()), "pos": (co_pos, int(c.sum().item()) - co_pos),
                    "rows": (co_rows, int(u.numel()) - co_rows)})
    return out


def bench_config(args, ci, extras):
    import numpy as np
    import torch
    import paper_2604_24073_amd as fs
    from paper_2604_24073_amd.schedule import StepLoop, TableBuffers
    from fs_workloads import CONFIGS, make_iterations, hash_init_rows, compact_rows
    from fs_workloads.checks import assert_close_f32, assert_rows_close

    dev = torch.device("cuda:0")
    cfg = CONFIGS[ci]
    T = cfg.iterations
    its_all = make_iterations(cfg)
    bufs = []
    for ti, tab in enumerate(cfg.tables):
        tdtype = torch.float32 if tab.dtype == "f32" else torch.bfloat16
        table = torch.empty((tab.num_rows, tab.dim), dtype=tdtype, device=dev)
        state = torch.zeros(tab.num_rows, dtype=torch.float32, device=dev)
        its = [x[ti] for x in its_all]
        bufs.append(TableBuffers(table, state, [torch.from_numpy(it.values).to(dev) for it in its],
                                 [torch.from_numpy(it.offsets).to(dev) for it in its],
                                 [torch.from_numpy(it.grads).to(dev) for it in its], cfg.lr, cfg.eps))
    multi = len(bufs) > 1
    loop = StepLoop(bufs, groups=args.table_groups if multi else 1,
                    iters_per_chain=None if multi else args.ahead_batch, keep_reduced=args.keep_reduced,
                    two_part=args.two_part, emb_rotation=3 if args.two_part else None, lookahead=args.lookahead,
                    row_ordered_lookup=args.lookup_order == "row")
    ctx = loop.ctxs[0]
    for b in bufs:
        fs.fs_init_table_hash(ctx, b.table)
    stats = [class_stats(b.values) for b in bufs]
    torch.cuda.synchronize()

    if args.calibration_copy > 0:
        src = torch.empty(args.calibration_copy << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        fs.fs_stream_copy(ctx, src, dst)
        torch.cuda.synchronize()
        del src, dst

    # ---- step 0 from the fresh tables, checked against the oracle on the touched rows with the parity tests' bars;
    # the oracle's step is what cpu_baseline times
    loop.run(0, 1)
    loop.join(check=True)
    cpu_baseline = None
    if not args.no_cpu_baseline:
        import oracle as O
        cpu_s, reps_all = 0.0, []
        budget = args.cpu_seconds / len(bufs)
        for ti, (tab, b) in enumerate(zip(cfg.tables, bufs)):
            its = [x[ti] for x in its_all]
            touched, (v0c, v1c) = compact_rows([its[0].values, its[1].values])
            w0 = np.concatenate([hash_init_rows(touched[i:i + 65536], tab.dim, tab.dtype)
                                 for i in range(0, len(touched), 65536)])
            if tab.dtype == "bf16":
                w0 = (w0.view(np.uint32) >> np.uint32(16)).astype(np.uint16)
            lay0 = O.unique_ids(v0c, len(touched))           # produced by the previous step: not timed
            reps, times, want = 0, [], None
            t_budget = time.perf_counter()
            while reps < 2 or (time.perf_counter() - t_budget < budget and reps < 100):
                t_ref, s_ref = w0.copy(), np.zeros(len(touched), np.float32)
                t0 = time.perf_counter()
                want = O.step(t_ref, s_ref, lay0, its[0].grads, v1c, its[1].offsets, cfg.lr, cfg.eps)
                times.append(time.perf_counter() - t0)
                reps += 1
            idx = torch.from_numpy(touched).to(dev)
            got_rows = b.table[idx]
            got_rows = (got_rows.cpu().numpy() if tab.dtype == "f32"
                        else got_rows.view(torch.int16).cpu().numpy().view(np.uint16))
            got_emb = b.emb_of_step(0)[:b.n[1 % b.T]]
            got_emb = (got_emb.cpu().numpy() if tab.dtype == "f32"
                       else got_emb.view(torch.int16).cpu().numpy().view(np.uint16))
            try:
                assert stats[ti][0]["u"] == len(lay0["unique"]), "number of distinct rows"
                assert stats[ti][0]["rows"][0] == len(want["split"]["co"]), "number of collision rows"
                assert_rows_close(got_rows, t_ref, "rows after step 0")
                assert_close_f32(b.state[idx].cpu().numpy(), s_ref, "Adagrad state after step 0")
                assert_rows_close(got_emb, want["emb_next"], "batch gathered by step 0")
            except AssertionError as e:
                print(f"bench.py: configs[{ci}] table {ti}: GPU step does not match the oracle: {e}", file=sys.stderr)
                return None
            cpu_s += statistics.median(times)
            reps_all.append(reps)
        rows0 = sum(s[0]["u"] for s in stats)
        cpu_baseline = {"value": rows0 / cpu_s, "unit": "rows/s", "cores": 1, "kind": "oracle",
                        "ms_per_step": cpu_s * 1e3,
                        "sample": f"the full step 0 of this workload ({len(bufs)} table(s), {rows0} distinct rows), per "
                                  f"table the median of {min(reps_all)}-{max(reps_all)} runs of the single-threaded C "
                                  f"oracle on a table holding only the touched rows (about {args.cpu_seconds:.0f} s of "
                                  "CPU work in all)",
                        "host_cpus": os.cpu_count()}

    # ---- warm-up, then `blocks` blocks of K steps with marks between them and no wait anywhere
    K, nblk = args.steps, args.blocks
    loop.run(1, args.warmup)
    loop.join()
    torch.cuda.synchronize()
    k0 = 1 + args.warmup
    fs.fs_ctx_set_kernel_timing(ctx, max(1, K * nblk // args.time_every + 2), args.time_every)
    for c in loop.ctxs:
        fs.fs_ctx_host_times(c, reset=True)
    marks = [[torch.cuda.Event(enable_timing=True) for _ in range(nblk + 1)] for _ in loop.streams]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for blk in range(nblk):
        for m, st in zip(marks, loop.streams):
            m[blk].record(st)
        loop.run(k0 + blk * K, K)
    for m, st in zip(marks, loop.streams):
        m[nblk].record(st)
    t_enq = time.perf_counter() - t0
    loop.join()                               # the index halves issued by the last steps are part of the timed work
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    loop.join(check=True)
    total_steps = K * nblk
    blk_us = sorted(max(m[blk].elapsed_time(m[blk + 1]) for m in marks) * 1e3 / K for blk in range(nblk))
    med_us = blk_us[len(blk_us) // 2] if nblk % 2 else 0.5 * (blk_us[nblk // 2 - 1] + blk_us[nblk // 2])
    ms_per_step = med_us * 1e-3

    names = ("wait_side_thread", "fork_and_post", "wait_side_stream", "priority_and_gather", "index_thread_enqueue",
             "side_thread_enqueue")
    host_phases = []
    for c in loop.ctxs:
        ht = fs.fs_ctx_host_times(c)
        host_phases.append({k: ht[i] / ht[6] for i, k in enumerate(names)} if ht[6] > 0 else None)
    kinds = {"gather": fs.FS_TIME_GATHER, "priority_pass": fs.FS_TIME_UPDATE_CO, "deferred_pass": fs.FS_TIME_UPDATE_EX}
    kernel_ms = {}
    for name, kind in kinds.items():
        vals = fs.fs_ctx_get_kernel_timing(ctx, kind, total_steps)
        kernel_ms[name] = (sum(vals) / len(vals)) if vals else None
    fs.fs_ctx_set_kernel_timing(ctx, 0)

    # ---- rows and bytes per step, averaged over the cycle of batches
    rows_per_step = sum(sum(s[b]["u"] for b in range(T)) / T for s in stats)
    step_bytes = 0.0
    parts = {"unique": 0.0, "split": 0.0, "gather": 0.0, "reduce_update": 0.0}
    for b_, s in zip(bufs, stats):
        for b in range(T):
            nb = (b + 1) % T
            by = algorithmic_bytes(b_.n[b], s[b]["u"], b_.n[nb], s[nb]["u"], b_.dim, b_.w)
            step_bytes += by["total"] / T
            for k in parts:
                parts[k] += by[k] / T
    step_gbps = step_bytes / (ms_per_step * 1e-3) / 1e9

    def class_pass_bytes(tables, c):
        # gradient rows + two index words per occurrence; row read+write, state read+write, row id per row
        return sum(sum(s[b]["pos"][c] * (t.dim * 4 + 8) + s[b]["rows"][c] * (2 * t.dim * t.w + 16) for b in range(T)) / T
                   for t, s in tables)

    # ---- roofline of the dominant kernel: the event pairs of the first group's context bracket what one call
    # enqueues of one kind (the class pass of one class, or the gathers) for ALL tables of that group - one launch
    # per row width - on the stream it is launched on, inside the timed steps
    grp0 = [(t, stats[bufs.index(t)]) for t in loop.groups[0]]
    widths = len({t.dim * t.w for t, _ in grp0})
    per_kernel = {}
    if kernel_ms.get("gather"):
        gb = sum(sum(algorithmic_bytes(t.n[b], s[b]["u"], t.n[(b + 1) % T], s[(b + 1) % T]["u"], t.dim, t.w)["gather"]
                     for b in range(T)) / T for t, s in grp0)
        per_kernel["gather_rows_kernel"] = (kernel_ms["gather"], gb, 1)
    if kernel_ms.get("priority_pass"):
        per_kernel["class_pass_kernel(priority_pass)"] = (kernel_ms["priority_pass"], class_pass_bytes(grp0, 0), 1)
    if kernel_ms.get("deferred_pass"):
        per_kernel["class_pass_kernel(deferred_pass)"] = (kernel_ms["deferred_pass"], class_pass_bytes(grp0, 1), 1)
    cand = dict(per_kernel)
    both = [v for k, v in per_kernel.items() if k.startswith("class_pass_kernel")]
    if len(both) == 2:
        cand = {k: v for k, v in per_kernel.items() if not k.startswith("class_pass_kernel")}
        cand["class_pass_kernel"] = ((both[0][0] + both[1][0]) / 2, (both[0][1] + both[1][1]) / 2, 2)
    traffic_tab = read_traffic()
    wl = f"configs[{ci}]"

    def traffic_of(name):
        # measured bytes of what one event pair brackets: the launches of every row width of that kind
        if name == "class_pass_kernel":
            t2 = [traffic_of(name + sfx) for sfx in ("(priority_pass)", "(deferred_pass)")]
            return (t2[0] + t2[1]) / 2 if all(t2) else None
        t = [v["bytes"] for (w_, k_), v in traffic_tab.items() if w_ == wl and k_.split("/")[0] == name]
        return sum(t) if t else None

    roofline = None
    if cand:
        name = max(cand, key=lambda k: cand[k][0] * cand[k][2])
        ms, nbytes, launches = cand[name]
        achieved = nbytes / (ms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "kernel": name, "launches_per_step": launches * widths, "achieved": achieved,
                    "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS,
                    "traffic": traffic_of(name), "avg_launch_us": ms * 1e3, "algorithmic_bytes_per_launch": nbytes,
                    "note": ("per launch; " if widths == 1 and not multi else
                             f"the {len(grp0)} tables of group 0 ({widths} launch(es) bracketed together); ") +
                            "duration from HIP event pairs on the kernel's own stream inside the timed steps, one "
                            f"step in {args.time_every}; in the pipelined step the kernel shares the chip with the other "
                            "passes",
                    "all_kernels": {nm: {"avg_launch_us": m * 1e3, "algorithmic_bytes": nb, "GBps": nb / (m * 1e-3) / 1e9,
                                         "traffic": traffic_of(nm)} for nm, (m, nb, _) in per_kernel.items()}}
    # what the counters say the whole step moves (all kernels of one iteration of every table)
    step_traffic = None
    if traffic_tab:
        rows_t = [v for (w_, _k), v in traffic_tab.items() if w_ == wl]
        if rows_t:
            step_traffic = sum(v["bytes"] * v["launches_per_step"] for v in rows_t)

    res = {
        "workload": (f"configs[{ci}] {cfg.name}: " +
                     (f"{len(bufs)} tables per shard, rows {[t.num_rows for t in cfg.tables]}, dims "
                      f"{[t.dim for t in cfg.tables]}" if multi else
                      f"1 table shard {cfg.tables[0].num_rows} rows x dim {cfg.tables[0].dim} {cfg.tables[0].dtype}") +
                     f" + fp32 row-wise Adagrad state, batch {cfg.batch}, {cfg.length_rule} UIH lengths "
                     f"[{cfg.length_lo},{cfg.length_hi}], Zipf({[t.zipf_alpha for t in cfg.tables]}) IDs"
                     f"{' with drifting hot set' if cfg.drift else ''}, {T} consecutive batches cycled"),
        "dtype": cfg.tables[0].dtype,
        "value": rows_per_step / (ms_per_step * 1e-3), "unit": "rows/s",
        "ms_per_step": ms_per_step, "us_per_step": med_us,
        "ms_per_step_whole_region": elapsed / total_steps * 1e3,
        "step_time_blocks_us": {"blocks": nblk, "steps_per_block": K, "min": blk_us[0], "median": med_us, "max": blk_us[-1]},
        "rows_per_step": rows_per_step,
        "ids_per_batch": [t.n for t in bufs], "unique_rows_per_batch": [[s[b]["u"] for b in range(T)] for s in stats],
        "collision_rows_per_batch": [[s[b]["rows"][0] for b in range(T)] for s in stats],
        "schedule": (f"{len(loop.groups)} group(s) of tables, each with a context and a stream; per step and group one "
                     f"multi-table pipelined call; index halves of {loop.K} iteration(s) of every table of a group per "
                     f"chain of launches, issued {loop.D} iterations ahead" + ("; two-part lookup" if args.two_part else "")),
        "table_groups": [[bufs.index(t) for t in g] for g in loop.groups],
        "host_enqueue_us_per_step": t_enq / total_steps * 1e6,
        "host_phase_us_per_step_and_group": host_phases,
        "step_algorithmic_bytes": step_bytes, "step_algorithmic_bytes_by_part": parts,
        "step_algorithmic_GBps": step_gbps, "step_frac_of_hbm_peak": step_gbps / HBM_PEAK_GBPS,
        "step_measured_traffic_bytes": step_traffic,
        "step_measured_traffic_frac_of_hbm_peak": (step_traffic / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS
                                                   if step_traffic else None),
        "kernel_avg_us": {k: (v * 1e3 if v is not None else None) for k, v in kernel_ms.items()},
        "roofline": roofline,
        "cpu_baseline": cpu_baseline,
    }
    if not args.no_extras:
        res["row_access_ceiling"] = measure_row_ceiling(loop, bufs, step_gbps)
        res["step_without_index_chains"] = measure_without_index(loop, k0 + total_steps, step_bytes, ms_per_step)
    if extras and not multi:
        res.update(measure_extras(args, cfg, loop, bufs[0], stats[0], k0 + total_steps, step_gbps))
    loop.close()
    del loop, bufs
    torch.cuda.empty_cache()
    return res


def measure_row_ceiling(loop, bufs, step_gbps):
    """The step's access pattern with nothing else in the way, on this workload's own tables: the distinct rows that
    the batches of a table touch, in a shuffled order, read whole by fs_stream_row_read and thrown away (one launch per
    table, no row twice, so no launch finds a row in a cache).  What the step could reach if every one
    of its bytes moved at this rate is `step_algorithmic_frac_of_ceiling`."""
    import torch
    import paper_2604_24073_amd as fs
    ctx, stream = loop.ctxs[0], loop.streams[0]
    dev = bufs[0].table.device
    sink = torch.zeros(1024, dtype=torch.int32, device=dev)
    jobs = []
    for t in bufs:
        u = torch.unique(torch.cat([t.values[b][:t.n[b]] for b in range(t.T)]))
        jobs.append((t.table, u[torch.randperm(u.numel(), device=dev)].contiguous()))
    by_batch = [sum(idx.numel() * tb.shape[1] * tb.element_size() for tb, idx in jobs)]
    reps = 10
    # a sweep of less than 1 GiB could find its rows in the 256 MB memory-side cache: such a sweep runs behind a
    # 1 GiB copy on the same stream; only the sweep itself is between the two events
    scrub = by_batch[0] < (1 << 30)
    if scrub:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
    loop.join()
    torch.cuda.synchronize()
    pairs = []
    for rep in range(reps + 1):
        if scrub:
            fs.fs_stream_copy(ctx, src, dst, stream=stream)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for tb, idx in jobs:
            fs.fs_stream_row_read(ctx, tb, idx, sink, stream=stream)
        e1.record(stream)
        if rep > 0:
            pairs.append((e0, e1))
    torch.cuda.synchronize()
    dt = sorted(a_.elapsed_time(b_) for a_, b_ in pairs)[len(pairs) // 2] * 1e-3
    if scrub:
        del src, dst
    gbps = by_batch[0] / dt / 1e9
    return {"random_row_read_GBps": gbps, "frac_of_hbm_peak": gbps / HBM_PEAK_GBPS, "launches": len(jobs),
            "bytes_per_sweep": by_batch[0], "step_algorithmic_frac_of_ceiling": step_gbps / gbps,
            "note": "the distinct rows touched by the batches of each table of this workload, shuffled, read whole and thrown away "
                    "(fs_stream_row_read), launches back to back on the step's stream" +
                    "; median of ten sweeps, each between two events" + ("; a 1 GiB copy before every sweep" if scrub else "")}


def measure_without_index(loop, s_next, step_bytes, ms_per_step):
    """What the index chains cost the step: the class passes and lookups of the two newest iterations replayed in
    turn with NO index work beside them (their layouts, splits and class orders are still in the rotating buffers, so
    every launch does the work it did in the timed region; the tables go on being updated).  Not a step of the
    method - the index half is part of the step - but it separates the row work from the index work."""
    import torch
    import paper_2604_24073_amd as fs
    P = loop.n_records
    window = [(s_next - 2) % P, (s_next - 1) % P]
    reps = 200

    def replay(n):
        for i in range(n):
            for c, st, rec in zip(loop.ctxs, loop.streams, loop.step_records):
                fs.fs_prioritized_step_pipelined_multi(c, rec[window[i % 2]], None, stream=st)

    loop.join()
    replay(4)
    loop.join()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    replay(reps)
    loop.join()
    torch.cuda.synchronize()
    us = (time.perf_counter() - t0) / reps * 1e6
    # once more with the kernels of one call in eight between event pairs (not the timed run: the records cost)
    ctx = loop.ctxs[0]
    fs.fs_ctx_set_kernel_timing(ctx, reps // 8 + 2, 8)
    replay(reps)
    loop.join()
    kinds = {"gather": fs.FS_TIME_GATHER, "priority_pass": fs.FS_TIME_UPDATE_CO, "deferred_pass": fs.FS_TIME_UPDATE_EX}
    kernel_us = {}
    for name, kind in kinds.items():
        vals = fs.fs_ctx_get_kernel_timing(ctx, kind, reps)
        kernel_us[name] = (sum(vals) / len(vals) * 1e3) if vals else None
    fs.fs_ctx_set_kernel_timing(ctx, 0)
    loop.join(check=True)
    return {"us_per_step": us, "kernel_avg_us": kernel_us, "frac_of_hbm_peak_on_the_step's_algorithmic_bytes": step_bytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBPS,
            "index_chains_cost_us_per_step": ms_per_step * 1e3 - us,
            "note": "priority pass, deferred pass and lookup of the two newest iterations replayed in turn, no index "
                    "launches beside them; 200 calls"}


def measure_extras(args, cfg, loop, t, stats, s_next, step_gbps):
    """Beside the metric, for one single-table workload: the chip's own copy rate and the step with the caches
    scrubbed between iterations; every kernel alone on the chip; the load balancer's data path."""
    import numpy as np
    import torch
    import paper_2604_24073_amd as fs
    dev = t.table.device
    ctx, stream = loop.ctxs[0], loop.streams[0]
    tab = cfg.tables[0]
    dim, w = t.dim, t.w
    out = {}

    src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)

    def timed_loop(f, reps):
        f(0)
        loop.join()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(reps):
            f(i + 1)
        loop.join()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / reps

    t_copy = timed_loop(lambda i: fs.fs_stream_copy(ctx, src, dst, stream=stream), 20)
    k1 = [s_next]

    def step_and_scrub(i):
        fs.fs_stream_copy(ctx, src, dst, stream=stream)
        loop.run(k1[0], 1)
        k1[0] += 1

    t_both = timed_loop(step_and_scrub, 20)
    # the step's access pattern with nothing else in the way: the gradient rows of one batch read in a random order
    # (what the class passes do with them), cold (behind the same 1 GiB copy) and back to back
    order = torch.randperm(t.n[0], device=dev)
    sink = torch.zeros(1024, dtype=torch.int32, device=dev)

    def read_and_scrub(i):
        fs.fs_stream_copy(ctx, src, dst, stream=stream)
        fs.fs_stream_row_read(ctx, t.grads[0], order, sink, stream=stream)

    t_rows_cold = timed_loop(read_and_scrub, 20) - t_copy
    t_rows_warm = timed_loop(lambda i: fs.fs_stream_row_read(ctx, t.grads[0], order, sink, stream=stream), 20)
    row_bytes_read = t.n[0] * t.grads[0].shape[1] * 4
    copy_gbps = 2 * src.numel() / t_copy / 1e9
    out["achievable_ceiling"] = {
        "stream_copy_GBps": copy_gbps, "stream_copy_frac_of_hbm_peak": copy_gbps / HBM_PEAK_GBPS,
        "bytes": 2 * src.numel(), "step_algorithmic_frac_of_stream_copy": step_gbps / copy_gbps,
        "cold_step_us": (t_both - t_copy) * 1e6,
        "cold_step_note": "20 steps, each behind a 1 GiB -> 1 GiB copy on the same stream, minus the time of the copies "
                          "alone; the steady-state loop does not flush anything",
        "random_row_read_GBps_cold": row_bytes_read / t_rows_cold / 1e9,
        "random_row_read_GBps_back_to_back": row_bytes_read / t_rows_warm / 1e9,
        "random_row_read_note": f"{t.n[0]} rows of {t.grads[0].shape[1] * 4} bytes (the gradient rows of one batch) read in "
                                "a random order by one launch of fs_stream_row_read and thrown away; cold = behind the "
                                "1 GiB copy, its time subtracted",
        "step_algorithmic_frac_of_random_row_read": step_gbps / (row_bytes_read / t_rows_cold / 1e9)}
    del src, dst

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

    loop.join()
    torch.cuda.synchronize()
    n = t.n
    by = algorithmic_bytes(n[0], stats[0]["u"], n[1], stats[1]["u"], dim, w)
    cpb = lambda c: stats[0]["pos"][c] * (dim * 4 + 8) + stats[0]["rows"][c] * (2 * dim * w + 16)
    lay_a = fs.fs_unique_ids(ctx, t.values[0], tab.num_rows)
    lay_b = fs.fs_unique_ids(ctx, t.values[1], tab.num_rows)
    sp_a = fs.fs_collision_split_classes(ctx, lay_a, lay_b["unique"], lay_b["n_unique"], n[1])
    emb = t.emb_of_step(0)
    iso = {
        "class_pass_kernel(priority_pass)": (alone(lambda: fs.fs_reduce_update_class(
            ctx, 0, t.table, t.state, cfg.lr, cfg.eps, t.grads[0], lay_a, sp_a)), cpb(0)),
        "class_pass_kernel(deferred_pass)": (alone(lambda: fs.fs_reduce_update_class(
            ctx, 1, t.table, t.state, cfg.lr, cfg.eps, t.grads[0], lay_a, sp_a)), cpb(1)),
        "gather_rows_kernel": (alone(lambda: fs.fs_gather_jagged(ctx, t.table, t.values[1], t.offsets[1], out=emb)), by["gather"]),
        "dedup (8 launches)": (alone(lambda: fs.fs_unique_ids(ctx, t.values[1], tab.num_rows, out=lay_b)), by["unique"]),
        "split + class order + records (3 launches)": (alone(lambda: fs.fs_collision_split_classes(
            ctx, lay_a, lay_b["unique"], lay_b["n_unique"], n[1], out=sp_a)), by["split"]),
    }
    if fs.fs_check_async(ctx) != fs.FS_OK:
        raise RuntimeError(ctx.last_error())
    out["isolated_kernels"] = {k: {"us": us, "algorithmic_bytes": nb, "GBps": nb / (us * 1e-6) / 1e9,
                                   "frac_of_hbm_peak": nb / (us * 1e-6) / 1e9 / HBM_PEAK_GBPS} for k, (us, nb) in iso.items()}

    # the load balancer's data path (Sections 4.1 and 4.2 of the paper) on the batch a job of 64 ranks with this
    # configuration's local batch would balance; each operation alone on the chip, outputs allocated beforehand
    nmax = max(n)
    if not args.no_widening and tab.dtype == "f32" and cfg.batch * 64 <= nmax:
        from fs_workloads.generators import powerlaw_lengths
        ranks, keys = 64, 4
        Bg = cfg.batch * ranks
        rng = np.random.default_rng(20240)
        lens = powerlaw_lengths(rng, Bg, 1.5, cfg.length_lo, cfg.length_hi)
        offs = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
        ng = int(offs[-1])
        d_len, d_off = torch.from_numpy(lens).to(dev), torch.from_numpy(offs).to(dev)
        d_ids = torch.randint(0, tab.num_rows, (ng,), dtype=torch.int64, device=dev)
        sample_of, rank_off = fs.fs_partition_fbs(ctx, d_len, cfg.length_hi, ranks)
        Bk = Bg // keys                                   # the same segments read as keys x samples
        _, rank_off_k = fs.fs_partition_fbs(ctx, d_len[:Bk], cfg.length_hi, ranks)
        disp = fs.fs_jagged_ranged_dispatch(ctx, d_ids, d_off, keys, Bk, rank_off_k)
        emb_rows, emb_off = t.embs[1][:n[1]], t.offsets[1]      # gathered rows of one local batch, 512 bytes each
        local_of, _ = fs.fs_partition_fbs(ctx, (emb_off[1:] - emb_off[:-1]).contiguous(), cfg.length_hi, 8)
        o_fbs = (torch.empty_like(sample_of), torch.empty_like(rank_off))
        o_ids = (torch.empty_like(d_ids), torch.empty_like(d_off))
        o_disp = (torch.empty_like(d_ids), torch.empty_like(d_off), torch.empty(ranks, dtype=torch.int64, device=dev))
        o_emb = (torch.empty_like(emb_rows), torch.empty_like(emb_off))
        seg_bytes = 3 * 8 * Bg
        ops = {
            f"fs_partition_fbs ({Bg} samples, {ranks} ranks)":
                (alone(lambda: fs.fs_partition_fbs(ctx, d_len, cfg.length_hi, ranks, out=o_fbs), 10), 8 * Bg + 4 * Bg),
            f"fs_jagged_indexed_permute ({ng} IDs of {Bg} samples, FBS order)":
                (alone(lambda: fs.fs_jagged_indexed_permute(ctx, d_ids, d_off, sample_of, ng, out=o_ids), 10), 16 * ng + seg_bytes),
            f"fs_jagged_ranged_dispatch ({ng} IDs, {keys} keys x {Bk} samples, {ranks} ranks)":
                (alone(lambda: fs.fs_jagged_ranged_dispatch(ctx, d_ids, d_off, keys, Bk, rank_off_k, out=o_disp), 10),
                 16 * ng + seg_bytes),
            "fs_jagged_ranged_combine (the same, back)":
                (alone(lambda: fs.fs_jagged_ranged_combine(ctx, disp[0], disp[1], keys, Bk, rank_off_k, out=o_ids), 10),
                 16 * ng + seg_bytes),
            f"fs_jagged_keyed_transpose ({ng} IDs, {keys} keys x {Bk} samples)":
                (alone(lambda: fs.fs_jagged_keyed_transpose(ctx, d_ids, d_off, keys, Bk, out=o_ids), 10), 16 * ng + seg_bytes),
            f"fs_jagged_indexed_permute ({n[1]} embedding rows of {dim * w} bytes, {cfg.batch} samples)":
                (alone(lambda: fs.fs_jagged_indexed_permute(ctx, emb_rows, emb_off, local_of, n[1], out=o_emb), 10),
                 2 * n[1] * dim * w),
        }
        if fs.fs_check_async(ctx) != fs.FS_OK:
            raise RuntimeError(ctx.last_error())
        out["load_balancer_path"] = {k: {"us": us, "algorithmic_bytes": nb, "GBps": nb / (us * 1e-6) / 1e9,
                                         "frac_of_hbm_peak": nb / (us * 1e-6) / 1e9 / HBM_PEAK_GBPS}
                                     for k, (us, nb) in ops.items()}
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50, help="steps per timed block")
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--blocks", type=int, default=10, help="timed blocks of --steps steps (the median block is reported)")
    ap.add_argument("--config", type=int, action="append", default=None,
                    help="workload configuration to time (repeatable); default: 2 (headline), 1, 3 and 4")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=5.0,
                    help="CPU time the oracle's step is repeated for, per configuration")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip what is measured beside the metric on configs[1]: every kernel alone on the chip, the copy "
                         "ceiling and the cold step, the load balancer's data path")
    ap.add_argument("--no-widening", action="store_true", help="of the extras, skip the load balancer's data path")
    ap.add_argument("--time-every", type=int, default=16,
                    help="bracket the kernels of one timed step in this many with HIP event pairs")
    ap.add_argument("--calibration-copy", type=int, default=0, metavar="MiB",
                    help="also launch one plain copy of this many MiB before the steps of every configuration: the "
                         "known-size dispatch that hardware byte counters are scaled by in a counter run")
    ap.add_argument("--ahead-batch", type=int, default=2, metavar="K",
                    help="single-table workloads: index halves of K consecutive iterations share their launches")
    ap.add_argument("--lookahead", type=int, default=None, metavar="D",
                    help="iterations between issuing a chain of index launches and stepping its first iteration "
                         "(default: K + 1, the least)")
    ap.add_argument("--table-groups", type=int, default=1, metavar="G",
                    help="workloads with several tables per shard: the tables are stepped in G groups, each with its "
                         "own context and stream")
    ap.add_argument("--lookup-order", choices=["row", "batch"], default="row",
                    help="the step's lookup walks the lookahead batch in row order (reads a row once for all its "
                         "occurrences) or in batch order (writes the output front to back)")
    ap.add_argument("--two-part", action="store_true",
                    help="the lookup in the two parts of Algorithm 2 (fs_prioritized_step_two_part_multi)")
    ap.add_argument("--keep-reduced", action="store_true",
                    help="also write the summed gradients to memory in the timed steps")
    ap.add_argument("--summarize-counters", nargs="+", metavar="DIR",
                    help="print per-kernel means of the rocprofv3 --pmc CSVs under these folders and exit")
    args = ap.parse_args()
    if args.summarize_counters:
        return summarize_counters(args.summarize_counters)
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (one embedding-table shard, no collectives); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        return 2
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    torch.cuda.set_device(0)
    args.blocks = max(1, args.blocks)
    configs = args.config if args.config else [2, 1, 3, 4]
    results = {}
    for ci in configs:
        t0 = time.perf_counter()
        r = bench_config(args, ci, extras=(not args.no_extras) and ci == 1)
        if r is None:
            return 4
        r["bench_seconds"] = time.perf_counter() - t0
        results[ci] = r
        print(f"bench.py: configs[{ci}] {r['us_per_step']:.1f} us/step, {r['step_frac_of_hbm_peak']:.3f} of HBM peak "
              f"({r['bench_seconds']:.0f} s)", file=sys.stderr, flush=True)
    head = results[configs[0]]
    out = {
        "metric": METRIC, "value": head["value"], "unit": "rows/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": head["dtype"], "data": "synthetic",
        "config": {"workload": head["workload"], "timed_blocks": args.blocks, "steps_per_block": args.steps,
                   "also_timed": [results[c]["workload"].split(":")[0] for c in configs[1:]]},
        "step_frac_of_hbm_peak": head["step_frac_of_hbm_peak"],
        "roofline": head["roofline"], "cpu_baseline": head["cpu_baseline"],
        "per_config": {f"configs[{c}]": results[c] for c in configs},
        "device": device_info(),
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
