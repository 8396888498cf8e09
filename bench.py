#!/usr/bin/env python3
"""Benchmark of the whole hot path (fikit_profile + fikit_gapfill) on one MI355X.

One "step" = one fikit_profile call over every launch record of the workload followed by one
fikit_gapfill call over every scenario, inputs resident in HBM.  Default workload: the batched
gap-fill configuration (65,536 scenarios; 4,096 + 16,384 launches each; 1.34 G records).

Prints ONE JSON line.  `value` is launch records per second through the whole step.
`roofline` describes the kernel with the largest share of device time, timed with HIP events
on the stream it runs on (the library's fikit_trace_* facility).  `cpu_baseline` is the CPU
oracle timed on a bounded sample of the same workload on this machine's host cores.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0

# Algorithmic bytes each kernel must move per record it processes (natural widths):
#   one-workgroup task kernels: read the 64-byte record, write the 8-byte ID (rows are negligible)
#   tile partition of long tasks: read the record, write the ID in launch order, write the tile-ordered
#     (ID, 32-bit execution time, 32-bit idle time)
#   one-workgroup kernels on units of a partitioned task: read the tile-ordered triple
#   general path: one sort pass (key, execution time, idle time read and written), per launch of a task that takes it
ALGO_BYTES_PER_RECORD = {
    "k_task_fused_small": 64 + 8,
    "k_task_fused_mid": 64 + 8,
    "k_task_fused_medium": 64 + 8,
    "k_tile_partition": 64 + 8 + 16,
    "k_onesweep_pass": 24 + 24,
    "k_unit_fused": 16,
}
GAPFILL_KERNELS = ("k_gf_predict", "k_gf_walk", "k_gf_predict32", "k_gf_walk_lanes")


def source_hash():
    """Hash of the library sources, to tell whether stored counter readings still describe the library as it stands."""
    from paper_2311_10359_amd import profile_summary
    return profile_summary.source_hash()


TRAFFIC_FILE = os.path.join("profiles", "hbm_traffic.json")


def stored_counters(workload):
    """The committed rocprofv3 counter readings (profiles/hbm_traffic.json, written by
    `python -m paper_2311_10359_amd.profile_summary hbm`) if they are of this workload and of the library as it
    stands, else None: counters read for another build say nothing about this one."""
    try:
        data = json.load(open(os.path.join(ROOT, TRAFFIC_FILE)))
    except (OSError, ValueError):
        log(f"[bench] no stored HBM counters ({TRAFFIC_FILE}): roofline.traffic and hbm_by_call are left out")
        return None
    if workload not in data.get("workloads", {}):
        log(f"[bench] stored HBM counters cover {sorted(data.get('workloads', {}))}, not {workload!r}: traffic left out")
        return None
    data = data["workloads"][workload]
    if data.get("source_hash") != source_hash():
        log(f"[bench] stored HBM counters are of library sources {data.get('source_hash')}, these are {source_hash()}: "
            "the kernels have changed since the counters were taken, traffic left out (null)")
        return None
    return data


def stored_traffic(data, kernel):
    """HBM bytes per launch of one kernel from the stored counter readings."""
    if not data:
        return None
    return data.get("kernels", {}).get(kernel, {}).get("hbm_bytes_per_launch")


def stored_call_traffic(data):
    """HBM bytes per call (all kernels of fikit_profile / of fikit_gapfill, one launch each per step)."""
    if not data:
        return None
    calls = {"fikit_profile": 0, "fikit_gapfill": 0}
    for kname, v in data.get("kernels", {}).items():
        nbytes = v["hbm_bytes_per_launch"]
        if kname in ("k_validate_offsets", "k_clear_ctrl", "k_fill_u32"):   # run in either call (negligible bytes)
            calls["fikit_profile"] += nbytes
            calls["fikit_gapfill"] += nbytes
        elif kname.startswith(("k_gf", "k_pf")):
            calls["fikit_gapfill"] += nbytes
        else:
            calls["fikit_profile"] += nbytes
    return calls


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


A_REF_BYTES_PER_RECORD = 504   # what the sort-based formulation of the profile pass moves per record (hash + measure 88,
                               # one histogram pass 8, eight scatter passes 48 each, reduce 24): the yardstick for "effective" GB/s


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="cfg4", choices=["cfg1", "cfg2", "cfg3", "cfg4"])
    ap.add_argument("--scenarios", type=int, default=None, help="cfg4 only: fewer scenarios (smoke runs)")
    ap.add_argument("--tasks", type=int, default=None, help="cfg1/cfg3 only: fewer tasks (smoke runs)")
    ap.add_argument("--workers", type=int, default=min(16, os.cpu_count() or 1),
                    help="processes that generate the input; 0 = generate in this process")
    ap.add_argument("--cpu-sample-tasks", type=int, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--replay", action="store_true",
                    help="after the timed steps, also time fikit_measure and fikit_gapfill_replay (reported beside "
                         "the metric, not part of it)")
    ap.add_argument("--prio", type=int, default=0, metavar="K",
                    help="after the timed steps, also time fikit_prio_fill with K low-priority tasks per scenario "
                         "(reported beside the metric, not part of it)")
    ap.add_argument("--pairing", action="store_true",
                    help="after the timed steps, also time fikit_pairing_best over the gap fill's results (reported "
                         "beside the metric, not part of it)")
    ap.add_argument("--merge", action="store_true",
                    help="after the timed steps, also time fikit_profile_merge of the profile with itself (reported "
                         "beside the metric, not part of it)")
    ap.add_argument("--rho", type=float, default=None,
                    help="scale of the per-Kernel-ID share of the spread of times in the generated traces (default 1: an ID "
                         "has a characteristic duration; 0: every launch is drawn independently)")
    ap.add_argument("--two-calls", action="store_true",
                    help="a step is fikit_profile followed by fikit_gapfill; default: the two as one call, "
                         "fikit_profile_gapfill, in which the profile's kernels hand the predictions to the gap fill")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run a plain 1 GiB device-to-device copy (reference for hardware counter runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        print(f"bench.py measures one GPU; --gpus {args.gpus} is not supported: tasks and scenarios are independent, "
              "so more GPUs would each run this same program on their own shard (no exchange).", file=sys.stderr)
        sys.exit(2)

    from paper_2311_10359_amd import traces

    if args.workload == "cfg4":
        cfg = traces.config(4, n_tasks=2 * args.scenarios if args.scenarios else None, rho=args.rho)
        sample_tasks = args.cpu_sample_tasks or min(cfg.n_tasks, 16384)   # about 12 s of oracle time
        name = "config 4: batched gap-fill"
    elif args.workload == "cfg2":
        cfg = traces.config(2, n_tasks=args.tasks, rho=args.rho)
        sample_tasks = args.cpu_sample_tasks or min(cfg.n_tasks, 12)
        name = "config 2: skewed IDs (profile only)"
    elif args.workload == "cfg3":
        cfg = traces.config(3, n_tasks=args.tasks, rho=args.rho)
        sample_tasks = args.cpu_sample_tasks or min(cfg.n_tasks, 48)
        name = "config 3: large profile (profile only)"
    else:
        cfg = traces.config(1, n_tasks=args.tasks, rho=args.rho)
        sample_tasks = args.cpu_sample_tasks or cfg.n_tasks
        name = "config 1: medium"
    off = traces.task_offsets(cfg)
    n = int(off[-1])
    hp, lp = traces.scenarios(cfg)
    n_scen = int(hp.size)
    go = traces.gap_offsets(off, hp)
    n_gaps = int(go[-1]) if n_scen else 0
    row_cap = sum(cfg.ids(t) for t in range(cfg.n_tasks))
    log(f"[bench] workload {name}: {n} records, {cfg.n_tasks} tasks, {n_scen} scenarios, {n_gaps} gaps")

    # ---- generate on the host (worker processes) and stream into HBM --------------------------
    t0 = time.time()
    if args.workers > 0:
        gen = traces.stream(cfg, workers=args.workers)
    else:
        # in-process generation: no child processes (use this under a profiler)
        def in_process(chunk=1 << 20):
            lo = 0
            while lo < cfg.n_tasks:
                hi = lo + 1
                while hi < cfg.n_tasks and int(off[hi + 1] - off[lo]) <= chunk:
                    hi += 1
                rec, _ = traces.build(cfg, tasks=range(lo, hi), threads=1 if cfg.launches(lo) < 100000 else 4)
                yield int(off[lo]), rec
                lo = hi
        gen = in_process()
    first_piece = next(gen)   # starts the worker pool before this process touches the GPU
    import torch
    from paper_2311_10359_amd import binding
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    d_rec = torch.empty((n, 64), dtype=torch.uint8, device=dev)
    sample_n = int(off[sample_tasks])
    sample = np.zeros(sample_n, dtype=traces.LAUNCH_DTYPE)
    pieces = 0
    last_print = time.time()

    def take(first, view):
        u8 = view.view(np.uint8).reshape(-1, 64)
        d_rec[first:first + u8.shape[0]].copy_(torch.from_numpy(u8))
        if first < sample_n:
            k = min(sample_n - first, u8.shape[0])
            sample.view(np.uint8).reshape(-1, 64)[first:first + k] = u8[:k]

    take(*first_piece)
    del first_piece
    for first, view in gen:
        take(first, view)
        pieces += 1
        if time.time() - last_print > 20:
            last_print = time.time()
            log(f"[bench] generated and uploaded piece {pieces} ({time.time() - t0:.0f}s)")
    torch.cuda.synchronize()
    log(f"[bench] inputs resident after {time.time() - t0:.1f}s")

    d_off = binding.to_device_u64(off, dev)
    d_hp, d_lp, d_go = binding.to_device_u32(hp, dev), binding.to_device_u32(lp, dev), binding.to_device_u64(go, dev)
    ids = torch.empty(n, dtype=torch.int64, device=dev)
    rows = torch.empty((row_cap, 128), dtype=torch.uint8, device=dev)
    tro = torch.empty(cfg.n_tasks + 1, dtype=torch.int64, device=dev)
    one_call = bool(n_scen) and not args.two_calls
    ws_bytes = max(binding.fikit_profile_workspace_bytes(n, cfg.n_tasks),
                   binding.fikit_gapfill_workspace_bytes(n, cfg.n_tasks, n_scen),
                   binding.fikit_profile_gapfill_workspace_bytes(n, cfg.n_tasks, n_scen) if one_call else 0)
    ws = binding.workspace(ws_bytes, dev)
    gf_out = binding.GapFill(torch.empty(n_gaps, dtype=torch.int32, device=dev),
                             torch.empty(n_gaps, dtype=torch.int64, device=dev),
                             torch.empty(n_scen, dtype=torch.int64, device=dev),
                             torch.empty(n_scen, dtype=torch.int64, device=dev))
    log(f"[bench] device memory in use: {torch.cuda.memory_allocated() / 2**30:.1f} GiB "
        f"(workspace {ws_bytes / 2**30:.1f} GiB)")

    def step(timers=None):
        e = [torch.cuda.Event(enable_timing=True) for _ in range(3)] if timers is not None else None
        if e:
            e[0].record()
        if one_call:
            prof, _ = binding.fikit_profile_gapfill(d_rec, d_off, d_hp, d_lp, d_go, margin_ns=cfg.margin_ns,
                                                    min_gap_ns=cfg.min_gap_ns, n_gaps=n_gaps, ids_out=ids, rows_out=rows,
                                                    task_row_offsets_out=tro, out=gf_out, workspace_buf=ws,
                                                    row_capacity=row_cap)
            if e:
                e[1].record()
                e[2].record()
                timers.append(e)
            return prof
        prof = binding.fikit_profile(d_rec, d_off, ids_out=ids, rows_out=rows, task_row_offsets_out=tro,
                                     workspace_buf=ws, row_capacity=row_cap)
        if e:
            e[1].record()
        if n_scen:
            binding.fikit_gapfill(ids, d_off, prof.rows, tro, d_hp, d_lp, d_go, margin_ns=cfg.margin_ns,
                                  min_gap_ns=cfg.min_gap_ns, n_gaps=n_gaps, n_ids=n, out=gf_out, workspace_buf=ws)
        if e:
            e[2].record()
            timers.append(e)
        return prof

    if args.calibration_copy:
        a = torch.zeros(1 << 28, dtype=torch.int32, device=dev)
        b = torch.empty_like(a)
        b.copy_(a)
        torch.cuda.synchronize()
        del a, b
    for i in range(args.warmup):
        prof = step()
        log(f"[bench] warmup {i + 1}/{args.warmup} done")
    binding.fikit_trace_enable(True)
    timers = []
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for i in range(args.steps):
        prof = step(timers)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    trace = binding.fikit_trace_read()
    binding.fikit_trace_enable(False)
    ms_per_step = elapsed / args.steps * 1e3
    step_ms = [a[0].elapsed_time(a[2]) for a in timers]   # every step by its own events (device time of its calls)
    prof_ms = float(np.median([a[0].elapsed_time(a[1]) for a in timers]))
    gf_ms = float(np.median([a[1].elapsed_time(a[2]) for a in timers]))
    if one_call:
        # one call: the gap fill's share is the time of its own kernels (the trace's gf_* and k_gf_* entries), the
        # profile's the rest; the predictions are written by the profile's kernels and count there
        gf_ms = sum(ms for k, (ms, _) in trace.items() if k.startswith(("gf_", "k_gf_"))) / args.steps
        prof_ms = prof_ms - gf_ms
    log(f"[bench] {ms_per_step:.2f} ms/step (profile {prof_ms:.2f} ms, gap fill {gf_ms:.2f} ms), {prof.n_rows} rows")
    for k, (ms, cnt) in sorted(trace.items(), key=lambda kv: -kv[1][0]):
        log(f"[bench]   {k:18s} {ms / args.steps:9.3f} ms/step  {cnt // args.steps:3d} launches/step")

    # ---- the replay against actual idle times (beside the metric) --------------------------------
    replay = None
    if args.replay and n_scen:
        d_exec, d_gap = binding.fikit_measure(d_rec, d_off, workspace_buf=ws)
        rp_out = binding.Replay(gf_out.fill_count, gf_out.filled_ns, gf_out.lp_completion_ns, gf_out.lp_placed)
        replay = {}
        for feedback in (False, True):
            binding.fikit_gapfill_replay(ids, d_off, prof.rows, tro, d_gap, d_hp, d_lp, d_go, margin_ns=cfg.margin_ns,
                                         min_gap_ns=cfg.min_gap_ns, feedback=feedback, n_gaps=n_gaps, n_ids=n,
                                         out=rp_out, workspace_buf=ws)
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
            binding.fikit_trace_enable(True)
            ev[0].record()
            for _ in range(args.steps):
                binding.fikit_gapfill_replay(ids, d_off, prof.rows, tro, d_gap, d_hp, d_lp, d_go, margin_ns=cfg.margin_ns,
                                             min_gap_ns=cfg.min_gap_ns, feedback=feedback, n_gaps=n_gaps, n_ids=n,
                                             out=rp_out, workspace_buf=ws)
            ev[1].record()
            torch.cuda.synchronize()
            rt = binding.fikit_trace_read()
            binding.fikit_trace_enable(False)
            ms = ev[0].elapsed_time(ev[1]) / args.steps
            replay["feedback" if feedback else "no_feedback"] = {
                "ms": round(ms, 3), "scenarios_per_s": round(n_scen / (ms * 1e-3), 1),
                "mean_hp_delay_ns": round(float(rp_out.hp_delay_ns.double().mean()), 1),
                "kernel_ms": {k: round(v[0] / args.steps, 3) for k, v in rt.items() if k.startswith("k_gf")}}
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        ev[0].record()
        for _ in range(args.steps):
            binding.fikit_measure(d_rec, d_off, exec_out=d_exec, gap_out=d_gap, workspace_buf=ws)
        ev[1].record()
        torch.cuda.synchronize()
        ms = ev[0].elapsed_time(ev[1]) / args.steps
        replay["measure"] = {"ms": round(ms, 3), "records_per_s": round(n / (ms * 1e-3), 1),
                             "algorithmic_GB/s": round(n * 80 / (ms * 1e-3) / 1e9, 1)}
        log(f"[bench] replay: {json.dumps(replay)}")
        del d_exec, d_gap

    # ---- best partner per high-priority task over the gap fill's results (beside the metric) -----
    pairing = None
    if args.pairing and n_scen:
        step()                                     # (the replay leg may have overwritten the gap fill's results)
        pr_out = binding.Pairing(torch.empty(n_scen, dtype=torch.int64, device=dev),
                                 torch.empty(cfg.n_tasks, dtype=torch.int64, device=dev),
                                 torch.empty(cfg.n_tasks, dtype=torch.int32, device=dev),
                                 torch.empty(cfg.n_tasks, dtype=torch.int64, device=dev))

        def pairing_call():
            binding.fikit_pairing_best(d_hp, d_lp, cfg.n_tasks, d_go, gf_out.filled_ns, gf_out.lp_completion_ns, out=pr_out,
                                       workspace_buf=ws)

        pairing_call()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        binding.fikit_trace_enable(True)
        ev[0].record()
        for _ in range(args.steps):
            pairing_call()
        ev[1].record()
        torch.cuda.synchronize()
        rt = binding.fikit_trace_read()
        binding.fikit_trace_enable(False)
        ms = ev[0].elapsed_time(ev[1]) / args.steps
        sum_ms = rt["k_pair_sum"][0] / args.steps
        pairing = {"ms": round(ms, 3), "scenarios_per_s": round(n_scen / (ms * 1e-3), 1),
                   "k_pair_sum_ms": round(sum_ms, 3), "k_pair_sum_algorithmic_GB/s": round(n_gaps * 8 / (sum_ms * 1e-3) / 1e9, 1),
                   "tasks_with_a_partner": int((pr_out.best_lp >= 0).sum()),
                   "mean_best_filled_ms": round(float(pr_out.best_filled_ns[pr_out.best_lp >= 0].double().mean()) / 1e6, 3)}
        log(f"[bench] pairing: {json.dumps(pairing)}")
        del pr_out

    # ---- the profile merged with a second profile of the same tasks (beside the metric) ----------
    merge = None
    if args.merge:
        n_rows = prof.n_rows
        m_rows = torch.empty((n_rows, 128), dtype=torch.uint8, device=dev)
        m_tro = torch.empty(cfg.n_tasks + 1, dtype=torch.int64, device=dev)

        def merge_call():
            return binding.fikit_profile_merge(prof.rows, tro, prof.rows, tro, row_capacity=n_rows, rows_out=m_rows,
                                               task_row_offsets_out=m_tro, workspace_buf=ws)

        merged = merge_call()
        assert merged.n_rows == n_rows
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        binding.fikit_trace_enable(True)
        ev[0].record()
        for _ in range(args.steps):
            merge_call()
        ev[1].record()
        torch.cuda.synchronize()
        rt = binding.fikit_trace_read()
        binding.fikit_trace_enable(False)
        ms = ev[0].elapsed_time(ev[1]) / args.steps
        merge = {"rows_in": 2 * n_rows, "rows_out": n_rows, "ms": round(ms, 3), "rows_out_per_s": round(n_rows / (ms * 1e-3), 1),
                 "algorithmic_GB/s": round(3 * n_rows * 128 / (ms * 1e-3) / 1e9, 1),
                 "kernel_ms": {k: round(v[0] / args.steps, 3) for k, v in rt.items() if k.startswith(("k_", "merge"))}}
        log(f"[bench] profile_merge: {json.dumps(merge)}")
        del m_rows, m_tro

    # ---- several low-priority tasks per scenario in priority queues (beside the metric) ----------
    prio = None
    if args.prio > 0 and n_scen:
        _, p_lo, p_lt, p_lq = traces.prio_scenarios(cfg, args.prio)
        d_plo, d_plt, d_plq = binding.to_device_u64(p_lo, dev), binding.to_device_u32(p_lt, dev), binding.to_device_u32(p_lq, dev)
        pf_out = binding.PrioFill(gf_out.fill_count, gf_out.filled_ns, torch.empty(p_lt.size, dtype=torch.int64, device=dev),
                                  torch.empty(p_lt.size, dtype=torch.int64, device=dev))

        def prio_call():
            binding.fikit_prio_fill(ids, d_off, prof.rows, tro, d_hp, d_plo, d_plt, d_plq, d_go, margin_ns=cfg.margin_ns,
                                    min_gap_ns=cfg.min_gap_ns, n_gaps=n_gaps, n_ids=n, out=pf_out, workspace_buf=ws)

        prio_call()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        binding.fikit_trace_enable(True)
        ev[0].record()
        for _ in range(args.steps):
            prio_call()
        ev[1].record()
        torch.cuda.synchronize()
        rt = binding.fikit_trace_read()
        binding.fikit_trace_enable(False)
        ms = ev[0].elapsed_time(ev[1]) / args.steps
        prio = {"lp_tasks_per_scenario": args.prio, "ms": round(ms, 3), "scenarios_per_s": round(n_scen / (ms * 1e-3), 1),
                "kernels_issued_per_s": round(float(pf_out.lp_placed.sum()) / (ms * 1e-3), 1),
                "mean_kernels_per_gap": round(float(pf_out.fill_count.double().mean()), 4),
                "kernel_ms": {k: round(v[0] / args.steps, 3) for k, v in rt.items() if k.startswith("k_")}}
        log(f"[bench] prio_fill: {json.dumps(prio)}")
        del d_plo, d_plt, d_plq, pf_out

    # ---- roofline of the dominant kernel ------------------------------------------------------
    lens = np.array([cfg.launches(t) for t in range(cfg.n_tasks)], dtype=np.int64)
    n_small = int(lens[lens <= 4096].sum())
    n_mid = int(lens[(lens > 4096) & (lens <= 8192)].sum())
    n_medium = int(lens[(lens > 8192) & (lens <= 16384)].sum())
    n_long = int(lens[lens > 16384].sum())
    n_hp = int(sum(cfg.launches(int(t)) for t in np.unique(hp))) if n_scen else 0
    n_lp = int(sum(cfg.launches(int(t)) for t in np.unique(lp))) if n_scen else 0
    units = {"k_task_fused_small": n_small, "k_task_fused_mid": n_mid, "k_task_fused_medium": n_medium,
             "k_tile_partition": n_long, "k_unit_fused": n_long,
             # (the launches of the long tasks: right where they all take the general path, as in workload 2, the only
             # workload in which this kernel can lead)
             "k_onesweep_pass": n_long}
    # the three launches over the units of partitioned tasks count as one kernel (the split between
    # them depends on the data)
    kernels = {k: v for k, v in trace.items() if k in ALGO_BYTES_PER_RECORD or k in GAPFILL_KERNELS}
    unit_parts = [v for k, v in trace.items() if k.startswith("k_unit_fused_")]
    if unit_parts:
        kernels["k_unit_fused"] = (sum(v[0] for v in unit_parts), max(v[1] for v in unit_parts))
    dom = max(kernels, key=lambda k: kernels[k][0])
    dom_ms, dom_cnt = kernels[dom]
    avg_ms = dom_ms / dom_cnt
    if dom in ALGO_BYTES_PER_RECORD:
        algo_bytes = ALGO_BYTES_PER_RECORD[dom] * units[dom]
        if one_call and n_scen >= 4096 and dom.startswith("k_task_fused_"):
            # one call: the task kernels also write the predictions that the gap fill reads (4 bytes per launch of a
            # task used as queue, 8 per launch of a task used as trace), which k_gf_predict32 writes otherwise
            lo, hi = {"k_task_fused_small": (0, 4096), "k_task_fused_mid": (4096, 8192), "k_task_fused_medium": (8192, 16384)}[dom]
            in_class = (lens > lo) & (lens <= hi)
            is_hp, is_lp = np.zeros(cfg.n_tasks, dtype=bool), np.zeros(cfg.n_tasks, dtype=bool)
            is_hp[hp] = True
            is_lp[lp] = True
            algo_bytes += 8 * int(lens[in_class & is_hp].sum()) + 4 * int(lens[in_class & is_lp].sum())
    elif dom == "k_gf_predict":      # IDs read; prefix sums, idle times and gap-open times written (8 bytes each)
        algo_bytes = 8 * (n_hp + n_lp) + 8 * n_lp + 16 * n_hp
    elif dom == "k_gf_predict32":    # IDs read; 32-bit execution times (queue) and (execution, idle) pairs (trace) written
        algo_bytes = 8 * (n_hp + n_lp) + 4 * n_lp + 8 * n_hp
    else:                            # every scenario reads its trace and its queue once and writes 12 bytes per gap
        per_hp, per_lp = (8, 8) if dom == "k_gf_walk" else (8, 4)
        algo_bytes = per_hp * n_hp * (n_scen // max(1, len(np.unique(hp)))) \
            + per_lp * n_lp * (n_scen // max(1, len(np.unique(lp)))) + 12 * n_gaps
    achieved = algo_bytes / (avg_ms * 1e-3) / 1e9
    # (stored counters of a workload with scenarios are of the one-call step)
    counters = stored_counters(name if one_call or not n_scen else name + " (two calls)") \
        if args.rho is None and not args.scenarios and not args.tasks else None
    traffic_source = (f"{TRAFFIC_FILE} (rocprofv3 FETCH_SIZE / WRITE_SIZE of an earlier run of this command on these library "
                      f"sources, hash {counters['source_hash']}; summary: {counters.get('summary')})") if counters else None
    roofline = {"kernel": dom, "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": stored_traffic(counters, dom),
                "traffic_source": traffic_source,
                "avg_launch_ms": round(avg_ms, 4), "algorithmic_bytes_per_launch": int(algo_bytes),
                "share_of_step": round(dom_ms / args.steps / ms_per_step, 3)}

    # ---- CPU oracle on a bounded sample -------------------------------------------------------
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        s_off = off[: sample_tasks + 1].copy()
        t1 = time.perf_counter()
        o_ids, o_rows, o_tro = oracle.profile(sample, s_off)
        t2 = time.perf_counter()
        pick = np.nonzero((hp < sample_tasks) & (lp < sample_tasks))[0] if n_scen else np.zeros(0, dtype=np.int64)
        s_hp, s_lp = hp[pick], lp[pick]
        o_fill = None
        if pick.size:
            o_fill = oracle.gapfill(o_ids, s_off, o_rows, o_tro, s_hp, s_lp, cfg.margin_ns, cfg.min_gap_ns,
                                    traces.gap_offsets(s_off, s_hp))
        t3 = time.perf_counter()
        cpu = {"value": round(sample_n / (t3 - t1), 1), "unit": "records/s", "cores": 1, "kind": "oracle",
               "sample": f"first {sample_tasks} tasks ({sample_n} records, {pick.size} scenarios) of the same workload: "
                         f"profile {t2 - t1:.2f}s + gap fill {t3 - t2:.2f}s, single thread",
               "profile_records_per_s": round(sample_n / (t2 - t1), 1),
               "gapfill_scenarios_per_s": round(pick.size / (t3 - t2), 1) if pick.size else None,
               "cpu_model": cpu_model(), "host_cpus": os.cpu_count()}
        # the sample doubles as a spot check of the timed run's output
        got_rows = binding.rows_to_numpy(prof.rows[: len(o_rows)])
        assert got_rows.tobytes() == o_rows.tobytes(), "benchmark output differs from the oracle on the sample (rows)"
        assert np.array_equal(binding.u64_to_numpy(ids[:sample_n]), o_ids), "benchmark output differs from the oracle on the sample (IDs)"
        checked = "rows and IDs"
        if o_fill is not None and replay is None and prio is None:      # (those legs reuse the gap fill's output buffers)
            assert np.array_equal(gf_out.lp_completion_ns.cpu().numpy()[pick], o_fill[2]), "completion times differ from the oracle"
            assert np.array_equal(binding.u64_to_numpy(gf_out.lp_placed)[pick], o_fill[3]), "kernels placed differ from the oracle"
            if np.array_equal(pick, np.arange(pick.size)):             # the sample's scenarios are the first ones: their gaps too
                k = int(go[pick.size])
                assert np.array_equal(binding.u32_to_numpy(gf_out.fill_count[:k]), o_fill[0]), "fill counts differ from the oracle"
                assert np.array_equal(gf_out.filled_ns[:k].cpu().numpy(), o_fill[1]), "filled times differ from the oracle"
            checked = "rows, IDs and gap-fill outputs"
        log(f"[bench] oracle sample: {cpu['value'] / 1e6:.2f} M records/s on one core; the sample's {checked} match")

    out = {
        "metric": "launch records/s profiled + gap-fill scenarios/s; % of peak HBM GB/s",
        "value": round(n / (ms_per_step * 1e-3), 1),
        "unit": "records/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int64", "data": "synthetic",
        "config": {"workload": name, "records": n, "tasks": cfg.n_tasks, "scenarios": n_scen, "gaps": n_gaps,
                   "rows": prof.n_rows, "margin_ns": cfg.margin_ns, "min_gap_ns": cfg.min_gap_ns,
                   "rho_exec": cfg.rho_exec, "rho_gap": cfg.rho_gap,
                   "entry_points": "fikit_profile_gapfill" if one_call else "fikit_profile, fikit_gapfill",
                   "generator": f"numpy {np.__version__} PCG64, base seed {traces.BASE_SEED}"},
        "profile_records_per_s": round(n / (prof_ms * 1e-3), 1),
        "gapfill_scenarios_per_s": round(n_scen / (gf_ms * 1e-3), 1) if n_scen else None,
        "profile_ms": round(prof_ms, 3), "gapfill_ms": round(gf_ms, 3),
        "step_ms_by_events": {"median": round(float(np.median(step_ms)), 3), "min": round(min(step_ms), 3),
                              "max": round(max(step_ms), 3)},
        # the profile call against the sort-based formulation's bytes: what that formulation would have to sustain
        # to be as fast (a design that moves fewer bytes shows up here as more than it could physically move)
        "profile_effective_GB/s_at_504_B_per_record": round(n * A_REF_BYTES_PER_RECORD / (prof_ms * 1e-3) / 1e9, 1),
        "kernel_ms_per_step": {k: round(ms / args.steps, 3) for k, (ms, _) in trace.items()},
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    if replay:
        out["replay"] = replay
    if prio:
        out["prio_fill"] = prio
    if pairing:
        out["pairing"] = pairing
    if merge:
        out["profile_merge"] = merge
    # whole calls against the HBM peak: counter-measured bytes of every kernel of the call / the call's time
    calls = stored_call_traffic(counters)
    if calls:
        out["hbm_by_call"] = {
            "traffic_source": traffic_source,
            "fikit_profile": {"bytes": calls["fikit_profile"], "GB/s": round(calls["fikit_profile"] / (prof_ms * 1e-3) / 1e9, 1),
                              "frac_of_peak": round(calls["fikit_profile"] / (prof_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)},
            "fikit_gapfill": {"bytes": calls["fikit_gapfill"], "GB/s": round(calls["fikit_gapfill"] / (gf_ms * 1e-3) / 1e9, 1),
                              "frac_of_peak": round(calls["fikit_gapfill"] / (gf_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)} if n_scen else None,
        }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
