"""Turns raw rocprofv3 output (CSV) into the short text summaries kept under profiles/.

A measurement aid beside bench.py: nothing in the library or its binding uses it.  Three sub-commands:

  python -m paper_2311_10359_amd.profile_summary ktrace <k_kernel_stats.csv> <out.txt> --cmd "..." [--note "..."]
                                                     [--trace <k_kernel_trace.csv>]
      per kernel: calls, total and average duration, share of device time (rocprofv3 --kernel-trace --stats);
      with --trace also the duration of the 1 GiB calibration copy (bench.py --calibration-copy), the longest
      copy kernel of the run, and the bandwidth it stands for

  python -m paper_2311_10359_amd.profile_summary hbm <fetch.csv> <write.csv> <out.txt> --cmd "..." --workload NAME
                                                     [--json profiles/hbm_traffic.json]
      HBM bytes per kernel and dispatch from two counter runs (FETCH_SIZE in one, WRITE_SIZE in the other; KiB
      per dispatch), each scaled by what the same counter reads for a plain 1 GiB device-to-device copy in the
      same run (bench.py --calibration-copy).  With --json also stores the per-kernel bytes under the
      workload's name, tagged with a hash of the library sources, for bench.py to quote.

  python -m paper_2311_10359_amd.profile_summary pmc <counter_collection.csv> [<more.csv> ...] <out.txt> --cmd "..."
                                                     [--kernels substring,substring]
      per kernel: the average of every collected counter per dispatch, plus a few ratios where their inputs
      were collected (VALU / LDS / memory instructions per wave, busy shares of the kernel's cycles)
"""
from __future__ import annotations

import argparse
import collections
import csv
import hashlib
import json
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GIB_IN_KIB = 1 << 20


def source_hash() -> str:
    """Hash of the library sources without their comments and white space: tells whether stored counter readings
    still describe the code of the library as it stands."""
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2311_10359_amd", "csrc")
    for name in sorted(os.listdir(d)):
        if name.endswith((".h", ".hip")):
            text = open(os.path.join(d, name), encoding="utf-8").read()
            text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
            text = re.sub(r"//[^\n]*", "", text)
            h.update(name.encode())
            h.update("".join(text.split()).encode())
    return h.hexdigest()[:16]


def short_name(kernel: str) -> str:
    return kernel.split("(")[0].replace("void ", "").strip()


def ktrace(args) -> None:
    rows = list(csv.DictReader(open(args.inputs[0])))
    out = args.inputs[1]
    with open(out, "w") as f:
        f.write("rocprofv3 kernel-trace summary\ncommand: " + args.cmd + "\n")
        if args.note:
            f.write(args.note + "\n")
        f.write(f"\n{'kernel':66s} {'calls':>6s} {'total_us':>14s} {'avg_us':>12s} {'pct':>7s}\n")
        for r in rows:
            f.write(f"{short_name(r['Name'])[:66]:66s} {int(r['Calls']):6d} {float(r['TotalDurationNs']) / 1e3:14.1f} "
                    f"{float(r['AverageNs']) / 1e3:12.1f} {float(r['Percentage']):7.2f}\n")
        if args.trace:
            copies = [int(r["End_Timestamp"]) - int(r["Start_Timestamp"]) for r in csv.DictReader(open(args.trace))
                      if "copyBuffer" in r["Kernel_Name"]]
            if copies:
                ns = max(copies)
                f.write(f"\nplain device-to-device copy of 1 GiB (the longest copy kernel of the run): {ns / 1e3:.1f} us = "
                        f"{2 * (1 << 30) / ns / 1e3:.2f} TB/s read + written\n")
    print(open(out).read())


def per_dispatch(path: str):
    """{kernel: {counter: {dispatch: value}}} (a counter's instances within a dispatch are summed)."""
    agg = collections.defaultdict(lambda: collections.defaultdict(lambda: collections.defaultdict(float)))
    for r in csv.DictReader(open(path)):
        agg[short_name(r["Kernel_Name"])][r["Counter_Name"]][r["Dispatch_Id"]] += float(r["Counter_Value"])
    return agg


def kernel_label(name: str) -> str:
    """The name bench.py's per-kernel timing uses for a kernel (template instances of the task kernel by shape)."""
    n = name.replace("fikit::", "")
    if n.startswith("k_task_fused<"):
        a = [x.strip() for x in n[len("k_task_fused<"):].rstrip(">").split(",")]
        shape = {("512", "8"): "small", ("512", "16"): "mid", ("1024", "16"): "medium"}.get((a[0], a[1]), "x".join(a[:2]))
        return ("k_unit_fused_" if a[5] == "true" else "k_task_fused_") + shape
    return n.split("<")[0]


def hbm(args) -> None:
    fetch_csv, write_csv, out = args.inputs
    f, w = per_dispatch(fetch_csv), per_dispatch(write_csv)

    def copy_reading(agg, counter):
        vals = [v for k in agg if "copyBuffer" in k for v in agg[k][counter].values()]
        if not vals:
            raise SystemExit("no copy kernel in the run: add --calibration-copy to the bench command")
        return max(vals)           # the 1 GiB calibration copy is the largest copy of the run
    cf, cw = copy_reading(f, "FETCH_SIZE"), copy_reading(w, "WRITE_SIZE")
    ff, fw = GIB_IN_KIB / cf, GIB_IN_KIB / cw
    kernels = {}
    lines = []
    total_r = total_w = 0.0
    for k in sorted(f, key=lambda k: -sum(f[k]["FETCH_SIZE"].values())):
        fd, wd = f[k]["FETCH_SIZE"], w.get(k, {}).get("WRITE_SIZE", {})
        n = len(fd)
        rd = sum(fd.values()) / n * ff * 1024
        wr = (sum(wd.values()) / max(1, len(wd))) * fw * 1024
        lines.append(f"{k[:62]:62s} {n:5d} {rd / 1e9:10.3f} {wr / 1e9:10.3f}")
        if k.startswith("fikit::"):
            lab = kernel_label(k)
            e = kernels.setdefault(lab, {"hbm_bytes_per_launch": 0, "read_bytes": 0, "write_bytes": 0, "launches": n})
            e["read_bytes"] += int(rd)
            e["write_bytes"] += int(wr)
            e["hbm_bytes_per_launch"] += int(rd + wr)
            total_r += rd * n / max(1, args.calls)
            total_w += wr * n / max(1, args.calls)
    with open(out, "w") as o:
        o.write("rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE summary (two runs, one counter each)\ncommands: " + args.cmd + "\n")
        if args.note:
            o.write(args.note + "\n")
        o.write(f"calibration: a plain 1 GiB device-to-device copy in the same runs read FETCH_SIZE = {cf:.0f} and "
                f"WRITE_SIZE = {cw:.0f}\n(KiB expected: {GIB_IN_KIB}); scale factors {ff:.4f} (fetch) and {fw:.4f} (write).\n\n")
        o.write(f"{'kernel (bytes per dispatch, averaged over its dispatches)':62s} {'disp':>5s} {'read GB':>10s} {'write GB':>10s}\n")
        o.write("\n".join(lines) + "\n")
        if args.calls:
            o.write(f"\nall library kernels, per call of the library ({args.calls} calls in the run): "
                    f"{total_r / 1e9:.2f} GB read + {total_w / 1e9:.2f} GB written = {(total_r + total_w) / 1e9:.2f} GB\n")
    print(open(out).read())
    if args.json:
        try:
            stored = json.load(open(args.json))
        except (OSError, ValueError):
            stored = {}
        stored.setdefault("workloads", {})[args.workload] = {
            "source_hash": source_hash(), "fetch_scale": ff, "write_scale": fw,
            "summary": os.path.relpath(os.path.abspath(out), ROOT), "kernels": kernels}
        json.dump({"workloads": stored["workloads"]}, open(args.json, "w"), indent=1)
        print("wrote", args.json)


def pmc(args) -> None:
    *inputs, out = args.inputs
    want = [s for s in (args.kernels or "").split(",") if s]
    merged = collections.defaultdict(dict)      # kernel -> counter -> (average per dispatch, dispatches)
    for path in inputs:
        for k, counters in per_dispatch(path).items():
            if want and not any(s in k for s in want):
                continue
            for c, d in counters.items():
                merged[k][c] = (sum(d.values()) / len(d), len(d))
    with open(out, "w") as o:
        o.write("rocprofv3 --pmc summary (averages per dispatch; a counter's instances are summed)\ncommands: " + args.cmd + "\n")
        if args.note:
            o.write(args.note + "\n")
        for k in sorted(merged):
            c = {name: v for name, (v, _) in merged[k].items()}
            o.write(f"\n{k}  ({max(n for _, n in merged[k].values())} dispatches)\n")
            for name in sorted(c):
                o.write(f"  {name:34s} {c[name]:18.1f}\n")
            waves = c.get("SQ_WAVES")
            if waves:
                for name in ("SQ_INSTS_VALU", "SQ_INSTS_SALU", "SQ_INSTS_LDS", "SQ_INSTS_VMEM_RD", "SQ_INSTS_VMEM_WR"):
                    if name in c:
                        o.write(f"  {name + ' per wave':34s} {c[name] / waves:18.1f}\n")
            busy = c.get("SQ_BUSY_CYCLES")
            if busy and "SQ_WAVE_CYCLES" in c:
                o.write(f"  {'waves resident per busy SQ cycle':34s} {c['SQ_WAVE_CYCLES'] / busy:18.2f}\n")
            wc = c.get("SQ_WAVE_CYCLES")
            if wc:
                for name in ("SQ_WAIT_INST_ANY", "SQ_WAIT_INST_LDS", "SQ_WAIT_ANY", "SQ_ACTIVE_INST_ANY", "SQ_ACTIVE_INST_VALU", "SQ_ACTIVE_INST_LDS",
                             "SQ_ACTIVE_INST_VMEM", "SQ_ACTIVE_INST_SCA"):
                    if name in c:
                        o.write(f"  {name + ' / SQ_WAVE_CYCLES':34s} {c[name] / wc:18.3f}\n")
            if c.get("SQ_LDS_IDX_ACTIVE") and "SQ_LDS_BANK_CONFLICT" in c:
                o.write(f"  {'LDS bank-conflict cycles / active':34s} {c['SQ_LDS_BANK_CONFLICT'] / c['SQ_LDS_IDX_ACTIVE']:18.3f}\n")
    print(open(out).read())


def main() -> None:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("what", choices=["ktrace", "hbm", "pmc"])
    ap.add_argument("inputs", nargs="+")
    ap.add_argument("--cmd", required=True, help="the full rocprofv3 command line(s) that produced the input")
    ap.add_argument("--note", default="")
    ap.add_argument("--workload", default="")
    ap.add_argument("--json", default="")
    ap.add_argument("--kernels", default="")
    ap.add_argument("--trace", default="", help="ktrace: the run's k_kernel_trace.csv")
    ap.add_argument("--calls", type=int, default=0, help="hbm: calls of the library in the run (warm-up + steps), for the per-call total")
    args = ap.parse_args()
    {"ktrace": ktrace, "hbm": hbm, "pmc": pmc}[args.what](args)


if __name__ == "__main__":
    main()
