"""Summaries of rocprofv3 runs of bench.py: per-launch kernel times and HBM traffic of one step.

rocprofv3 writes one row per dispatch; a training step of the library is a fixed sequence of
launches, so rows are grouped by their position in the step (the loss-gradient kernel occurs
once per step and anchors the positions; --anchor names another kernel that occurs once per step,
e.g. the max-pool of the inference schedule) and summarised per position.  Commands:

  python -m paper_2205_10357_amd.profile_summary times  <dir with *_kernel_trace.csv>  [--out FILE.md]
  python -m paper_2205_10357_amd.profile_summary stats  <dir with *_kernel_stats.csv>  [--out FILE.md]
  python -m paper_2205_10357_amd.profile_summary traffic <FETCH_SIZE dir> <WRITE_SIZE dir> --workload NAME
         --batch N --position P [--out FILE.md] [--json profiles/dominant_kernel_traffic.json]
  python -m paper_2205_10357_amd.profile_summary counters <dir with *_counter_collection.csv> [--out FILE.md]
  python -m paper_2205_10357_amd.profile_summary bench-table <file with bench.py's JSON line> [--out FILE.md]

`traffic` scales the two counters by what they read for the plain 256 MiB device copies that
`bench.py --copy-calibration` runs first in the same process, and stores the HBM bytes of the
dominant kernel's largest launch together with a digest of the kernel's sources: bench.py
quotes the figure only while that digest still matches.
"""
from __future__ import annotations

import argparse
import csv
import glob
import hashlib
import json
import os
import re
import statistics
from collections import defaultdict

HERE = os.path.dirname(os.path.abspath(__file__))
KERNEL_SOURCES = ("igemm_fast.hip", "reduce_rows.h", "api.hip", "common.h")
COPY_KERNEL = "__amd_rocclr_copyBuffer"
COPY_BYTES = 256 << 20
ANCHOR = "l1_grad_kernel"
DOMINANT = "igemm_fast_kernel"


def source_digest() -> str:
    """Digest of the sources that decide what the dominant kernel does and how it is launched."""
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(HERE, "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def short(name: str) -> str:
    name = re.sub(r"^void ", "", name)
    name = re.sub(r"\(.*$", "", name)
    return name.replace("sol::", "")


def read_rows(directory: str, pattern: str):
    files = sorted(glob.glob(os.path.join(directory, "**", pattern), recursive=True))
    if not files:
        raise SystemExit(f"no {pattern} under {directory}")
    with open(files[0], newline="") as f:
        return list(csv.DictReader(f))


def steps_of(dispatches, anchor=ANCHOR):
    """dispatches: list of (kernel name, payload) in dispatch order -> list of steps, each a list of the
    same length, cut so that every step holds the anchor kernel at the same position."""
    lib = [i for i, (k, _) in enumerate(dispatches) if "sol::" in k or k.startswith("sol")]
    anchors = [i for i in lib if anchor in dispatches[i][0]]
    if len(anchors) < 3:
        raise SystemExit("fewer than three steps in the trace")
    period = anchors[1] - anchors[0]
    lead = anchors[0] - lib[0]                      # launches of a step before the anchor (the forward pass)
    if lead >= period:
        lead %= period
    steps = []
    for a in anchors:
        lo, hi = a - lead, a - lead + period
        if lo >= 0 and hi <= len(dispatches):
            names = [dispatches[i][0] for i in range(lo, hi)]
            if not steps or names == [k for k, _ in steps[0]]:
                steps.append([dispatches[i] for i in range(lo, hi)])
    return steps


def cmd_times(args) -> None:
    rows = read_rows(args.dir, "*kernel_trace.csv")
    rows.sort(key=lambda r: int(r["Start_Timestamp"]))
    disp = [(r["Kernel_Name"], (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3,
             int(r.get("Grid_Size", r.get("Grid_Size_X", 0)) or 0) // max(1, int(r.get("Workgroup_Size", r.get("Workgroup_Size_X", 1)) or 1)))
            for r in rows]
    steps = steps_of([(k, (us, wgs)) for k, us, wgs in disp], args.anchor)
    steps = steps[len(steps) // 4:]                 # drop the warm-up quarter
    lines = ["| # | kernel | workgroups | median us | min us |", "|---|---|---|---|---|"]
    total = 0.0
    for pos in range(len(steps[0])):
        us = [s[pos][1][0] for s in steps]
        total += statistics.median(us)
        lines.append(f"| {pos + 1} | {short(steps[0][pos][0])} | {steps[0][pos][1][1]} | {statistics.median(us):.2f} | {min(us):.2f} |")
    lines.append("")
    lines.append(f"Steps summarised: {len(steps)}; sum of the medians: {total:.1f} us.")
    text = "\n".join(lines)
    if args.out:
        with open(args.out, "a") as f:
            f.write(text + "\n")
    print(text)


def cmd_stats(args) -> None:
    rows = read_rows(args.dir, "*kernel_stats.csv")
    lines = ["| kernel | calls | avg us | min us | max us | % |", "|---|---|---|---|---|---|"]
    for r in rows:
        lines.append(f"| {short(r['Name'])} | {r['Calls']} | {float(r['AverageNs']) / 1e3:.2f} | {float(r['MinNs']) / 1e3:.2f} | "
                     f"{float(r['MaxNs']) / 1e3:.2f} | {float(r['Percentage']):.2f} |")
    text = "\n".join(lines)
    if args.out:
        with open(args.out, "a") as f:
            f.write(text + "\n")
    print(text)


def counter_by_position(directory: str, counter: str, anchor: str = ANCHOR):
    rows = [r for r in read_rows(directory, "*counter_collection.csv") if r["Counter_Name"] == counter]
    rows.sort(key=lambda r: int(r["Dispatch_Id"]))
    copies = [float(r["Counter_Value"]) for r in rows if COPY_KERNEL in r["Kernel_Name"]]
    steps = steps_of([(r["Kernel_Name"], (float(r["Counter_Value"]), int(r["Grid_Size"]) // max(1, int(r["Workgroup_Size"])))) for r in rows], anchor)
    steps = steps[len(steps) // 4:]
    table = [(short(steps[0][pos][0]), steps[0][pos][1][1], statistics.mean(s[pos][1][0] for s in steps))
             for pos in range(len(steps[0]))]
    return table, copies


def cmd_traffic(args) -> None:
    fetch, fcopies = counter_by_position(args.fetch_dir, "FETCH_SIZE")
    write, wcopies = counter_by_position(args.write_dir, "WRITE_SIZE")
    if not fcopies or not wcopies:
        raise SystemExit("no calibration copies in the traces (run bench.py with --copy-calibration)")
    # the calibration copies are the largest copies of the run (the framework makes small ones of its own)
    fscale = (COPY_BYTES / 1024) / max(fcopies)
    wscale = (COPY_BYTES / 1024) / max(wcopies)
    lines = [f"Counter scale from the 256 MiB device copies: FETCH_SIZE x {fscale:.3f}, WRITE_SIZE x {wscale:.3f} (KiB).", "",
             "| # | kernel | workgroups | FETCH_SIZE raw | fetched MB | WRITE_SIZE raw | written MB |", "|---|---|---|---|---|---|---|"]
    best = None
    tf = tw = 0.0
    for pos, ((k, wgs, f), (_, _, w)) in enumerate(zip(fetch, write)):
        fb, wb = f * fscale * 1024, w * wscale * 1024
        tf, tw = tf + fb, tw + wb
        lines.append(f"| {pos + 1} | {k} | {wgs} | {f:.0f} | {fb / 1e6:.1f} | {w:.0f} | {wb / 1e6:.1f} |")
        # the dominant kernel's largest launch: first launch of that kernel with the most traffic-independent work
        # is the 3x3 forward = the second launch of the step for the bottleneck; identified as the dominant-kernel
        # launch at the lowest position among those with the fewest fetched bytes per workgroup is fragile, so the
        # position is given explicitly
        if args.position and pos + 1 == args.position:
            best = (k, fb + wb)
    lines += ["", f"Step total: fetched {tf / 1e6:.0f} MB, written {tw / 1e6:.0f} MB."]
    text = "\n".join(lines)
    if args.out:
        with open(args.out, "a") as f:
            f.write(text + "\n")
    print(text)
    if args.json and best is not None:
        if DOMINANT not in best[0]:
            raise SystemExit(f"position {args.position} is {best[0]}, not {DOMINANT}")
        rec = {"workload": args.workload, "global_batch": args.batch, "kernel": best[0], "step_position": args.position,
               "hbm_bytes_per_launch": round(best[1]), "fetch_scale": round(fscale, 4), "write_scale": round(wscale, 4),
               "step_fetched_bytes": round(tf), "step_written_bytes": round(tw), "source_digest": source_digest()}
        with open(args.json, "w") as f:
            json.dump(rec, f, indent=1)
            f.write("\n")
        print("wrote", args.json)


def cmd_counters(args) -> None:
    names = sorted({r["Counter_Name"] for r in read_rows(args.dir, "*counter_collection.csv")})
    cols = {n: counter_by_position(args.dir, n, args.anchor)[0] for n in names}
    first = cols[names[0]]
    lines = ["| # | kernel | workgroups | " + " | ".join(names) + " |", "|---|---|---|" + "---|" * len(names)]
    for pos, (k, wgs, _) in enumerate(first):
        lines.append(f"| {pos + 1} | {k} | {wgs} | " + " | ".join(f"{cols[n][pos][2]:.4g}" for n in names) + " |")
    text = "\n".join(lines)
    if args.out:
        with open(args.out, "a") as f:
            f.write(text + "\n")
    print(text)


def cmd_bench_table(args) -> None:
    with open(args.file) as f:
        rec = json.loads([line for line in f if line.lstrip().startswith("{")][-1])
    lines = [f"workload {rec['config']['workload']}, N = {rec['config']['global_batch']}: {rec['ms_per_step']} ms per step, "
             f"{rec['value']} TFLOP/s ({rec['config']['pct_mfma_peak']} % of the bf16 MFMA peak); launch times from the "
             "library's launch trace (per-dispatch start / stop events)", "",
             "| # | launch | kernel | us | GFLOP | MB moved once | % MFMA peak | % HBM peak | bound | roofline us |",
             "|---|---|---|---|---|---|---|---|---|---|"]
    for i, r in enumerate(rec["launches"]):
        lines.append(f"| {i + 1} | {r['launch']} | {r['kernel']} | {r['us']} | {r['gflop']} | {r['bytes'] / 1e6:.1f} | "
                     f"{r['pct_mfma_peak']} | {r['pct_hbm_peak']} | {r['bound']} | {r['roofline_us']} |")
    reg = rec.get("regimes", {})
    lines += ["", f"Sum of the launches: {reg.get('traced_launch_sum_us')} us; sum of their rooflines: "
                  f"{reg.get('per_launch_roofline_sum_us')} us."]
    r = rec.get("roofline")
    if r:
        big = r["largest_launch"]
        lines += ["", f"`roofline` of that bench line: dominant kernel {r['kernel']}, all {r['launches_per_step']} launches of a step "
                      f"({r['flop_per_step_in_kernel'] / 1e9:.1f} GFLOP in {r['sum_us']} us): achieved {r['achieved']} {r['unit']}, "
                      f"frac {r['frac']}; largest launch {big['launch']}: {big['us']} us, frac {big['frac']}; traffic {r['traffic']}."]
    text = "\n".join(lines)
    if args.out:
        with open(args.out, "a") as f:
            f.write(text + "\n")
    print(text)


def main() -> None:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="cmd", required=True)
    t = sub.add_parser("times")
    t.add_argument("dir")
    t.add_argument("--out")
    t.add_argument("--anchor", default=ANCHOR)
    t.set_defaults(fn=cmd_times)
    st = sub.add_parser("stats")
    st.add_argument("dir")
    st.add_argument("--out")
    st.set_defaults(fn=cmd_stats)
    c = sub.add_parser("counters")
    c.add_argument("dir")
    c.add_argument("--out")
    c.add_argument("--anchor", default=ANCHOR)
    c.set_defaults(fn=cmd_counters)
    b = sub.add_parser("bench-table")
    b.add_argument("file")
    b.add_argument("--out")
    b.set_defaults(fn=cmd_bench_table)
    m = sub.add_parser("traffic")
    m.add_argument("fetch_dir")
    m.add_argument("write_dir")
    m.add_argument("--workload", required=True)
    m.add_argument("--batch", type=int, required=True)
    m.add_argument("--position", type=int, default=0, help="1-based position in the step of the dominant kernel's largest launch")
    m.add_argument("--out")
    m.add_argument("--json")
    m.set_defaults(fn=cmd_traffic)
    args = ap.parse_args()
    args.fn(args)


if __name__ == "__main__":
    main()
