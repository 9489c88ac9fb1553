"""Summaries of rocprofv3 runs of bench.py: per-launch kernel times and HBM traffic of one step.

rocprofv3 writes one row per dispatch; a training step of the library is a fixed sequence of
launches, so rows are grouped by their position in the step (the loss-gradient kernel occurs
once per step and anchors the positions) and summarised per position.  Two commands:

  python -m paper_2205_10357_amd.profile_summary times  <dir with *_kernel_trace.csv>  [--out FILE.md]
  python -m paper_2205_10357_amd.profile_summary traffic <FETCH_SIZE dir> <WRITE_SIZE dir> --workload NAME
         --batch N [--out FILE.md] [--json profiles/dominant_kernel_traffic.json]

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
KERNEL_SOURCES = ("igemm_fast.hip", "api.hip", "common.h")
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


def steps_of(dispatches):
    """dispatches: list of (kernel name, payload) in dispatch order -> list of steps, each a list of the
    same length, cut so that every step holds the anchor kernel at the same position."""
    lib = [i for i, (k, _) in enumerate(dispatches) if "sol::" in k or k.startswith("sol")]
    anchors = [i for i in lib if ANCHOR in dispatches[i][0]]
    if len(anchors) < 3:
        raise SystemExit("fewer than three steps in the trace")
    period = anchors[1] - anchors[0]
    lead = anchors[0] - lib[0]                      # launches of a step before the anchor (the forward pass)
    if lead >= period:
        lead %= period
    steps = []
    for a in anchors:
        lo, hi = a - lead, a - lead + period
        if lo >= 0 and hi <= len(dispatches) and all(ANCHOR in dispatches[lo + lead][0] for _ in (0,)):
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
    steps = steps_of([(k, (us, wgs)) for k, us, wgs in disp])
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


def counter_by_position(directory: str, counter: str):
    rows = [r for r in read_rows(directory, "*counter_collection.csv") if r["Counter_Name"] == counter]
    rows.sort(key=lambda r: int(r["Dispatch_Id"]))
    copies = [float(r["Counter_Value"]) for r in rows if COPY_KERNEL in r["Kernel_Name"]]
    steps = steps_of([(r["Kernel_Name"], (float(r["Counter_Value"]), int(r["Grid_Size"]) // max(1, int(r["Workgroup_Size"])))) for r in rows])
    steps = steps[len(steps) // 4:]
    table = [(short(steps[0][pos][0]), steps[0][pos][1][1], statistics.mean(s[pos][1][0] for s in steps))
             for pos in range(len(steps[0]))]
    return table, copies


def cmd_traffic(args) -> None:
    fetch, fcopies = counter_by_position(args.fetch_dir, "FETCH_SIZE")
    write, wcopies = counter_by_position(args.write_dir, "WRITE_SIZE")
    if not fcopies or not wcopies:
        raise SystemExit("no calibration copies in the traces (run bench.py with --copy-calibration)")
    fscale = (COPY_BYTES / 1024) / statistics.median(fcopies)
    wscale = (COPY_BYTES / 1024) / statistics.median(wcopies)
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


def main() -> None:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="cmd", required=True)
    t = sub.add_parser("times")
    t.add_argument("dir")
    t.add_argument("--out")
    t.set_defaults(fn=cmd_times)
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
