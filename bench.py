#!/usr/bin/env python3
"""Throughput of the fused conv + affine (+ residual) + ReLU blocks, forward and backward.

One step = one pass of the whole path over one batch of synthetic input already resident in
HBM: forward of every block of the workload, the L1-loss gradient, backward of every block
(data gradient, weight gradient, affine-parameter gradients).  The default workload is the
14x14 bottleneck (1x1 1024->256, 3x3 256->256, 1x1 256->1024 + identity shortcut + ReLU, N = 64,
bf16 with fp32 accumulation), the configuration the throughput target is quoted on.

Prints ONE JSON line.
  value / ms_per_step   K steps bracketed by synchronisations, same buffers every step (hot regime).
  launches              every kernel launch of one step, timed live with HIP events on the launch stream
                        (the library's launch trace) after the timed region: microseconds, flops, bytes every
                        operand read / result written once, and the fraction of the roofline that binds it
                        (bf16 MFMA peak or HBM bandwidth).
  roofline              the dominant kernel (the pipelined bf16 MFMA implicit-GEMM kernel that serves forward
                        and data gradient): flops of ALL its launches of a step over the sum of their times.
  regimes               step time with the loss-gradient kernel taken out, and in the cold regime (buffer sets
                        rotated so that the working set exceeds the 256 MB memory-side cache).
  host_enqueue_us       host time to issue one step (no synchronisation), per launch mode.
  cpu_baseline          the fp64 CPU checker timed on a bounded sample of the same workload on this host.
"""
import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0      # MI355X dense bf16 MFMA peak
HBM_PEAK_GBS = 8000.0               # MI355X HBM3E peak
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "dominant_kernel_traffic.json")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=300,
                    help="untimed steps before the timed ones (the clocks settle within the first ~50 ms of work: "
                         "10 warm-up steps measure ~2 %% slower than 300)")
    ap.add_argument("--workload", type=int, default=3, choices=[2, 3, 4, 5])
    ap.add_argument("--batch", type=int, default=0, help="override N (0 = the workload's own)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--launch", choices=["prepared", "eager", "graph"], default="prepared",
                    help="prepared: the step recorded once as a prepared sequence of the library and issued by one "
                         "native call (default); eager: one Python call per block; graph: replay a captured HIP graph")
    ap.add_argument("--lanes", type=int, default=1, choices=[1, 2],
                    help="streams of the backward pass (eager / graph only): 1 = one call per block on one stream "
                         "(the weight re-pack then rides along with the weight-gradient launch), 2 = weight branches "
                         "on a second stream beside the data-gradient chain (measured: no faster)")
    ap.add_argument("--tune", action="store_true",
                    help="before the warm-up, time the candidate launch plans of every layer shape and install the "
                         "winners (seconds; outside the timed region)")
    ap.add_argument("--cpu-sample-images", type=int, default=0,
                    help="images the CPU checker is timed on (0 = per workload: the whole batch of the stem and the "
                         "bottleneck, 8 images of the ResNet-50 and stage-2 schedules: 5 to 30 s)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="first run three plain device copies of 256 MiB (torch's copy kernel): under a counter "
                         "profile their FETCH_SIZE / WRITE_SIZE readings give the scale of those counters")
    ap.add_argument("--no-regimes", action="store_true", help="skip the cold-cache and host-enqueue measurements")
    return ap.parse_args()


def cpu_baseline(wl_factory, images: int):
    """The CPU checker, as it stands, on the first `images` images of the workload."""
    import numpy as np
    from oracle import oracle as orc
    wl = wl_factory(images)
    shp = wl.tensor_shapes()
    t0 = time.perf_counter()
    acts = {0: wl.x.astype(np.float64)}
    for o in wl.ops:
        if o.op != "conv":
            acts[o.out] = orc.maxpool(acts[o.inp], o.k, o.stride, o.pad)
            continue
        p = wl.params[o.layer]
        _, h, w = shp[o.inp]
        d = orc.Desc(wl.n, h, w, o.c_in, o.c_out, o.k, o.k, o.stride, o.pad, o.relu)
        acts[o.out] = orc.block_fwd(d, acts[o.inp], p["W"], p["scale"], p["shift"],
                                    acts[o.res] if o.res is not None else None)
    last = wl.conv_blocks()[-1].out
    grads = {last: orc.l1_grad(acts[last], wl.target)} if wl.train else {}
    for o in reversed(wl.conv_blocks() if wl.train else []):
        p = wl.params[o.layer]
        _, h, w = shp[o.inp]
        d = orc.Desc(wl.n, h, w, o.c_in, o.c_out, o.k, o.k, o.stride, o.pad, o.relu)
        need_dx = not (o.inp == 0 and not wl.need_input_grad)
        g = orc.block_bwd(d, grads[o.out], acts[o.inp], p["W"], acts[o.out], p["scale"], need_dx=need_dx,
                          need_dres=o.res is not None)
        if need_dx:
            grads[o.inp] = g["dx"] if o.inp not in grads else grads[o.inp] + g["dx"]
        if o.res is not None:
            grads[o.res] = g["dres"] if o.res not in grads else grads[o.res] + g["dres"]
    dt = time.perf_counter() - t0
    return wl.flops_step() / dt / 1e12, dt, orc.num_threads()


def stored_traffic(workload: str, n: int):
    """HBM bytes per launch of the dominant kernel's largest launch, from the counter passes summarised in
    profiles/ (written by `python -m paper_2205_10357_amd.profile_summary`), or None when there is no figure for
    this workload or the kernel sources have changed since it was taken."""
    try:
        with open(TRAFFIC_FILE) as f:
            rec = json.load(f)
    except (OSError, ValueError):
        return None
    from paper_2205_10357_amd.profile_summary import source_digest
    if rec.get("workload") != workload or rec.get("global_batch") != n or rec.get("source_digest") != source_digest():
        return None
    return rec.get("hbm_bytes_per_launch")


def launch_costs(wl, seq, B):
    """(kind name, tag) -> (flops, bytes, note) for the launches of one step: flops by the 2*M*K*C_out
    convention, bytes = every operand read once and every result written once by that launch (bf16 tensors
    2 bytes, fp32 4 bytes; for the split weight gradient that includes the fp32 partial tiles)."""
    from paper_2205_10357_amd import workloads
    shp = wl.tensor_shapes()
    n = wl.n
    costs = {}
    calls = {c["op"].layer: c for c in getattr(seq, "_bwd_calls", [])}
    for b in wl.conv_blocks():
        c_in, h, w = shp[b.inp]
        c_out, ho, wo = shp[b.out]
        fl = workloads.conv_flops(n, h, w, b)
        x_b, y_b, w_el = n * h * w * c_in * 2, n * ho * wo * c_out * 2, c_out * b.k * b.k * c_in
        # a strided 1x1 reads only the sampled pixels
        x_read = x_b if b.k > 1 or b.stride == 1 else n * ho * wo * c_in * 2
        costs[("fwd", b.layer)] = (fl, x_read + w_el * 2 + y_b * (2 if b.res is not None else 1), "x + W + y (+ residual)")
        if c_in <= 4:        # few-channel layers: a launch that pads the image to 4 channels precedes the GEMM
            costs[("prepare", b.layer)] = (0, n * h * w * (c_in + 4) * 2, "x + padded x")
        c = calls.get(b.layer)
        if c is None:
            continue
        dg = y_b + w_el * 2 + x_b + (x_b if c["addend"] is not None else 0) + (x_b if c["dx_mask"] is not None else 0)
        costs[("dgrad", b.layer)] = (fl, dg, "dy + packed W + dx (+ addend) (+ mask)")
        if b.k < b.stride:   # pixels no tap reaches (1x1 / stride 2: three of four) are written by a launch of their own
            frac = 1.0 - 1.0 / (b.stride * b.stride)
            per_pixel = 1 + (c["addend"] is not None) + (c["addend"] is not None and c.get("addend_mask") is not None) + \
                (c["dx_mask"] is not None)
            costs[("fill", b.layer)] = (0, int(frac * x_b * per_pixel), "dx (+ addend) (+ masks) on the untouched pixels")
        ws = B.sol_block_workspace_bytes(c["desc"], B.SOL_PASS_BWD)
        part = max(0, ws - w_el * 2)                       # fp32 partial tiles of the split (the rest: packed weights)
        costs[("wgrad", b.layer)] = (fl, y_b + x_read + part + w_el * 4, "dy + x + partials + packed W written")
        costs[("reduce", b.layer)] = (0, part + w_el * 2 + w_el * 4, "partials + W + dW")
    for o in wl.ops:
        if o.op == "maxpool":
            c, h, w = shp[o.inp]
            _, ho, wo = shp[o.out]
            costs[("maxpool", -1)] = (0, n * c * (h * w + ho * wo) * 2, "x + y")
    if wl.train:
        last = wl.conv_blocks()[-1]
        c_out, ho, wo = shp[last.out]
        costs[("l1", -2)] = (0, 3 * n * ho * wo * c_out * 2, "y + t + dy")
    return costs


def per_launch_table(trace, wl, seq, B, steps):
    """Median time per position of the step and the roofline that binds each launch."""
    per_step = len(trace) // steps
    assert per_step * steps == len(trace), (len(trace), steps)
    assert all(trace[s * per_step + i][:2] == trace[i][:2] for s in range(steps) for i in range(per_step)), \
        "the traced steps differ in their launches"
    costs = launch_costs(wl, seq, B)
    names = {b.layer: b.name for b in wl.conv_blocks()}
    rows = []
    seen_gemm = {}
    for pos in range(per_step):
        kind, tag = trace[pos][0], trace[pos][1]
        us = statistics.median(trace[s * per_step + pos][2] for s in range(steps))
        kname = B.sol_trace_kind_name(kind)
        role = None
        if "implicit GEMM" in kname or "few-channel forward" in kname or kname == "fp32 direct":
            # first implicit-GEMM launch of a layer in a step is its forward, the second its data gradient
            seen_gemm[tag] = seen_gemm.get(tag, 0) + 1
            role = "fwd" if seen_gemm[tag] == 1 else "dgrad"
        elif "weight-gradient" in kname:
            role = "wgrad"
        elif kname == "split reduction":
            role = "reduce"
        elif kname == "L1-loss gradient":
            role = "l1"
        elif kname == "max-pool":
            role = "maxpool"
        elif kname == "few-channel prepare":
            role = "prepare"
        elif kname == "tap-less pixel fill":
            role = "fill"
        fl, by, what = costs.get((role, tag), (0, 0, ""))
        if kname.endswith("+ split reduction"):        # the launch also carries the reduction of the weight gradient
            by += costs.get(("reduce", tag), (0, 0, ""))[1]
            role = "dgrad + reduce"
        t_mfma = fl / (MFMA_BF16_PEAK_TFLOPS * 1e12) * 1e6
        t_hbm = by / (HBM_PEAK_GBS * 1e9) * 1e6
        rows.append({
            "launch": f"{names.get(tag, 'loss' if tag == -2 else 'glue')} {role or kname}", "kernel": kname,
            "us": round(us, 2), "gflop": round(fl / 1e9, 3), "bytes": by,
            "pct_mfma_peak": round(100 * t_mfma / us, 1) if us > 0 else None,
            "pct_hbm_peak": round(100 * t_hbm / us, 1) if us > 0 else None,
            "bound": "mfma" if t_mfma >= t_hbm else "hbm",
            "roofline_us": round(max(t_mfma, t_hbm), 2),
        })
    return rows


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU only (the library has no multi-GPU path); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2205_10357_amd import binding as B
    from paper_2205_10357_amd import runner, workloads

    B.lib()
    factories = {
        2: lambda n: workloads.stem_bf16(n=n),
        3: lambda n: workloads.bottleneck14_bf16(n=n),
        4: lambda n: workloads.resnet50_infer_bf16(n=n),
        5: lambda n: workloads.stage2_train_bf16(n=n),
    }
    default_n = {2: 32, 3: 64, 4: 128, 5: 128}[args.workload]
    n = args.batch or default_n
    wl = factories[args.workload](n)
    torch.cuda.set_device(0)
    seq = runner.Sequencer(wl, "cuda:0")
    stream = torch.cuda.current_stream()

    if args.copy_calibration:
        a = torch.ones(64 << 20, dtype=torch.float32, device="cuda:0")
        b = torch.empty_like(a)
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
        del a, b

    tuned = None
    if args.tune:
        from paper_2205_10357_amd import tuning
        seq.step()                                   # real activations and gradients in the buffers the sweep times on
        report = tuning.tune(seq)
        tuned = {name: {k: v["plan"] for k, v in e.items() if v["plan"] is not None} for name, e in report.items()}
        tuned = {k: v for k, v in tuned.items() if v}

    # one step = the same kernels whichever way they are launched
    lanes = args.lanes if args.launch != "prepared" else 1

    def stepper(mode, s):
        if mode == "graph":
            return s.capture(lanes).replay
        if mode == "prepared":
            s.prepared()
            return lambda: s.step_prepared(stream)
        return lambda: s.step(stream, lanes=lanes)

    run_step = stepper(args.launch, seq)
    for _ in range(args.warmup):
        run_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run_step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms = dt / args.steps * 1e3
    flops = wl.flops_step()
    value = flops / (ms * 1e-3) / 1e12

    # ---- every launch of the step, timed with events on the launch stream (the library's launch trace) ----
    trace_steps = max(20, min(100, args.steps))
    points = trace_steps * (8 * len(wl.ops) + 8)       # more than any schedule launches (a backward call: at most 7)
    B.sol_trace_start(points)
    for _ in range(trace_steps):
        seq.step_prepared(stream)
    trace = B.sol_trace_stop(points)
    torch.cuda.synchronize()
    table = per_launch_table(trace, wl, seq, B, trace_steps)
    dom = [r for r in table if r["kernel"].startswith("implicit GEMM (pipelined)")]
    if dom:
        dom_flops = sum(r["gflop"] for r in dom) * 1e9
        dom_us = sum(r["us"] for r in dom)
        achieved = dom_flops / (dom_us * 1e-6) / 1e12
        big = max(dom, key=lambda r: r["gflop"])
        roofline = {"bound": "mfma", "achieved": round(achieved, 2), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": round(achieved / MFMA_BF16_PEAK_TFLOPS, 4),
                    "traffic": stored_traffic(wl.name, n), "traffic_unit": "HBM bytes of the largest launch",
                    "kernel": "igemm_fast_kernel", "launches_per_step": len(dom),
                    "flop_per_step_in_kernel": dom_flops, "avg_us": round(dom_us / len(dom), 3),
                    "sum_us": round(dom_us, 2),
                    "largest_launch": {"launch": big["launch"], "us": big["us"], "algorithmic_bytes": big["bytes"],
                                       "frac": round(big["pct_mfma_peak"] / 100, 4)}}
        # the same figure over the launches that only multiply (the others also carry a split reduction, whose time
        # is in `achieved` above but whose work is bytes, not flops)
        plain = [r for r in dom if r["kernel"] == "implicit GEMM (pipelined)"]
        if plain and len(plain) < len(dom):
            pf, pu = sum(r["gflop"] for r in plain) * 1e9, sum(r["us"] for r in plain)
            roofline["launches_without_riding_reduction"] = {
                "launches_per_step": len(plain), "sum_us": round(pu, 2), "achieved": round(pf / (pu * 1e-6) / 1e12, 2),
                "frac": round(pf / (pu * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4)}
    else:
        roofline = None
    loss_us = sum(r["us"] for r in table if r["kernel"] == "L1-loss gradient")
    kernel_sum_us = sum(r["us"] for r in table)
    roof_sum_us = sum(r["roofline_us"] for r in table)

    regimes = {"hot_ms_per_step": round(ms, 5),
               "hot_ms_per_step_without_loss_gradient": round(ms - loss_us * 1e-3, 5),
               "traced_launch_sum_us": round(kernel_sum_us, 2), "per_launch_roofline_sum_us": round(roof_sum_us, 2),
               # step time not inside any kernel (launch gaps), per launch
               "gap_us_per_launch": round((ms * 1e3 - kernel_sum_us) / max(1, len(table)), 2)}
    host = {}
    if not args.no_regimes:
        # host time to issue a step: enqueue without waiting (few enough steps for the queue to take them all)
        for mode in ("eager", "prepared"):
            f = stepper(mode, seq)
            for _ in range(20):
                f()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(40):
                f()
            host[mode] = round((time.perf_counter() - t0) / 40 * 1e6, 1)
            torch.cuda.synchronize()
        # cold regime: rotate buffer sets until the working set exceeds the 256 MB memory-side cache
        per_set = sum(v for k, v in seq.memory_report().items() if k == "total_training") or \
            seq.memory_report().get("activation_buffers_allocated", 0)
        sets = max(3, int(300e6 // max(per_set, 1)) + 1) if per_set < 300e6 else 1
        if sets > 1 and sets <= 8:
            seqs = [seq] + [runner.Sequencer(wl, "cuda:0") for _ in range(sets - 1)]
            steppers = [stepper("prepared", s) for s in seqs]
            for i in range(3 * sets):
                steppers[i % sets]()
            torch.cuda.synchronize()
            k = max(sets * 10, args.steps // 2 // sets * sets)
            t0 = time.perf_counter()
            for i in range(k):
                steppers[i % sets]()
            torch.cuda.synchronize()
            cold_ms = (time.perf_counter() - t0) / k * 1e3
            regimes["cold_ms_per_step"] = round(cold_ms, 5)
            regimes["cold_buffer_sets"] = sets
            regimes["cold_working_set_bytes"] = int(per_set * sets)
            del seqs, steppers

    blocks = wl.conv_blocks()
    out = {
        "metric": "TFLOP/s fused conv+BN+ReLU fwd+bwd, ResNet-50 shapes bf16; % MFMA peak",
        "value": round(value, 3),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": wl.name, "global_batch": n, "blocks": len(blocks),
                   "launch": {"graph": "hip_graph", "prepared": "prepared_sequence", "eager": "eager"}[args.launch],
                   "backward_lanes": lanes, "installed_plans": tuned,
                   "flop_per_step": flops, "pct_mfma_peak": round(100 * value / MFMA_BF16_PEAK_TFLOPS, 2),
                   "memory_plan_bytes": seq.memory_report()},
        "roofline": roofline,
        "regimes": regimes,
        "host_enqueue_us": host,
        "launches": table,
    }
    if not args.no_cpu_baseline:
        images = min(args.cpu_sample_images or {2: 32, 3: 64, 4: 8, 5: 8}[args.workload], n)
        v, secs, cores = cpu_baseline(factories[args.workload], images)
        out["cpu_baseline"] = {"value": round(v, 6), "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
                               "sample": f"first {images} of {n} images, " +
                                         ("forward + L1 gradient + backward, " if wl.train else "forward, ") +
                                         f"{secs:.1f} s; flops counted dense, while the checker's backward loops skip "
                                         "output elements whose masked gradient is zero (about half after a ReLU), so "
                                         "the rate overstates its arithmetic speed by up to that share of the backward work"}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
