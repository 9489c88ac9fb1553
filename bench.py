#!/usr/bin/env python3
"""Throughput of the fused conv + affine (+ residual) + ReLU blocks, forward and backward.

One step = one pass of the whole path over one batch of synthetic input already resident in
HBM: forward of every block of the workload, the L1-loss gradient, backward of every block
(data gradient, weight gradient, affine-parameter gradients).  The default workload is the
14x14 bottleneck (1x1 1024->256, 3x3 256->256, 1x1 256->1024 + identity shortcut + ReLU, N = 64,
bf16 with fp32 accumulation), the configuration the throughput target is quoted on.

Prints ONE JSON line.  `roofline` describes the dominant kernel (the pipelined bf16 MFMA
implicit-GEMM kernel, which serves the forward pass and the data gradient; timed on its largest
launch of the step, the 3x3 forward convolution, in a loop of its own after the timed steps) with
HIP events on the launch stream; `cpu_baseline` is the fp64 CPU checker timed on a bounded sample of the same
workload on this host.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0      # MI355X dense bf16 MFMA peak

# HBM bytes per launch of the dominant kernel on the default workload (3x3 forward convolution of the 14x14 bottleneck,
# N = 64), from the FETCH_SIZE / WRITE_SIZE passes summarised in profiles/bottleneck14_bf16_step_counters.md:
# 8004.5 KiB x 2.000 (copy-kernel scale) fetched + 6272 KiB written.  Valid for the kernel those passes ran; set to None
# whenever csrc/igemm_fast.hip or its launch heuristics change, until the passes are repeated.
DOMINANT_KERNEL_TRAFFIC_BYTES = {("bottleneck14_bf16", 64): (8004.5 * 2.000 + 6272) * 1024}


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
    ap.add_argument("--launch", choices=["eager", "graph"], default="eager",
                    help="eager: launch every kernel from the host (default; measured fastest); graph: replay a "
                         "captured HIP graph of the step")
    ap.add_argument("--lanes", type=int, default=1, choices=[1, 2],
                    help="streams of the backward pass: 1 = one call per block on one stream (default; the weight "
                         "re-pack then rides along with the weight-gradient launch), 2 = weight branches on a second "
                         "stream beside the data-gradient chain (measured: no faster)")
    ap.add_argument("--tune", action="store_true",
                    help="before the warm-up, time the candidate launch plans of every layer shape and install the "
                         "winners (seconds; outside the timed region)")
    ap.add_argument("--cpu-sample-images", type=int, default=0,
                    help="images the CPU checker is timed on (0 = per workload: the whole batch of the stem and the "
                         "bottleneck, 8 images of the ResNet-50 and stage-2 schedules: 5 to 30 s)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="first run three plain device copies of 256 MiB (torch's copy kernel): under a counter "
                         "profile their FETCH_SIZE / WRITE_SIZE readings give the scale of those counters")
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


def workloads_bytes(n, shp, b):
    """Operands read once + result written once for one forward launch of block b (bf16)."""
    c_in, h, w = shp[b.inp]
    c_out, ho, wo = shp[b.out]
    x = n * h * w * c_in * 2
    y = n * ho * wo * c_out * 2
    wgt = c_out * b.k * b.k * c_in * 2
    return x + wgt + y + (y if b.res is not None else 0)


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

    # one step = the same kernels either way
    lanes = args.lanes
    run_step = seq.capture(lanes).replay if args.launch == "graph" else (lambda: seq.step(lanes=lanes))
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

    # ---- dominant kernel: the implicit-GEMM kernel on the largest forward launch of the step ----
    shp = wl.tensor_shapes()
    blocks = wl.conv_blocks()
    big = max(blocks, key=lambda b: workloads.conv_flops(n, shp[b.inp][1], shp[b.inp][2], b))
    kflops = workloads.conv_flops(n, shp[big.inp][1], shp[big.inp][2], big)
    p = seq.params[big.layer]
    reps = max(50, args.steps)

    def launch():
        B.sol_block_fwd(seq.desc[big.layer], seq.act[big.inp], p["W"], p["scale"], p["shift"],
                        seq.act[big.res] if big.res is not None else None, seq.act[big.out], seq.ws, None, stream)

    for _ in range(10):
        launch()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(reps):
        launch()
    e1.record(stream)
    torch.cuda.synchronize()
    k_us = e0.elapsed_time(e1) / reps * 1e3
    achieved = kflops / (k_us * 1e-6) / 1e12

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
                   "launch": "hip_graph" if args.launch == "graph" else "eager", "backward_lanes": lanes,
                   "installed_plans": tuned,
                   "flop_per_step": flops, "pct_mfma_peak": round(100 * value / MFMA_BF16_PEAK_TFLOPS, 2),
                   "memory_plan_bytes": seq.memory_report()},
        "roofline": {"bound": "mfma", "achieved": round(achieved, 2), "peak": MFMA_BF16_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": round(achieved / MFMA_BF16_PEAK_TFLOPS, 4),
                     "traffic": DOMINANT_KERNEL_TRAFFIC_BYTES.get((wl.name, n)), "traffic_unit": "bytes/launch",
                     "algorithmic_bytes": workloads_bytes(n, shp, big),
                     "kernel": "igemm_fast_kernel", "launch": f"{big.name} forward", "avg_us": round(k_us, 3)},
    }
    if not args.no_cpu_baseline:
        images = min(args.cpu_sample_images or {2: 32, 3: 64, 4: 8, 5: 8}[args.workload], n)
        v, secs, cores = cpu_baseline(factories[args.workload], images)
        out["cpu_baseline"] = {"value": round(v, 6), "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
                               "sample": f"first {images} of {n} images, " +
                                         ("forward + L1 gradient + backward, " if wl.train else "forward, ") +
                                         f"{secs:.1f} s"}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
