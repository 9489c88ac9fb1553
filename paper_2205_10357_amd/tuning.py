"""Per-layer launch plans found by timing.

The paper tunes the implementation of every layer when a network is compiled (section "SOL
architecture", auto-tuning).  The library's own choice of tile shape, pipeline depth and
weight-gradient split comes from thresholds measured once over the benchmark network; this
module repeats that measurement for the layers of one workload on the GPU at hand: every
distinct layer shape is timed with each candidate plan, using the sequencer's own buffers,
and the fastest is installed with ``sol_block_set_plan`` when it beats the library's choice
by a margin.  A sweep takes well under a second per layer shape.

Only speed depends on a plan (see the header: forward and data gradient are plan-independent
bit for bit, the weight gradient differs in the order of its fp32 partial sums).  The timed
calls overwrite the sequencer's activations and gradients: run a step afterwards.
"""
from __future__ import annotations

from typing import Callable, Dict, List, Optional, Tuple

import torch

from . import binding as B
from .runner import Sequencer

GEMM_CANDIDATES: List[Tuple[int, int]] = [(t, s) for t in (0, 1, 2) for s in (2, 3, 4)]
LARGE_TILE_CANDIDATES: List[Tuple[int, int]] = [(3, 2), (3, 3)]
WGRAD_TARGETS = (192, 256, 384, 512, 768)       # workgroups aimed at; the split count follows from the tile count


def _time_ms(call: Callable[[], None], iters: int) -> float:
    for _ in range(2):
        call()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    start.record()
    for _ in range(iters):
        call()
    stop.record()
    stop.synchronize()
    return start.elapsed_time(stop) / iters


def _shape_key(d: B.BlockDesc) -> tuple:
    return (d.N, d.H, d.W, d.C_in, d.C_out, d.KH, d.KW, d.stride, d.pad, d.dtype)


def _best(desc: B.BlockDesc, which: int, candidates: List[tuple], call: Callable[[], None], iters: int,
          margin: float, before: Optional[Callable[[], None]] = None) -> dict:
    """Times the library's own choice and every candidate; leaves the winner installed (or nothing)."""
    B.sol_block_set_plan(desc, which, None)
    if before:
        before()
    t_default = _time_ms(call, iters)
    best_plan, best_t = None, t_default
    for plan in candidates:
        B.sol_block_set_plan(desc, which, plan)
        if before:
            before()
        t = _time_ms(call, iters)
        if t < best_t:
            best_plan, best_t = plan, t
    if best_plan is not None and best_t < (1.0 - margin) * t_default:
        B.sol_block_set_plan(desc, which, best_plan)
    else:
        B.sol_block_set_plan(desc, which, None)
        best_plan, best_t = None, t_default
    return {"plan": best_plan, "default_ms": t_default, "best_ms": best_t}


def tune(seq: Sequencer, iters: int = 20, margin: float = 0.03) -> Dict[str, Dict[str, dict]]:
    """Install the fastest plan for every distinct layer shape of ``seq``'s workload.

    Returns {layer name: {"fwd" | "dgrad" | "wgrad": {"plan", "default_ms", "best_ms"}}} for the layers
    that were timed (the first layer of each shape; layers the pipelined kernels do not serve are skipped).
    """
    if not seq.bf16:
        return {}
    report: Dict[str, Dict[str, dict]] = {}
    seen = set()
    bwd_calls = {c["op"].layer: c for c in getattr(seq, "_bwd_calls", [])}
    for o in seq.ops:
        if o.op != "conv":
            continue
        d = seq.desc[o.layer]
        if _shape_key(d) in seen or d.C_in % 64 or d.C_out % 8:
            continue
        seen.add(_shape_key(d))
        p = seq.params[o.layer]
        entry: Dict[str, dict] = {}
        rows = d.N * d.Ho * d.Wo
        gemm = GEMM_CANDIDATES + (LARGE_TILE_CANDIDATES if rows >= 256 * 256 else [])
        res = seq.act[o.res] if o.res is not None else None

        def fwd():
            B.sol_block_fwd(d, seq.act[o.inp], p["W"], p["scale"], p["shift"], res, seq.act[o.out], seq.ws, None)
        entry["fwd"] = _best(d, B.SOL_PLAN_FWD, [(t, s, 0) for t, s in gemm], fwd, iters, margin)

        c = bwd_calls.get(o.layer)
        if c is not None:
            g = seq.grads[o.layer]
            # Both gradients are timed in the call the sequencer issues: one backward call for dx and dW together.  Its
            # launches share work (the weight re-pack rides with the weight gradient, the split reduction with the data
            # gradient), so a plan that wins for one branch alone can lose in the call.
            def backward():
                B.sol_block_bwd(c["desc"], c["dy"], seq.act[o.inp], p["W"], None, c["dx"], g["dW"], g["dscale"],
                                g["dshift"], p["scale"], None, c["addend"], None, c["dx_mask"], seq.ws, None)
            if c["dx"] is not None and d.stride * d.stride <= 4:
                in_rows = d.N * d.H * d.W
                cand = GEMM_CANDIDATES + (LARGE_TILE_CANDIDATES if in_rows >= 256 * 256 else [])
                entry["dgrad"] = _best(c["desc"], B.SOL_PLAN_DGRAD, [(t, s, 0) for t, s in cand], backward, iters, margin)
            wgrad = backward

            def grow_workspace():               # more splits need more room for the fp32 partial tiles
                need = B.sol_block_workspace_bytes(c["desc"], B.SOL_PASS_BWD)
                if need > seq.ws.numel():
                    torch.cuda.synchronize()
                    seq.ws = torch.empty((need,), dtype=torch.uint8, device=seq.device)
                    seq._prepared = None          # a prepared step recorded the old workspace
            tiles = -(-(d.KH * d.KW * d.C_in) // 128) * -(-d.C_out // 128)
            splits = sorted({max(1, -(-t // tiles)) for t in WGRAD_TARGETS})
            entry["wgrad"] = _best(c["desc"], B.SOL_PLAN_WGRAD, [(-1, s, k) for k in splits for s in (2, 3)], wgrad,
                                   iters, margin, before=grow_workspace)
            grow_workspace()
        report[o.name] = entry
    torch.cuda.synchronize()
    return report
