"""Static layer-list sequencing of fused blocks on one GPU.

The paper's compiled network is a single library holding the whole execution pipeline
with a static schedule (section "SOL architecture", last paragraph before the SDK note;
section on memory consumption).  Here the schedule is the op list of a
``workloads.Workload``: one ``sol_block_fwd`` per convolution block in order, the loss
gradient, then one ``sol_block_bwd`` per block in reverse order.  torch is used only to
own device buffers and the stream; every arithmetic step runs in the library's kernels.

Layer merging across blocks in the backward pass (the paper's grouping of connected layers):
  * every stored activation gradient is already masked by the ReLU of the block that produced
    the activation: the loss kernel masks by its own y, and every data-gradient epilogue masks
    by the block input it differentiates (``dx_mask``).  Blocks therefore run backward without
    SOL_RELU and without reading their y in the two gradient GEMMs;
  * shortcut gradients never get a pass of their own: an identity shortcut is added in the
    epilogue of the data gradient that writes the block input's gradient (``dx_addend``), and a
    projection shortcut simply takes the tail block's (masked) gradient as its dy.

Two lanes in the backward pass.  Only the data gradients form a chain (each block's dx is the next
block's dy); a block's weight branch (weight gradient, its reduction, dscale, dshift) is a leaf that
needs nothing but that block's dy and x.  At ResNet sizes neither kind of kernel fills the chip
(a data-gradient GEMM has fewer tiles than there are compute units), so ``backward(lanes=2)``
issues the weight branches on a second stream that waits, block by block, for the gradient they
read, and joins the first stream at the end of the step.  The second lane has a workspace of its
own: where a call keeps its packed weights and its split partials inside the workspace depends on
the block's shape, and the weight branch of one block is still running when the data branch of
the next one starts.  Measured, two lanes are no faster than one (the large kernels of both lanes
each want the whole chip, and a captured graph runs its branches no faster than one stream), so
one lane is the default.
"""
from __future__ import annotations

from typing import Dict, List, Optional

import numpy as np
import torch

from . import binding as B
from .workloads import ConvBlock, Workload, out_size


def nchw_to_nhwc(a: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(np.transpose(a, (0, 2, 3, 1)))


def nhwc_to_nchw(a: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(np.transpose(a, (0, 3, 1, 2)))


def oihw_to_krsc(w: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(np.transpose(w, (0, 2, 3, 1)))


def krsc_to_oihw(w: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(np.transpose(w, (0, 3, 1, 2)))


def upload(a: np.ndarray, dtype: torch.dtype, device) -> torch.Tensor:
    """float32 host values (already on the storage grid of `dtype`) -> device tensor."""
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device=device, dtype=dtype)


def download(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(device="cpu", dtype=torch.float64).numpy()


class Sequencer:
    """Device buffers + launch order for one workload."""

    def __init__(self, wl: Workload, device="cuda:0", retain_activations: Optional[bool] = None):
        """retain_activations: keep every activation in a buffer of its own.  Training always does (the
        backward pass reads them); inference by default does not (None -> planned arena), unless a caller
        wants to look at the intermediate tensors afterwards."""
        self.wl = wl
        self.retain = wl.train or bool(retain_activations)
        self.device = torch.device(device)
        self.bf16 = wl.dtype == "bf16"
        self.sol_dtype = B.SOL_BF16 if self.bf16 else B.SOL_F32
        self.tdtype = torch.bfloat16 if self.bf16 else torch.float32
        self.shapes = wl.tensor_shapes()              # tensor id -> (C, H, W)
        self.ops = wl.ops
        n = wl.n
        self.act: Dict[int, torch.Tensor] = {}        # NHWC activations
        self.act[0] = upload(nchw_to_nhwc(wl.x), self.tdtype, self.device)
        if self.retain:
            # the backward pass reads every block input and every mask: one buffer per activation
            for o in self.ops:
                c, h, w = self.shapes[o.out]
                self.act[o.out] = torch.empty((n, h, w, c), dtype=self.tdtype, device=self.device)
        else:
            # inference version of the schedule: nothing is retained, activations share one arena whose
            # ranges are reused as soon as a tensor's last reader has run (planned from the static op order)
            offsets, arena_bytes = wl.plan_inference_arena()
            self.arena = torch.empty((max(arena_bytes, 256),), dtype=torch.uint8, device=self.device)
            es = 2 if self.bf16 else 4
            for o in self.ops:
                c, h, w = self.shapes[o.out]
                nbytes = n * h * w * c * es
                self.act[o.out] = self.arena[offsets[o.out]:offsets[o.out] + nbytes].view(self.tdtype).view(n, h, w, c)
        self.params: Dict[int, Dict[str, torch.Tensor]] = {}
        self.desc: Dict[int, B.BlockDesc] = {}
        ws_bytes = 0
        for o in self.ops:
            if o.op != "conv":
                continue
            p = wl.params[o.layer]
            self.params[o.layer] = {
                "W": upload(oihw_to_krsc(p["W"]), self.tdtype, self.device),
                "scale": upload(p["scale"], torch.float32, self.device),
                "shift": upload(p["shift"], torch.float32, self.device),
            }
            _, h, w = self.shapes[o.inp]
            d = B.BlockDesc(n, h, w, o.c_in, o.c_out, o.k, o.k, o.stride, o.pad, self.sol_dtype,
                            B.SOL_RELU if o.relu else 0)
            self.desc[o.layer] = d
            ws_bytes = max(ws_bytes, B.sol_block_workspace_bytes(d, B.SOL_PASS_FWD))
            if wl.train:
                # the backward calls carry the descriptor without SOL_RELU (gradients are stored masked);
                # the answer depends on the flags, so ask for that one (and for the block's own, for callers
                # that run a block's backward by hand)
                for fl in (0, d.flags):
                    ws_bytes = max(ws_bytes, B.sol_block_workspace_bytes(
                        B.BlockDesc(n, h, w, o.c_in, o.c_out, o.k, o.k, o.stride, o.pad, self.sol_dtype, fl),
                        B.SOL_PASS_BWD))
        self.ws = torch.empty((max(ws_bytes, 256),), dtype=torch.uint8, device=self.device)
        self._side: Optional[torch.cuda.Stream] = None
        self._ws_side: Optional[torch.Tensor] = None      # workspace of the second backward lane
        self._prepared: Optional[B.Sequence] = None       # the step as a prepared sequence of the library
        self.grads: Dict[int, Dict[str, torch.Tensor]] = {}
        self.dact: Dict[int, torch.Tensor] = {}
        self.target: Optional[torch.Tensor] = None
        if wl.train:
            self.target = upload(nchw_to_nhwc(wl.target), self.tdtype, self.device)
            for o in self.ops:
                if o.op != "conv":
                    continue
                p = self.params[o.layer]
                self.grads[o.layer] = {
                    "dW": torch.empty(p["W"].shape, dtype=torch.float32, device=self.device),
                    "dscale": torch.empty(o.c_out, dtype=torch.float32, device=self.device),
                    "dshift": torch.empty(o.c_out, dtype=torch.float32, device=self.device),
                }
            # one gradient buffer per activation that some backward call reads or writes densely
            for tid, (c, h, w) in self.shapes.items():
                if tid == 0 and not wl.need_input_grad:
                    continue
                self.dact[tid] = torch.empty((n, h, w, c), dtype=self.tdtype, device=self.device)
            self._plan_backward()

    def memory_report(self) -> Dict[str, int]:
        """Bytes of this schedule by kind of data (static: shapes and execution order only)."""
        plan = self.wl.memory_plan(workspace_bytes=int(self.ws.numel()))
        plan["activation_buffers_allocated"] = int(self.arena.numel()) if not self.retain else \
            sum(int(t.numel()) * t.element_size() for k, t in self.act.items() if k != 0)
        return plan

    # ------------------------------------------------------------------ forward
    def forward(self, stream=None) -> torch.Tensor:
        for o in self.ops:
            if o.op == "conv":
                p = self.params[o.layer]
                B.sol_block_fwd(self.desc[o.layer], self.act[o.inp], p["W"], p["scale"], p["shift"],
                                self.act[o.res] if o.res is not None else None, self.act[o.out],
                                self.ws, None, stream)
            else:
                c, h, w = self.shapes[o.inp]
                B.sol_maxpool_fwd(self.sol_dtype, self.act[o.inp], self.act[o.out], self.wl.n, h, w, c,
                                  o.k, o.stride, o.pad, stream)
        return self.act[self.ops[-1].out]

    # ---------------------------------------------------------------- loss grad
    def loss_grad(self, stream=None) -> torch.Tensor:
        last_op = self.ops[-1]
        y = self.act[last_op.out]
        B.sol_l1_loss_grad(self.sol_dtype, y, self.target, self.dact[last_op.out], y.numel(),
                           bool(getattr(last_op, "relu", False)), stream)
        return self.dact[last_op.out]

    # ----------------------------------------------------------------- backward
    def _plan_backward(self) -> None:
        """Resolve, once, the arguments of every backward call (reverse op order)."""
        for o in self.ops:
            if o.op != "conv":
                raise NotImplementedError("backward through the max-pool is not part of any training workload")
        producer = {o.out: o for o in self.ops}
        readers: Dict[int, List[ConvBlock]] = {}
        for o in self.ops:
            readers.setdefault(o.inp, []).append(o)
        # where the (masked) gradient of a tensor lives: its own buffer, or the buffer of the
        # tail block whose shortcut is the tensor's only use
        grad_of: Dict[int, torch.Tensor] = {self.ops[-1].out: self.dact[self.ops[-1].out]}
        shortcut: Dict[int, torch.Tensor] = {}     # shortcut gradient waiting to be added to a tensor
        written: Dict[int, bool] = {}
        calls: List[dict] = []
        for o in reversed(self.ops):
            if o.out not in grad_of:
                if o.out in shortcut and not readers.get(o.out):
                    if o.relu:
                        raise NotImplementedError("shortcut-only gradient into a block with its own ReLU")
                    grad_of[o.out] = shortcut.pop(o.out)
                else:
                    raise RuntimeError(f"no gradient reaches {o.name}")
            d = self.desc[o.layer]
            desc = B.BlockDesc(d.N, d.H, d.W, d.C_in, d.C_out, d.KH, d.KW, d.stride, d.pad, d.dtype,
                               d.flags & ~B.SOL_RELU)            # dy is stored already masked
            call = dict(op=o, desc=desc, dy=grad_of[o.out], dx=None, addend=None, dx_mask=None)
            if o.res is not None:
                if o.res in shortcut or written.get(o.res):
                    raise NotImplementedError("more than one shortcut into a tensor, or a late shortcut")
                shortcut[o.res] = grad_of[o.out]
            if not (o.inp == 0 and not self.wl.need_input_grad):
                call["dx"] = self.dact[o.inp]
                if written.get(o.inp):
                    call["addend"] = self.dact[o.inp]               # accumulate in place
                elif o.inp in shortcut:
                    call["addend"] = shortcut.pop(o.inp)
                written[o.inp] = True
                grad_of[o.inp] = self.dact[o.inp]
                is_last_writer = readers[o.inp][0] is o
                src = producer.get(o.inp)
                if is_last_writer and src is not None and src.relu:
                    call["dx_mask"] = self.act[o.inp]
            calls.append(call)
        self._bwd_calls = calls

    def backward(self, stream=None, lanes: int = 1) -> None:
        if lanes == 1:
            for c in self._bwd_calls:
                o = c["op"]
                p, g = self.params[o.layer], self.grads[o.layer]
                B.sol_block_bwd(c["desc"], c["dy"], self.act[o.inp], p["W"], None, c["dx"], g["dW"], g["dscale"],
                                g["dshift"], p["scale"], None, c["addend"], None, c["dx_mask"], self.ws, None, stream)
            return
        main = stream if stream is not None else torch.cuda.current_stream(self.device)
        if self._side is None:
            self._side = torch.cuda.Stream(device=self.device)       # default priority
            self._ws_side = torch.empty_like(self.ws)
        side = self._side
        for c in self._bwd_calls:
            o = c["op"]
            p, g = self.params[o.layer], self.grads[o.layer]
            # dy of this block is complete on the main lane here (loss kernel or the previous data gradient)
            side.wait_stream(main)
            B.sol_block_bwd(c["desc"], c["dy"], self.act[o.inp], p["W"], None, None, g["dW"], g["dscale"],
                            g["dshift"], p["scale"], None, None, None, None, self._ws_side, None, side)
            if c["dx"] is not None:
                B.sol_block_bwd(c["desc"], c["dy"], self.act[o.inp], p["W"], None, c["dx"], None, None, None,
                                p["scale"], None, c["addend"], None, c["dx_mask"], self.ws, None, main)
        main.wait_stream(side)

    def capture(self, lanes: int = 2) -> "torch.cuda.CUDAGraph":
        """Record one step into a HIP graph; ``graph.replay()`` then runs it without per-launch host
        work, the weight branches of the backward pass as parallel branches of the graph (lanes=2).
        The library itself allocates nothing and enqueues only on the stream it is given, so a step is
        capturable as it is (no memsets are recorded)."""
        warm = torch.cuda.Stream(device=self.device)
        warm.wait_stream(torch.cuda.current_stream(self.device))
        with torch.cuda.stream(warm):
            self.step(lanes=lanes)           # first use of every kernel happens outside the capture
        torch.cuda.current_stream(self.device).wait_stream(warm)
        torch.cuda.synchronize(self.device)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            self.step(lanes=lanes)
        self.graph = graph
        return graph

    def prepared(self) -> "B.Sequence":
        """The whole step (forward, loss gradient, one-lane backward) recorded once as a prepared sequence of
        the library: running it issues every launch of the step from native code, in the order ``step`` uses."""
        if self._prepared is None:
            q = B.Sequence()
            for o in self.ops:
                if o.op == "conv":
                    p = self.params[o.layer]
                    q.add_fwd(self.desc[o.layer], self.act[o.inp], p["W"], p["scale"], p["shift"],
                              self.act[o.res] if o.res is not None else None, self.act[o.out], self.ws, None, o.layer)
                else:
                    c, h, w = self.shapes[o.inp]
                    q.add_maxpool(self.sol_dtype, self.act[o.inp], self.act[o.out], self.wl.n, h, w, c, o.k, o.stride,
                                  o.pad, -1)
            self._prepared_fwd = len(q)
            if self.wl.train:
                last_op = self.ops[-1]
                y = self.act[last_op.out]
                q.add_l1_loss_grad(self.sol_dtype, y, self.target, self.dact[last_op.out], y.numel(),
                                   bool(getattr(last_op, "relu", False)), -2)
                for c in self._bwd_calls:
                    o = c["op"]
                    p, g = self.params[o.layer], self.grads[o.layer]
                    q.add_bwd(c["desc"], c["dy"], self.act[o.inp], p["W"], None, c["dx"], g["dW"], g["dscale"],
                              g["dshift"], p["scale"], None, c["addend"], None, c["dx_mask"], self.ws, None, o.layer)
            self._prepared = q
        return self._prepared

    def step_prepared(self, stream=None) -> None:
        """``step(lanes=1)`` through the prepared sequence: one library call for the whole step."""
        self.prepared().run(stream=stream if stream is not None else torch.cuda.current_stream(self.device))

    def step(self, stream=None, lanes: int = 1) -> None:
        """One pass of the whole path: forward, and for training the loss gradient and backward."""
        if stream is None:
            stream = torch.cuda.current_stream(self.device)     # looked up once per step, not once per call
        self.forward(stream)
        if self.wl.train:
            self.loss_grad(stream)
            self.backward(stream, lanes)
