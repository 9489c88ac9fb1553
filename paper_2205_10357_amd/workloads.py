"""Seeded synthetic inputs and layer geometry for the fused-block workloads.

This module holds no arithmetic of the method itself: it only draws random tensors,
snaps them to the storage grid of the dtype they will be stored in, and describes
which layers a workload consists of.  Both the GPU path and the CPU checker are fed
from here so that they see bit-identical inputs; neither of them is imported here.

The paper's workload is the TorchVision ResNet-50 (section "SOL Benefits",
performance paragraph and the caption of its figure 3); no dataset or trained weight
is needed for throughput or parity of dense convolutions, so every tensor is a seeded
draw from a simple distribution with the network's shapes.

Conventions
  * tensors are generated in *logical* order: activations ``[N, C, H, W]``,
    weights ``[C_out, C_in, KH, KW]``, float32;
  * one independent ``numpy.random.Generator(PCG64(seed))`` stream per tensor,
    ``seed = 1000*workload + 10*layer + kind`` with kind 0 = weight, 1 = scale,
    2 = shift, 3 = input, 4 = target (the single weight of workload 1 uses seed 0);
  * weights are Kaiming-normal with ``std = sqrt(2 / (C_in*KH*KW))``;
  * folded-BN parameters: ``scale ~ U(0.5, 1.5)``, ``shift ~ N(0, 0.1**2)``.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

import numpy as np

KIND_W, KIND_SCALE, KIND_SHIFT, KIND_X, KIND_T = 0, 1, 2, 3, 4


# ----------------------------------------------------------------------------- draws
def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(int(seed)))


def seed_for(workload: int, layer: int, kind: int) -> int:
    if workload == 1 and layer == 0 and kind == KIND_W:
        return 0
    return 1000 * workload + 10 * layer + kind


def draw_uniform01(seed: int, shape) -> np.ndarray:
    return _rng(seed).random(size=shape, dtype=np.float32)


def draw_normal(seed: int, shape, std: float = 1.0) -> np.ndarray:
    a = _rng(seed).standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    return a


def draw_weight(seed: int, c_out: int, c_in: int, kh: int, kw: int) -> np.ndarray:
    std = float(np.sqrt(2.0 / (c_in * kh * kw)))
    return draw_normal(seed, (c_out, c_in, kh, kw), std)


def draw_scale(seed: int, c: int) -> np.ndarray:
    return (np.float32(0.5) + _rng(seed).random(size=(c,), dtype=np.float32)).astype(np.float32)


def draw_shift(seed: int, c: int) -> np.ndarray:
    return draw_normal(seed, (c,), 0.1)


def snap_to_bf16(a: np.ndarray) -> np.ndarray:
    """Return float32 values that are exactly representable in bfloat16.

    Storage-grid snapping of an *input* (round to nearest, ties to even on the upper
    16 bits of the IEEE-754 binary32 pattern).  Finite inputs only.
    """
    a = np.ascontiguousarray(a, dtype=np.float32)
    bits = a.view(np.uint32).astype(np.uint64)
    lsb = (bits >> np.uint64(16)) & np.uint64(1)
    bits = (bits + np.uint64(0x7FFF) + lsb) & np.uint64(0xFFFF0000)
    return bits.astype(np.uint32).view(np.float32).reshape(a.shape)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """Upper 16 bits of float32 values that already lie on the bfloat16 grid."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    bits = a.view(np.uint32)
    if np.any(bits & np.uint32(0xFFFF)):
        raise ValueError("values are not on the bfloat16 grid")
    return (bits >> np.uint32(16)).astype(np.uint16).reshape(a.shape)


# -------------------------------------------------------------------------- geometry
@dataclass(frozen=True)
class ConvBlock:
    """One fused block: conv (no bias) -> per-channel affine -> (+ residual) -> (ReLU)."""

    name: str
    c_in: int
    c_out: int
    k: int
    stride: int
    pad: int
    relu: bool
    inp: int                     # tensor id of the input activation
    out: int                     # tensor id of the output activation
    res: Optional[int] = None    # tensor id added before the ReLU, if any
    layer: int = 0               # running conv index inside the workload (for seeds)
    op: str = "conv"


@dataclass(frozen=True)
class MaxPool:
    """3x3 / stride 2 / pad 1 max-pool (glue between the stem and stage 1)."""

    name: str
    inp: int
    out: int
    k: int = 3
    stride: int = 2
    pad: int = 1
    op: str = "maxpool"


def out_size(h: int, k: int, stride: int, pad: int) -> int:
    return (h + 2 * pad - k) // stride + 1


def conv_flops(n: int, h: int, w: int, blk: ConvBlock) -> int:
    """2*M*K*C_out for one pass, padding taps counted as dense."""
    ho, wo = out_size(h, blk.k, blk.stride, blk.pad), out_size(w, blk.k, blk.stride, blk.pad)
    return 2 * n * ho * wo * blk.c_out * blk.c_in * blk.k * blk.k


def bottleneck(ops: list, name: str, tin: int, next_tid: int, layer0: int, c_in: int, width: int,
               stride: int, project: bool):
    """Append conv1(1x1) -> conv2(3x3, stride) -> [proj 1x1, stride] -> conv3(1x1)+res+ReLU.

    Returns (output tensor id, next free tensor id, next layer index).
    """
    t1, t2, tout = next_tid, next_tid + 1, next_tid + 2
    next_tid += 3
    layer = layer0
    ops.append(ConvBlock(f"{name}.conv1", c_in, width, 1, 1, 0, True, tin, t1, None, layer)); layer += 1
    ops.append(ConvBlock(f"{name}.conv2", width, width, 3, stride, 1, True, t1, t2, None, layer)); layer += 1
    res = tin
    if project:
        tp = next_tid
        next_tid += 1
        ops.append(ConvBlock(f"{name}.proj", c_in, 4 * width, 1, stride, 0, False, tin, tp, None, layer)); layer += 1
        res = tp
    ops.append(ConvBlock(f"{name}.conv3", width, 4 * width, 1, 1, 0, True, t2, tout, res, layer)); layer += 1
    return tout, next_tid, layer


def resnet50_ops() -> List[object]:
    """All 53 convolution blocks of a ResNet-50-shaped stack plus the stem max-pool.

    Stride 2 sits on the 3x3 of the first bottleneck of stages 2-4; the first bottleneck
    of every stage has a 1x1 projection (affine, no ReLU) feeding conv3's residual.
    Tensor 0 is the network input.
    """
    ops: List[object] = []
    ops.append(ConvBlock("stem", 3, 64, 7, 2, 3, True, 0, 1, None, 0))
    ops.append(MaxPool("pool", 1, 2))
    tin, next_tid, layer = 2, 3, 1
    c_in = 64
    for si, (nblk, width) in enumerate(zip((3, 4, 6, 3), (64, 128, 256, 512))):
        for b in range(nblk):
            stride = 2 if (b == 0 and si > 0) else 1
            tin, next_tid, layer = bottleneck(ops, f"s{si + 1}.b{b}", tin, next_tid, layer, c_in, width,
                                              stride, project=(b == 0))
            c_in = 4 * width
    assert layer == 53
    return ops


def stage2_ops(faithful: bool = True) -> List[object]:
    """Stage 2 of the ResNet-50-shaped stack: 4 bottlenecks, widths 128/512.

    faithful: block 0 takes 256 channels at 56x56, has the stride-2 3x3 and a stride-2
    projection; blocks 1-3 are identity bottlenecks at 28x28 (13 convs).
    not faithful ("uniform"): 4 identity bottlenecks on a 512-channel 28x28 input (12 convs).
    """
    ops: List[object] = []
    tin, next_tid, layer = 0, 1, 0
    c_in = 256 if faithful else 512
    for b in range(4):
        first = faithful and b == 0
        tin, next_tid, layer = bottleneck(ops, f"s2.b{b}", tin, next_tid, layer, c_in, 128,
                                          2 if first else 1, project=first)
        c_in = 512
    return ops


def bottleneck14_ops() -> List[object]:
    """One identity bottleneck: 1x1 1024->256, 3x3 256->256, 1x1 256->1024 + input + ReLU."""
    ops: List[object] = []
    bottleneck(ops, "b", 0, 1, 0, 1024, 256, 1, project=False)
    return ops


# ------------------------------------------------------------------------- workloads
@dataclass
class Workload:
    """A list of ops plus everything needed to run it: input, parameters, loss target."""

    ident: int                      # 1..5, the position in the list of configurations
    name: str
    dtype: str                      # "f32" or "bf16": storage type of activations / weights
    n: int
    h: int
    w: int
    c: int
    ops: List[object]
    x: np.ndarray                   # [N, C, H, W] float32 (on the storage grid of `dtype`)
    params: Dict[int, Dict[str, np.ndarray]] = field(default_factory=dict)   # layer -> W/scale/shift
    target: Optional[np.ndarray] = None      # [N, C_out, Ho, Wo] float32, for the L1 loss
    need_input_grad: bool = True
    train: bool = True

    def conv_blocks(self) -> List[ConvBlock]:
        return [o for o in self.ops if o.op == "conv"]

    def tensor_shapes(self) -> Dict[int, tuple]:
        """tensor id -> (C, H, W) for every tensor of the op list."""
        shp = {0: (self.c, self.h, self.w)}
        for o in self.ops:
            c, h, w = shp[o.inp]
            ho, wo = out_size(h, o.k, o.stride, o.pad), out_size(w, o.k, o.stride, o.pad)
            shp[o.out] = ((o.c_out if o.op == "conv" else c), ho, wo)
        return shp

    def flops_forward(self) -> int:
        shp = self.tensor_shapes()
        return sum(conv_flops(self.n, shp[b.inp][1], shp[b.inp][2], b) for b in self.conv_blocks())

    def memory_plan(self, workspace_bytes: int = 0) -> Dict[str, int]:
        """Bytes of the static schedule by kind of data, known before the first run (the paper's section on
        memory consumption estimates the peak the same way, from the execution order and the tensor sizes).

        Training keeps every activation between the passes (the backward pass reads the block inputs and the
        masks) and one gradient per activation; inference needs a tensor only until its last reader has run, so
        its activation peak is the largest set of tensors alive at one op of the schedule (a residual keeps the
        block input alive across the three convolutions)."""
        es = 2 if self.dtype == "bf16" else 4
        shp = self.tensor_shapes()
        size = {t: self.n * c * h * w * es for t, (c, h, w) in shp.items()}
        plan = {"input": size[0], "parameters": 0, "outputs": size[self.ops[-1].out]}
        for b in self.conv_blocks():
            c_in = shp[b.inp][0]
            plan["parameters"] += b.c_out * b.k * b.k * c_in * es + 2 * b.c_out * 4
        inter = [o.out for o in self.ops[:-1]]
        plan["intermediates_all_kept"] = sum(size[t] for t in inter)
        last_use = {0: 0}
        for i, o in enumerate(self.ops):
            last_use[o.inp] = i
            if getattr(o, "res", None) is not None:
                last_use[o.res] = i
        peak = 0
        for i, o in enumerate(self.ops):           # alive while op i runs: its output and everything still to be read
            alive = size[o.out] + sum(size[t] for t, lu in last_use.items() if lu >= i and t != o.out and
                                      (t == 0 or any(oo.out == t for oo in self.ops[:i])))
            peak = max(peak, alive)
        plan["inference_peak_activations"] = peak      # includes the input while it is alive
        if self.train:
            plan["target"] = size[self.ops[-1].out]
            plan["parameter_gradients"] = sum(b.c_out * b.k * b.k * shp[b.inp][0] * 4 + 2 * b.c_out * 4
                                              for b in self.conv_blocks())
            plan["activation_gradients"] = sum(size[t] for t in shp if t != 0 or self.need_input_grad)
        plan["workspace"] = int(workspace_bytes)
        keep = ("input", "parameters", "outputs", "workspace")
        if self.train:
            plan["total_training"] = sum(plan[k] for k in keep) + plan["intermediates_all_kept"] + plan["target"] + \
                plan["parameter_gradients"] + plan["activation_gradients"]
        else:
            plan["inference_arena"] = self.plan_inference_arena()[1]   # what the planned buffers really take (first fit)
            plan["total_inference_all_kept"] = sum(plan[k] for k in keep) + plan["intermediates_all_kept"]
            plan["total_inference_minimum"] = plan["parameters"] + plan["workspace"] + plan["inference_peak_activations"]
        return plan

    def plan_inference_arena(self, align: int = 256) -> Tuple[Dict[int, int], int]:
        """Byte offsets of the activations of an inference run inside one arena, and the arena's size.

        The inference version of the schedule retains nothing for a backward pass (the paper generates the
        inference and the training version of a network separately): a tensor occupies its bytes from the op
        that writes it to its last reader, both included, so an op never writes over what it reads.  Placement
        is the usual offline heuristic for such interval problems: largest tensor first, each at the lowest
        offset where it meets no already placed tensor whose lifetime overlaps its own.  The network input
        (tensor 0) is the caller's buffer and is not part of the arena; the final output lives to the end."""
        es = 2 if self.dtype == "bf16" else 4
        shp = self.tensor_shapes()
        size = {t: -(-(self.n * c * h * w * es) // align) * align for t, (c, h, w) in shp.items() if t != 0}
        born = {o.out: i for i, o in enumerate(self.ops)}
        dies = dict(born)                                    # an output nobody reads dies where it is born
        for i, o in enumerate(self.ops):
            for t in (o.inp, getattr(o, "res", None)):
                if t is not None and t != 0:
                    dies[t] = i
        dies[self.ops[-1].out] = len(self.ops)
        offset: Dict[int, int] = {}
        top = 0
        for t in sorted(size, key=lambda t: (-size[t], born[t])):
            busy = sorted((offset[u], offset[u] + size[u]) for u in offset
                          if born[u] <= dies[t] and born[t] <= dies[u])
            at = 0
            for lo, hi in busy:
                if at + size[t] <= lo:
                    break
                at = max(at, hi)
            offset[t] = at
            top = max(top, at + size[t])
        return offset, top

    def flops_step(self) -> int:
        """Forward only for inference; x3 for training, x2 for blocks whose dx is skipped."""
        if not self.train:
            return self.flops_forward()
        shp = self.tensor_shapes()
        total = 0
        for b in self.conv_blocks():
            f = conv_flops(self.n, shp[b.inp][1], shp[b.inp][2], b)
            skip_dx = (b.inp == 0 and not self.need_input_grad)
            total += f * (2 if skip_dx else 3)
        return total


def _fill_params(wl: Workload, snap: bool) -> None:
    for b in wl.conv_blocks():
        w = draw_weight(seed_for(wl.ident, b.layer, KIND_W), b.c_out, b.c_in, b.k, b.k)
        if snap:
            w = snap_to_bf16(w)
        wl.params[b.layer] = {
            "W": w,
            "scale": draw_scale(seed_for(wl.ident, b.layer, KIND_SCALE), b.c_out),
            "shift": draw_shift(seed_for(wl.ident, b.layer, KIND_SHIFT), b.c_out),
        }


def _make(ident, name, dtype, n, c, h, w, ops, x_dist, train, need_input_grad=True) -> Workload:
    snap = dtype == "bf16"
    seed_x = seed_for(ident, 0, KIND_X)
    x = draw_normal(seed_x, (n, c, h, w)) if x_dist == "normal" else draw_uniform01(seed_x, (n, c, h, w))
    if snap:
        x = snap_to_bf16(x)
    wl = Workload(ident, name, dtype, n, h, w, c, ops, x, train=train, need_input_grad=need_input_grad)
    _fill_params(wl, snap)
    if train:
        co, ho, wo = wl.tensor_shapes()[ops[-1].out]
        t = draw_uniform01(seed_for(ident, 0, KIND_T), (n, co, ho, wo))
        wl.target = snap_to_bf16(t) if snap else t
    return wl


def single_block_f32(n: int = 1, c: int = 16, hw: int = 16) -> Workload:
    """Workload 1: one 3x3 / s1 / p1 block in fp32, C_in = C_out = 16, 16x16, N = 1."""
    ops = [ConvBlock("block", c, c, 3, 1, 1, True, 0, 1, None, 0)]
    return _make(1, "single_block_f32", "f32", n, c, hw, hw, ops, "uniform", True)


def stem_bf16(n: int = 32, hw: int = 224) -> Workload:
    """Workload 2: 7x7 / s2 / p3 stem 3->64 + affine + ReLU, bf16, no gradient to the image."""
    ops = [ConvBlock("stem", 3, 64, 7, 2, 3, True, 0, 1, None, 0)]
    return _make(2, "stem_bf16", "bf16", n, 3, hw, hw, ops, "normal", True, need_input_grad=False)


def bottleneck14_bf16(n: int = 64, hw: int = 14) -> Workload:
    """Workload 3: identity bottleneck 1024/256 at 14x14, bf16, forward + full backward."""
    return _make(3, "bottleneck14_bf16", "bf16", n, 1024, hw, hw, bottleneck14_ops(), "normal", True)


def resnet50_infer_bf16(n: int = 128, hw: int = 224) -> Workload:
    """Workload 4: all 53 conv blocks (+ max-pool), inference, bf16, x ~ U[0,1)."""
    return _make(4, "resnet50_infer_bf16", "bf16", n, 3, hw, hw, resnet50_ops(), "uniform", False)


def stage2_train_bf16(n: int = 128, faithful: bool = True, hw: Optional[int] = None) -> Workload:
    """Workload 5: training step over stage 2 (4 bottlenecks, 128/512 channels)."""
    if hw is None:
        hw = 56 if faithful else 28
    c = 256 if faithful else 512
    name = "stage2_train_bf16" + ("" if faithful else "_uniform")
    return _make(5, name, "bf16", n, c, hw, hw, stage2_ops(faithful), "uniform", True)


WORKLOADS = {
    1: single_block_f32,
    2: stem_bf16,
    3: bottleneck14_bf16,
    4: resnet50_infer_bf16,
    5: stage2_train_bf16,
}
