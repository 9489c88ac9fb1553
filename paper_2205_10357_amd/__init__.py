"""Fused Conv2d + folded-BatchNorm affine (+ residual) (+ ReLU) blocks, forward and
backward, as hand-written gfx950 kernels behind a small C-ABI library.

The paper replaces the model forward pass (step 1) and backward pass (step 3) of the
training loop with compiled, layer-merged code (section "SOL principle"); for
ResNet-50-style networks those passes are these fused blocks.

Sub-modules
  workloads : seeded synthetic inputs and the ResNet-50 layer geometry (numpy only)
  binding   : ctypes binding to ``libsol_block.so`` (same names as the C-ABI)
  build     : hipcc driver that builds the library in-tree
  runner    : static layer-list sequencing for multi-block workloads

Nothing is imported eagerly, so the input generators can be used without the
compiled library being present.
"""

__all__ = ["workloads", "binding", "build", "runner"]
