"""GPU parity: the HIP path, called through the C-ABI, against the CPU checker on the same
seeded inputs.  Tolerances: max relative L2 error 1e-5 (fp32) / 1e-2 (bf16) per output tensor,
ReLU mask and masked gradients bit-exact."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from oracle import oracle as orc                              # noqa: E402
from paper_2205_10357_amd import binding as B                 # noqa: E402
from paper_2205_10357_amd import workloads as wl              # noqa: E402
from tests import parity_util as pu                           # noqa: E402


def show(name, errs):
    print(f"[parity] {name}: " + " ".join(f"{k}={v:.3g}" if isinstance(v, float) else f"{k}={v}" for k, v in errs.items()),
          flush=True)


# ------------------------------------------------------------------ workload 1 (fp32)
def test_single_block_fp32_matches_checker():
    w = wl.single_block_f32()
    p = w.params[0]
    case = dict(d=orc.Desc(1, 16, 16, 16, 16, 3, 3, 1, 1, True), bf16=False, x=w.x, w=p["W"], scale=p["scale"],
                shift=p["shift"], res=None, t=w.target)
    got = pu.gpu_block(case)
    errs = pu.check_block(case, got)
    show("single_block_f32", errs)
    assert errs["mask_band"] == 0        # no pre-activation of this seed sits inside the rounding band


@pytest.mark.parametrize("shape", [
    dict(N=2, H=9, W=7, C_in=5, C_out=6, K=3, stride=1, pad=1, res=True),
    dict(N=1, H=11, W=10, C_in=3, C_out=4, K=7, stride=2, pad=3),
    dict(N=2, H=8, W=8, C_in=8, C_out=4, K=1, stride=2, pad=0, relu=False),
])
def test_fp32_other_shapes(shape):
    case = pu.make_case(31, bf16=False, **shape)
    got = pu.gpu_block(case, want_dres=True)
    show(f"f32 {shape}", pu.check_block(case, got))


# --------------------------------------------------- bf16: the distinct ResNet-50 layer shapes
RESNET_SHAPES = [  # (name, C_in, C_out, H, k, stride, pad, residual)
    ("stem", 3, 64, 224, 7, 2, 3, False),
    ("s1.conv1a", 64, 64, 56, 1, 1, 0, False),
    ("s1.conv2", 64, 64, 56, 3, 1, 1, False),
    ("s1.proj", 64, 256, 56, 1, 1, 0, False),
    ("s1.conv3", 64, 256, 56, 1, 1, 0, True),
    ("s1.conv1b", 256, 64, 56, 1, 1, 0, False),
    ("s2.conv1a", 256, 128, 56, 1, 1, 0, False),
    ("s2.conv2a", 128, 128, 56, 3, 2, 1, False),
    ("s2.proj", 256, 512, 56, 1, 2, 0, False),
    ("s2.conv3", 128, 512, 28, 1, 1, 0, True),
    ("s2.conv1b", 512, 128, 28, 1, 1, 0, False),
    ("s2.conv2b", 128, 128, 28, 3, 1, 1, False),
    ("s3.conv1a", 512, 256, 28, 1, 1, 0, False),
    ("s3.conv2a", 256, 256, 28, 3, 2, 1, False),
    ("s3.proj", 512, 1024, 28, 1, 2, 0, False),
    ("s3.conv3", 256, 1024, 14, 1, 1, 0, True),
    ("s3.conv1b", 1024, 256, 14, 1, 1, 0, False),
    ("s3.conv2b", 256, 256, 14, 3, 1, 1, False),
    ("s4.conv1a", 1024, 512, 14, 1, 1, 0, False),
    ("s4.conv2a", 512, 512, 14, 3, 2, 1, False),
    ("s4.proj", 1024, 2048, 14, 1, 2, 0, False),
    ("s4.conv3", 512, 2048, 7, 1, 1, 0, True),
    ("s4.conv1b", 2048, 512, 7, 1, 1, 0, False),
    ("s4.conv2b", 512, 512, 7, 3, 1, 1, False),
]


@pytest.mark.parametrize("spec", RESNET_SHAPES, ids=[s[0] for s in RESNET_SHAPES])
def test_bf16_resnet50_layer_shapes(spec):
    name, c_in, c_out, h, k, stride, pad, res = spec
    n = 1 if h >= 56 else (2 if h >= 14 else 5)          # several pixel tiles and a ragged last one
    relu = "proj" not in name
    case = pu.make_case(100 + len(name), n, h, h, c_in, c_out, k, stride, pad, relu=relu, res=res)
    got = pu.gpu_block(case, need_dx=(name != "stem"))
    show(name, pu.check_block(case, got, need_dx=(name != "stem")))


@pytest.mark.parametrize("spec", RESNET_SHAPES[1:], ids=[s[0] for s in RESNET_SHAPES[1:]])
def test_bf16_resnet50_layer_shapes_layer_merged_backward(spec):
    """The same shapes the way the sequencer runs them backward: the gradient arrives already masked, the
    block is called without SOL_RELU and without y, a shortcut gradient is added and the stored dx is masked
    by the block input.  With channel counts that are multiples of 64 this is the pipelined data-gradient
    and weight-gradient path (the call above, which masks dy itself, takes the general kernels)."""
    name, c_in, c_out, h, k, stride, pad, res = spec
    n = 1 if h >= 56 else (2 if h >= 14 else 5)
    relu = "proj" not in name
    case = pu.make_case(200 + len(name), n, h, h, c_in, c_out, k, stride, pad, relu=relu, res=res)
    r = np.random.default_rng(201)
    dxm = wl.snap_to_bf16(np.maximum(r.standard_normal(case["x"].shape), 0).astype(np.float32))
    ad = wl.snap_to_bf16(r.standard_normal(case["x"].shape).astype(np.float32))
    got = pu.gpu_block(case, addend=ad, dx_mask=dxm, premasked=True)
    show(name + " merged", pu.check_block(case, got, addend=ad, dx_mask=dxm, premasked=True))


PLAN_SHAPES = {
    "3x3_s1_res_ragged": dict(N=2, H=19, W=17, C_in=64, C_out=136, K=3, stride=1, pad=1, res=True),
    "3x3_s2": dict(N=2, H=15, W=13, C_in=64, C_out=64, K=3, stride=2, pad=1),
    "1x1_s2_long_reduction": dict(N=2, H=14, W=14, C_in=512, C_out=256, K=1, stride=2, pad=0, relu=False),
    "1x1_s1_many_rows": dict(N=3, H=14, W=14, C_in=128, C_out=192, K=1, stride=1, pad=0),
}
FAST_PLANS = [(t, s) for t in (0, 1, 2, 3) for s in (2, 3, 4) if not (t == 3 and s == 4)]


@pytest.mark.parametrize("shape", list(PLAN_SHAPES), ids=list(PLAN_SHAPES))
def test_every_installable_plan_matches_checker(shape):
    """Every (tile, ring depth) a caller can install for the pipelined forward / data-gradient kernel and every
    ring depth (and a few split counts) of the pipelined weight-gradient kernel, each compared with the CPU
    checker -- not with the default plan's result."""
    case = pu.make_case(81, **PLAN_SHAPES[shape])
    d = case["d"]
    desc = B.BlockDesc(d.N, d.H, d.W, d.C_in, d.C_out, d.KH, d.KW, d.stride, d.pad, B.SOL_BF16, 0)
    r = np.random.default_rng(82)
    dxm = wl.snap_to_bf16(np.maximum(r.standard_normal(case["x"].shape), 0).astype(np.float32))
    ad = wl.snap_to_bf16(r.standard_normal(case["x"].shape).astype(np.float32))
    wgrad_plans = [(2, 0), (3, 1), (4, 3), (2, 5), (3, 0), (4, 0)]
    try:
        for i, (tile, stages) in enumerate(FAST_PLANS):
            ws, wsplit = wgrad_plans[i % len(wgrad_plans)]
            B.sol_block_set_plan(desc, B.SOL_PLAN_FWD, (tile, stages, 0))
            B.sol_block_set_plan(desc, B.SOL_PLAN_DGRAD, (tile, stages, 0))
            B.sol_block_set_plan(desc, B.SOL_PLAN_WGRAD, (-1, ws, wsplit))
            assert B.sol_block_get_plan(desc, B.SOL_PLAN_DGRAD) == (tile, stages, 0)
            print(f"[plan] {shape}: tile {tile} stages {stages}; wgrad stages {ws} splits {wsplit}", flush=True)
            got = pu.gpu_block(case, addend=ad, dx_mask=dxm, premasked=True)
            errs = pu.check_block(case, got, addend=ad, dx_mask=dxm, premasked=True)
        show(f"plans {shape} (last)", errs)
    finally:
        B.sol_clear_plans()


PANEL_SHAPES = {
    # forward runs the panel kernel (64 .. 256 input channels, output channels a multiple of 128) ...
    "k64_to_384_res": dict(N=2, H=9, W=11, C_in=64, C_out=384, K=1, stride=1, pad=0, res=True),
    "k192_to_512_ragged": dict(N=3, H=7, W=9, C_in=192, C_out=512, K=1, stride=1, pad=0, relu=False),
    "k256_to_1024_res": dict(N=1, H=14, W=14, C_in=256, C_out=1024, K=1, stride=1, pad=0, res=True),
    # ... the data gradient does where the roles are swapped (it gathers dy: C_out channels, writes C_in) ...
    "dgrad_k128_to_256": dict(N=2, H=10, W=13, C_in=256, C_out=128, K=1, stride=1, pad=0),
    "dgrad_k256_to_512": dict(N=1, H=12, W=11, C_in=512, C_out=256, K=1, stride=1, pad=0, relu=False),
    # ... and both do here
    "both_256": dict(N=2, H=14, W=14, C_in=256, C_out=256, K=1, stride=1, pad=0, res=True),
}


@pytest.mark.parametrize("tiles", [0, 1, 2, 3, 8], ids=lambda t: f"tiles{t}")
@pytest.mark.parametrize("shape", list(PANEL_SHAPES), ids=list(PANEL_SHAPES))
def test_panel_kernel_matches_checker(shape, tiles, sol_env):
    """The kernel that keeps a pixel panel in LDS and walks over several channel tiles (plan tile 4), forced for the
    forward and the data-gradient GEMM, with every number of tiles per workgroup from one (no streaming across tiles)
    to more than the layer has (all in one workgroup): forward with and without residual, data gradient with an
    addend and an output mask.  Compared with the CPU checker."""
    if tiles:
        sol_env("SOL_PANEL_TILES", tiles)
    case = pu.make_case(91, **PANEL_SHAPES[shape])
    d = case["d"]
    desc = B.BlockDesc(d.N, d.H, d.W, d.C_in, d.C_out, d.KH, d.KW, d.stride, d.pad, B.SOL_BF16, 0)
    r = np.random.default_rng(92)
    dxm = wl.snap_to_bf16(np.maximum(r.standard_normal(case["x"].shape), 0).astype(np.float32))
    ad = wl.snap_to_bf16(r.standard_normal(case["x"].shape).astype(np.float32))
    try:
        B.sol_block_set_plan(desc, B.SOL_PLAN_FWD, (4, 0, 0))
        B.sol_block_set_plan(desc, B.SOL_PLAN_DGRAD, (4, 0, 0))
        print(f"[panel] {shape}: tiles per workgroup {tiles or 'auto'}", flush=True)
        got = pu.gpu_block(case, addend=ad, dx_mask=dxm, premasked=True)
        errs = pu.check_block(case, got, addend=ad, dx_mask=dxm, premasked=True)
        show(f"panel {shape} tiles {tiles}", errs)
        # the same launches by the one-tile-per-workgroup kernel: identical bit for bit (same order of accumulation)
        B.sol_block_set_plan(desc, B.SOL_PLAN_FWD, (0, 4, 0))
        B.sol_block_set_plan(desc, B.SOL_PLAN_DGRAD, (0, 4, 0))
        ref = pu.gpu_block(case, addend=ad, dx_mask=dxm, premasked=True)
        for key in ("y", "dx"):
            a, b = (np.ascontiguousarray(v[key], dtype=np.float32).view(np.uint32) for v in (got, ref))
            assert np.array_equal(a, b), f"{key}: {int((a != b).sum())} elements differ from the one-tile kernel"
    finally:
        B.sol_clear_plans()


@pytest.mark.parametrize("shape", [
    dict(N=1, H=1, W=1, C_in=8, C_out=8, K=3, stride=1, pad=1),               # single pixel, only the centre tap
    dict(N=3, H=5, W=7, C_in=16, C_out=24, K=3, stride=1, pad=1, res=True),   # fewer rows than one tile
    dict(N=1, H=13, W=11, C_in=12, C_out=20, K=3, stride=1, pad=1),           # channels not a multiple of 8
    dict(N=2, H=9, W=11, C_in=24, C_out=16, K=3, stride=2, pad=1),            # odd sizes under stride 2
    dict(N=2, H=7, W=9, C_in=16, C_out=40, K=1, stride=2, pad=0, relu=False), # 1x1/s2: 3 of 4 pixel classes see no tap
    dict(N=2, H=14, W=14, C_in=64, C_out=512, K=1, stride=2, pad=0, relu=False),  # same, long reduction (deep copy ring)
    dict(N=1, H=12, W=12, C_in=3, C_out=8, K=7, stride=2, pad=3),             # stem-like with a data gradient
    dict(N=2, H=30, W=530, C_in=3, C_out=64, K=7, stride=2, pad=3),           # few-channel kernel: 3 row segments, ragged
    dict(N=3, H=9, W=11, C_in=4, C_out=64, K=3, stride=2, pad=1, relu=False), # few-channel kernel, 3x3, 4 channels
    dict(N=1, H=16, W=16, C_in=1, C_out=64, K=5, stride=2, pad=2),            # few-channel kernel, 1 channel
    dict(N=1, H=33, W=31, C_in=64, C_out=136, K=3, stride=1, pad=1),          # ragged in pixels and channels
    dict(N=2, H=6, W=6, C_in=8, C_out=8, K=5, stride=1, pad=2),               # 5x5
    dict(N=1, H=8, W=8, C_in=16, C_out=16, K=3, stride=1, pad=0),             # no padding
    dict(N=2, H=9, W=11, C_in=64, C_out=72, K=5, stride=1, pad=2, res=True),  # 25 taps on the pipelined kernel (tap mask, 5 tap rows)
    dict(N=2, H=10, W=9, C_in=64, C_out=64, K=5, stride=2, pad=2),            # same, strided: four pixel classes with 9 / 6 / 6 / 4 taps
    dict(N=1, H=6, W=7, C_in=128, C_out=64, K=3, stride=1, pad=2),            # padding 2 under a 3x3: border pixels lose two tap rows and two tap columns
])
def test_bf16_edge_shapes(shape):
    case = pu.make_case(7, **shape)
    got = pu.gpu_block(case, want_dres=True)
    show(f"edge {shape}", pu.check_block(case, got))


def _random_pipelined_shapes(count, seed):
    """Seeded draw of layer shapes the pipelined kernels take (input channels a multiple of 64, output channels a
    multiple of 8): filter 1 / 3 / 5, stride 1 / 2, padding from none to one more than 'same', ragged pixel counts."""
    r = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        k = int(r.choice([1, 3, 3, 5]))
        stride = int(r.choice([1, 1, 2]))
        pad = int(r.integers(0, k // 2 + 2)) if k > 1 else 0
        c_in = int(r.choice([64, 128, 192, 256]))
        c_out = int(r.choice([8, 24, 64, 72, 128, 136, 256, 384]))
        n, h, w = int(r.integers(1, 4)), int(r.integers(5, 19)), int(r.integers(5, 19))
        if h + 2 * pad < k or w + 2 * pad < k:
            continue
        out.append(dict(N=n, H=h, W=w, C_in=c_in, C_out=c_out, K=k, stride=stride, pad=pad,
                        relu=bool(r.integers(0, 2)), res=bool(r.integers(0, 2))))
    return out


RANDOM_SHAPES = _random_pipelined_shapes(24, 20250)


@pytest.mark.parametrize("idx", range(len(RANDOM_SHAPES)), ids=lambda i: "k{K}s{stride}p{pad}_{C_in}to{C_out}_{N}x{H}x{W}".format(**RANDOM_SHAPES[i]))
def test_random_layer_shapes_on_the_pipelined_kernels(idx):
    """Forward, data gradient (with an addend and an output mask) and weight gradient of seeded random layer shapes,
    gradient masked upstream so that every GEMM runs on the pipelined kernels; compared with the CPU checker."""
    shape = RANDOM_SHAPES[idx]
    case = pu.make_case(300 + idx, **shape)
    r = np.random.default_rng(400 + idx)
    dxm = wl.snap_to_bf16(np.maximum(r.standard_normal(case["x"].shape), 0).astype(np.float32))
    ad = wl.snap_to_bf16(r.standard_normal(case["x"].shape).astype(np.float32))
    print(f"[random shape {idx}] {shape}", flush=True)
    got = pu.gpu_block(case, addend=ad, dx_mask=dxm, premasked=True)
    errs = pu.check_block(case, got, addend=ad, dx_mask=dxm, premasked=True)
    show(f"random shape {idx}", errs)


@pytest.mark.parametrize("idx", range(len(RANDOM_SHAPES)), ids=lambda i: "k{K}s{stride}p{pad}_{C_in}to{C_out}_{N}x{H}x{W}".format(**RANDOM_SHAPES[i]))
def test_random_layer_shapes_riding_reduction_changes_no_bit(idx, sol_env):
    """The same shapes with the split reduction as the library places it (riding with the data-gradient launch where
    the launch can carry it), with a forced odd number of riding workgroups, and as a launch of its own: dx, dW,
    dscale and dshift are the same bits in all three."""
    shape = RANDOM_SHAPES[idx]
    case = pu.make_case(300 + idx, **shape)
    r = np.random.default_rng(400 + idx)
    dxm = wl.snap_to_bf16(np.maximum(r.standard_normal(case["x"].shape), 0).astype(np.float32))
    ad = wl.snap_to_bf16(r.standard_normal(case["x"].shape).astype(np.float32))
    out = {}
    for mode in (1, 7, 0):
        sol_env("SOL_REDUCE_RIDES", mode)
        print(f"[random shape {idx}] {shape} SOL_REDUCE_RIDES={mode}", flush=True)
        out[mode] = pu.gpu_block(case, addend=ad, dx_mask=dxm, premasked=True)
    for mode in (1, 7):
        for key in ("dx", "dW", "dscale", "dshift"):
            a, b = out[mode][key], out[0][key]
            assert np.array_equal(a, b), f"SOL_REDUCE_RIDES={mode}, {key}: {int((a != b).sum())} elements differ"


@pytest.mark.parametrize("tile", [0, 1, 2, 3])
def test_bf16_every_tile_shape(tile, sol_env):
    sol_env("SOL_IGEMM_TILE", tile)
    case = pu.make_case(9, 2, 19, 17, 32, 136, 3, 1, 1, res=True)
    got = pu.gpu_block(case)
    show(f"tile{tile}", pu.check_block(case, got))


@pytest.mark.parametrize("premask", [0, 1])
@pytest.mark.parametrize("want_dres", [False, True])
@pytest.mark.parametrize("shape", [
    dict(N=2, H=14, W=14, C_in=64, C_out=128, K=3, stride=1, pad=1, res=True),
    dict(N=2, H=15, W=13, C_in=128, C_out=64, K=1, stride=2, pad=0),
])
def test_block_that_masks_its_own_gradient(shape, want_dres, premask, sol_env):
    """sol_block_bwd with SOL_RELU and y, the call as the interface states it.  By default the library writes the
    masked gradient once (into dres when the caller asks for it, else into the workspace) and runs both gradient
    GEMMs with the pipelined kernels; SOL_PREMASK=0 keeps the mask inside the general kernels' operand staging.
    Same checks either way, dres bit-exact."""
    sol_env("SOL_PREMASK", premask)
    case = pu.make_case(91, **shape)
    got = pu.gpu_block(case, want_dres=want_dres)
    show(f"own mask premask={premask} dres={want_dres} {shape}", pu.check_block(case, got))


@pytest.mark.parametrize("splits", [1, 3, 50])
def test_bf16_wgrad_split_counts(splits, sol_env):
    sol_env("SOL_WGRAD_SPLITS", splits)
    case = pu.make_case(10, 2, 21, 19, 32, 40, 3, 1, 1)
    got = pu.gpu_block(case)
    show(f"splits{splits}", pu.check_block(case, got))


RIDING_SHAPES = {
    # name: (block, plan tile of the data-gradient GEMM); K = KH * KW * C_in decides the team width and the chunks
    "k64_one_wave_per_row": (dict(N=2, H=9, W=11, C_in=64, C_out=192, K=1, stride=1, pad=0, relu=False), 0),
    "k256_one_wave_per_row": (dict(N=1, H=12, W=11, C_in=256, C_out=128, K=1, stride=1, pad=0, relu=False), 0),
    "k512_two_waves_per_row": (dict(N=2, H=7, W=9, C_in=512, C_out=64, K=1, stride=1, pad=0, relu=False), 3),
    "k576_whole_workgroup": (dict(N=2, H=10, W=9, C_in=64, C_out=128, K=3, stride=1, pad=1, relu=False), 0),
    "k1152_two_chunks": (dict(N=1, H=11, W=10, C_in=128, C_out=64, K=3, stride=1, pad=1, relu=False), 0),
    "k2304_three_chunks": (dict(N=1, H=9, W=9, C_in=256, C_out=192, K=3, stride=1, pad=1, relu=False), 3),
    "k4608_two_passes_stride2": (dict(N=1, H=9, W=10, C_in=512, C_out=64, K=3, stride=2, pad=1, relu=False), 0),
    "panel_k128_to_256": (dict(N=2, H=10, W=13, C_in=256, C_out=128, K=1, stride=1, pad=0, relu=False), 4),
    # the two smaller tiles carry the form of the reduction that needs few registers (one chunk, 8 splits in flight)
    "k128_tile_128x64": (dict(N=2, H=9, W=11, C_in=128, C_out=192, K=1, stride=1, pad=0, relu=False), 1),
    "k1152_tile_128x64": (dict(N=1, H=11, W=10, C_in=128, C_out=64, K=3, stride=1, pad=1, relu=False), 1),
    "k576_tile_64x64": (dict(N=2, H=10, W=9, C_in=64, C_out=128, K=3, stride=1, pad=1, relu=False), 2),
}


@pytest.mark.parametrize("riders", [1, 3, 40], ids=lambda r: "riders_auto" if r == 1 else f"riders{r}")
@pytest.mark.parametrize("shape", list(RIDING_SHAPES), ids=list(RIDING_SHAPES))
def test_split_reduction_riding_with_the_data_gradient(shape, riders, sol_env):
    """A backward call that computes both branches with the pipelined kernels appends the reduction of the split weight
    gradient to the data-gradient launch (workgroups behind the tiles): every team width and chunk count of the row
    reduction, on every tile of the pipelined kernel and on the panel kernel, with the library's own number of riding workgroups, with
    3 (every workgroup walks over many rows) and with 40, and with the accumulate flag.  The launch trace shows that
    the reduction rode; results are compared with the CPU checker and, bit for bit, with the reduction as a launch
    of its own."""
    spec, tile = RIDING_SHAPES[shape]
    case = pu.make_case(131, **spec)
    d = case["d"]
    r = np.random.default_rng(132)
    init = r.standard_normal(case["w"].shape).astype(np.float32)
    try:
        for flags in (0, B.SOL_DW_ACCUMULATE):
            desc = B.BlockDesc(d.N, d.H, d.W, d.C_in, d.C_out, d.KH, d.KW, d.stride, d.pad, B.SOL_BF16, flags)
            B.sol_block_set_plan(desc, B.SOL_PLAN_DGRAD, (tile, 2 if tile == 3 else 0, 0))
        out = {}
        for mode in (riders, 0):
            sol_env("SOL_REDUCE_RIDES", mode)
            print(f"[riding] {shape}: SOL_REDUCE_RIDES={mode}", flush=True)
            B.sol_trace_start(64)
            plain = pu.gpu_block(case)
            acc = pu.gpu_block(case, accumulate=True, dw_init=init)
            kinds = [B.sol_trace_kind_name(k) for k, _, _, _ in B.sol_trace_stop(64)]
            rode = sum("+ split reduction" in k for k in kinds)
            alone = kinds.count("split reduction")
            assert (rode, alone) == ((2, 0) if mode else (0, 2)), kinds
            out[mode] = (plain, acc)
        show(f"riding {shape} riders {riders}", pu.check_block(case, out[riders][0]))
        for which in (0, 1):
            for key in ("dx", "dW", "dscale", "dshift"):
                a, b = out[riders][which][key], out[0][which][key]
                assert np.array_equal(a, b), f"{key} (accumulate={which}): {int((a != b).sum())} elements differ"
        np.testing.assert_allclose(out[riders][1]["dW"], out[riders][0]["dW"] + init, rtol=1e-6, atol=1e-7)
    finally:
        B.sol_clear_plans()


def test_bf16_addend_mask_and_accumulate():
    case = pu.make_case(11, 2, 10, 9, 16, 24, 3, 1, 1, res=True)
    r = np.random.default_rng(12)
    ad = wl.snap_to_bf16(r.standard_normal(case["x"].shape).astype(np.float32))
    am = wl.snap_to_bf16(np.maximum(r.standard_normal(case["x"].shape), 0).astype(np.float32))
    got = pu.gpu_block(case, addend=ad, addend_mask=am, want_dres=True)
    show("addend+mask", pu.check_block(case, got, addend=ad, addend_mask=am))
    got = pu.gpu_block(case, addend=ad)
    show("addend", pu.check_block(case, got, addend=ad))
    # accumulate flag: results are added to what the buffers held
    base = pu.gpu_block(case)
    init = r.standard_normal(case["w"].shape).astype(np.float32)
    acc = pu.gpu_block(case, accumulate=True, dw_init=init)
    np.testing.assert_allclose(acc["dW"], base["dW"] + init, rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(acc["dscale"], base["dscale"] + 1.0, rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(acc["dshift"], base["dshift"] - 2.0, rtol=1e-6, atol=1e-7)


@pytest.mark.parametrize("shape", [
    dict(N=2, H=14, W=14, C_in=64, C_out=128, K=3, stride=1, pad=1, res=True),      # pipelined kernel
    dict(N=2, H=14, W=14, C_in=128, C_out=64, K=1, stride=1, pad=0),
    dict(N=2, H=15, W=13, C_in=64, C_out=64, K=3, stride=2, pad=1),
    dict(N=2, H=15, W=13, C_in=64, C_out=128, K=1, stride=2, pad=0, relu=False),    # 3 of 4 pixels see no tap: fill launch
    dict(N=1, H=9, W=9, C_in=24, C_out=40, K=3, stride=1, pad=1),                   # general kernel
    dict(N=1, H=8, W=8, C_in=8, C_out=8, K=3, stride=1, pad=1, bf16=False),          # fp32 path
])
def test_premasked_gradient_and_dx_mask(shape):
    """The layer-merged backward: dy arrives already masked (loss kernel with mask_by_y), the block runs
    without SOL_RELU / y, and its dx is masked by the upstream activation in the epilogue."""
    case = pu.make_case(21, **shape)
    r = np.random.default_rng(22)
    snap = wl.snap_to_bf16 if case["bf16"] else (lambda a: a)
    dxm = snap(np.maximum(r.standard_normal(case["x"].shape), 0).astype(np.float32))
    ad = snap(r.standard_normal(case["x"].shape).astype(np.float32))
    got = pu.gpu_block(case, addend=ad, dx_mask=dxm, premasked=True)
    show(f"premasked {shape}", pu.check_block(case, got, addend=ad, dx_mask=dxm, premasked=True))


@pytest.mark.parametrize("shape", [
    dict(N=4, H=14, W=14, C_in=256, C_out=64, K=3, stride=1, pad=1),                  # pipelined kernels
    dict(N=2, H=15, W=13, C_in=24, C_out=40, K=3, stride=2, pad=1),                   # general kernels
    dict(N=1, H=8, W=8, C_in=8, C_out=8, K=3, stride=1, pad=1, bf16=False),           # fp32 path
])
def test_data_and_weight_branch_as_two_calls(shape):
    """Backward issued as two calls on two streams (dW = NULL / dx = NULL) sharing one workspace: same bits as
    the single call, and parity with the checker."""
    case = pu.make_case(31, res=True, **shape)
    one = pu.gpu_block(case, want_dres=True)
    two = pu.gpu_block(case, want_dres=True, two_calls=True)
    for k in ("dx", "dW", "dscale", "dshift", "dres"):
        assert np.array_equal(one[k], two[k]), k
    show(f"two calls {shape}", pu.check_block(case, two))


@pytest.mark.parametrize("shape", [
    dict(N=2, H=30, W=530, C_in=3, C_out=64, K=7, stride=2, pad=3),            # stem: 3 row segments, ragged
    dict(N=3, H=9, W=11, C_in=4, C_out=64, K=3, stride=2, pad=1),              # 3x3, 4 channels: only filter rows 0..2
    dict(N=1, H=16, W=16, C_in=1, C_out=64, K=5, stride=2, pad=2),             # 1 channel
    dict(N=5, H=64, W=64, C_in=3, C_out=64, K=7, stride=2, pad=3),             # more row segments than workgroups share evenly
])
def test_few_channel_weight_gradient(shape):
    """The stem's own weight-gradient kernels (gradient masked upstream, no data gradient), including accumulation."""
    case = pu.make_case(41, **shape)
    got = pu.gpu_block(case, need_dx=False, premasked=True)
    show(f"few-channel wgrad {shape}", pu.check_block(case, got, need_dx=False, premasked=True))
    again = pu.gpu_block(case, need_dx=False, premasked=True)
    for k in ("dW", "dscale", "dshift"):
        assert np.array_equal(got[k], again[k]), k
    init = np.random.default_rng(42).standard_normal(case["w"].shape).astype(np.float32)
    acc = pu.gpu_block(case, need_dx=False, premasked=True, accumulate=True, dw_init=init)
    np.testing.assert_allclose(acc["dW"], got["dW"] + init, rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(acc["dscale"], got["dscale"] + 1.0, rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(acc["dshift"], got["dshift"] - 2.0, rtol=1e-6, atol=1e-7)


def test_untouched_pixels_take_addend_and_masks():
    """1x1 / stride 2: pixels no tap reaches get the (gated) addend and the output mask from the fill launch."""
    case = pu.make_case(51, 2, 14, 14, 64, 128, 1, 2, 0, relu=False)
    r = np.random.default_rng(52)
    ad = wl.snap_to_bf16(r.standard_normal(case["x"].shape).astype(np.float32))
    am = wl.snap_to_bf16(np.maximum(r.standard_normal(case["x"].shape), 0).astype(np.float32))
    dxm = wl.snap_to_bf16(np.maximum(r.standard_normal(case["x"].shape), 0).astype(np.float32))
    got = pu.gpu_block(case, addend=ad, addend_mask=am, dx_mask=dxm)
    show("untouched pixels", pu.check_block(case, got, addend=ad, addend_mask=am, dx_mask=dxm))
    expect = np.where((am > 0) & (dxm > 0), ad, 0.0)
    assert np.array_equal(got["dx"][:, :, 1::2, :], expect[:, :, 1::2, :])      # odd rows: no tap, exact copy
    assert np.array_equal(got["dx"][:, :, :, 1::2], expect[:, :, :, 1::2])


@pytest.mark.parametrize("shape", [
    dict(N=8, H=23, W=23, C_in=64, C_out=256, K=1, stride=1, pad=0, res=True),          # forward: K = 64
    dict(N=8, H=23, W=23, C_in=128, C_out=512, K=1, stride=1, pad=0, relu=False),       # K = 128, plain epilogue
    dict(N=8, H=23, W=23, C_in=256, C_out=1024, K=1, stride=1, pad=0, res=True),        # K = 256
    dict(N=8, H=23, W=23, C_in=512, C_out=256, K=1, stride=1, pad=0, res=True),         # K = 512
    dict(N=8, H=23, W=23, C_in=256, C_out=64, K=1, stride=1, pad=0, relu=False),        # data gradient: K = 64 -> 256 channels
    dict(N=8, H=23, W=23, C_in=1024, C_out=256, K=1, stride=1, pad=0, relu=False),      # data gradient: K = 256 -> 1024 channels
])
def test_pointwise_layers_with_short_reduction(shape):
    """1x1 / stride 1 with a short reduction and >= 256 output channels (forward of an expand layer, data
    gradient of a reduce layer): 4232 pixels, not a multiple of any tile height, many tiles per compute
    unit's worth of workgroups.  The data gradient carries a gated addend and an output mask."""
    case = pu.make_case(61, **shape)
    r = np.random.default_rng(62)
    dxm = wl.snap_to_bf16(np.maximum(r.standard_normal(case["x"].shape), 0).astype(np.float32))
    ad = wl.snap_to_bf16(r.standard_normal(case["x"].shape).astype(np.float32))
    am = wl.snap_to_bf16(np.maximum(r.standard_normal(case["x"].shape), 0).astype(np.float32))
    got = pu.gpu_block(case, addend=ad, addend_mask=am, dx_mask=dxm, premasked=True)
    show(f"pointwise {shape}", pu.check_block(case, got, addend=ad, addend_mask=am, dx_mask=dxm, premasked=True))


def test_gates_treat_signed_zero_and_denormals_like_the_comparison():
    """A gate lets a value through where the mask is > 0: -0.0 and +0.0 block, the smallest positive bf16
    denormal passes, negative values (denormal, -inf) block, +inf passes."""
    case = pu.make_case(71, 2, 14, 14, 64, 128, 1, 1, 0, relu=False)
    r = np.random.default_rng(72)
    specials = np.array([-0.0, 0.0, 1e-40, -1e-40, 1.0, -1.0, np.inf, -np.inf], dtype=np.float32)
    pick = lambda: wl.snap_to_bf16(specials[r.integers(0, len(specials), size=case["x"].shape)])
    am, dxm = pick(), pick()
    assert (am == 0).any() and np.signbit(am[am == 0]).any() and (np.abs(am[am != 0]) < 1e-38).any()
    ad = wl.snap_to_bf16(r.standard_normal(case["x"].shape).astype(np.float32))
    got = pu.gpu_block(case, addend=ad, addend_mask=am, dx_mask=dxm, premasked=True)
    show("special gates", pu.check_block(case, got, addend=ad, addend_mask=am, dx_mask=dxm, premasked=True))
    assert np.all(got["dx"][~(dxm > 0)] == 0)
    w0 = dict(case, w=np.zeros_like(case["w"]))                  # no convolution term: dx is the gated addend itself
    got = pu.gpu_block(w0, addend=ad, addend_mask=am, dx_mask=dxm, premasked=True)
    assert np.array_equal(got["dx"], np.where((am > 0) & (dxm > 0), ad, 0.0))


def test_runs_are_bitwise_reproducible():
    case = pu.make_case(13, 2, 28, 28, 64, 128, 3, 1, 1, res=True)
    a, b = pu.gpu_block(case), pu.gpu_block(case)
    for k in ("y", "dx", "dW", "dscale", "dshift"):
        assert np.array_equal(a[k], b[k]), k


def test_masked_gradient_is_exactly_zero_where_y_is_zero():
    case = pu.make_case(14, 2, 14, 14, 32, 64, 1, 1, 0)
    got = pu.gpu_block(case, want_dres=True)
    assert np.all(got["dres"][got["y"] == 0] == 0)
    assert np.array_equal(got["dres"][got["y"] > 0], got["dy"][got["y"] > 0])
    # weights = 0 and shift < 0: every output is 0, so every gradient must be exactly 0
    case["w"] = np.zeros_like(case["w"])
    case["shift"] = -np.abs(case["shift"]) - 0.1
    got = pu.gpu_block(case)
    assert np.all(got["y"] == 0) and np.all(got["dx"] == 0) and np.all(got["dW"] == 0)
    assert np.all(got["dscale"] == 0) and np.all(got["dshift"] == 0)


def test_error_codes_on_device_pointers():
    d = B.BlockDesc(1, 8, 8, 8, 8, 3, 3, 1, 1, B.SOL_BF16, B.SOL_RELU)
    t = torch.zeros(4096, dtype=torch.bfloat16, device="cuda")
    f = torch.zeros(64, dtype=torch.float32, device="cuda")
    assert B.sol_block_fwd(d, t, t, f, f, None, None, None, 0, check=False) == -1          # y NULL
    assert B.sol_block_fwd(d, t.data_ptr() + 2, t, f, f, None, t, None, 0, check=False) == -3   # misaligned
    ws = torch.zeros(16, dtype=torch.uint8, device="cuda")
    assert B.sol_block_bwd(d, t, t, t, t, t, f, f, f, f, None, None, None, None, ws, 16, check=False) == -5
