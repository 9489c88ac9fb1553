"""Synthetic-input recipe: shapes, layer counts, FLOP totals, storage-grid snapping."""
import numpy as np

from oracle import oracle as orc
from paper_2205_10357_amd import workloads as wl


def test_resnet50_stack_has_53_convs_and_expected_flops():
    ops = wl.resnet50_ops()
    convs = [o for o in ops if o.op == "conv"]
    assert len(convs) == 53 and sum(o.op == "maxpool" for o in ops) == 1
    w = wl.Workload(4, "t", "bf16", 1, 224, 224, 3, ops, np.zeros((1, 3, 1, 1), np.float32), train=False)
    shp = w.tensor_shapes()
    assert shp[ops[-1].out] == (2048, 7, 7)
    assert abs(w.flops_forward() / 1e9 - 8.17) < 0.01           # per image


def test_bottleneck_and_stage2_flops():
    w3 = wl.Workload(3, "t", "bf16", 64, 14, 14, 1024, wl.bottleneck14_ops(), np.zeros((1,), np.float32))
    assert abs(w3.flops_step() / 1e9 - 83.85) < 0.01
    w5 = wl.Workload(5, "t", "bf16", 128, 56, 56, 256, wl.stage2_ops(True), np.zeros((1,), np.float32))
    assert len(w5.conv_blocks()) == 13 and abs(w5.flops_forward() / 1e9 - 263.07) < 0.01
    w5u = wl.Workload(5, "t", "bf16", 128, 28, 28, 512, wl.stage2_ops(False), np.zeros((1,), np.float32))
    assert len(w5u.conv_blocks()) == 12 and abs(w5u.flops_forward() / 1e9 - 223.61) < 0.01
    w2 = wl.Workload(2, "t", "bf16", 32, 224, 224, 3, wl.resnet50_ops()[:1], np.zeros((1,), np.float32),
                     need_input_grad=False)
    assert abs(w2.flops_step() / 1e9 - 15.1) < 0.01


def test_single_block_recipe():
    w = wl.single_block_f32()
    assert w.x.shape == (1, 16, 16, 16) and w.x.dtype == np.float32
    assert w.x.min() >= 0 and w.x.max() < 1
    p = w.params[0]
    assert p["W"].shape == (16, 16, 3, 3)
    assert np.array_equal(p["W"], wl.draw_weight(0, 16, 16, 3, 3))            # weight stream uses seed 0
    assert abs(p["W"].std() - np.sqrt(2.0 / 144)) < 0.01
    assert p["scale"].min() >= 0.5 and p["scale"].max() < 1.5
    assert w.target.shape == (1, 16, 16, 16)
    again = wl.single_block_f32()
    assert np.array_equal(again.x, w.x) and np.array_equal(again.target, w.target)


def test_streams_are_independent_per_tensor():
    w = wl.bottleneck14_bf16(n=1, hw=4)
    a, b = w.params[0]["W"], w.params[2]["W"]
    assert a.shape == (256, 1024, 1, 1) and b.shape == (1024, 256, 1, 1)
    assert not np.array_equal(a.ravel()[:64], b.ravel()[:64])


def test_snap_to_bf16_agrees_with_checker_quantiser():
    a = (np.random.default_rng(0).standard_normal(50000) * 3).astype(np.float32)
    s = wl.snap_to_bf16(a)
    assert np.array_equal(s.astype(np.float64), orc.quantize_bf16(a.astype(np.float64)))
    assert np.array_equal(wl.snap_to_bf16(s), s)
    bits = wl.bf16_bits(s)
    assert bits.dtype == np.uint16
    assert np.array_equal((bits.astype(np.uint32) << 16).view(np.float32), s)


def test_memory_plan_of_the_static_schedule():
    """Bytes by kind, from shapes and execution order alone (hand-computed for the 14x14 bottleneck)."""
    w3 = wl.Workload(3, "t", "bf16", 64, 14, 14, 1024, wl.bottleneck14_ops(), np.zeros((1,), np.float32))
    m = w3.memory_plan(workspace_bytes=1000)
    px = 64 * 14 * 14
    assert m["input"] == px * 1024 * 2 and m["outputs"] == px * 1024 * 2 and m["target"] == px * 1024 * 2
    assert m["intermediates_all_kept"] == 2 * px * 256 * 2
    weights = 1024 * 256 + 9 * 256 * 256 + 256 * 1024
    assert m["parameters"] == weights * 2 + 2 * 4 * (256 + 256 + 1024)
    assert m["parameter_gradients"] == weights * 4 + 2 * 4 * (256 + 256 + 1024)
    assert m["activation_gradients"] == px * (1024 + 256 + 256 + 1024) * 2
    # inference: x stays alive for the shortcut; the peak is at the last block (x, a2, y)
    assert m["inference_peak_activations"] == px * (1024 + 256 + 1024) * 2
    assert m["workspace"] == 1000
    # ResNet-50 inference at N = 128: the largest tensor is the stem output (205.5 MB); the peak holds it twice over
    ops = wl.resnet50_ops()
    w4 = wl.Workload(4, "t", "bf16", 128, 224, 224, 3, ops, np.zeros((1,), np.float32), train=False)
    m4 = w4.memory_plan()
    assert abs(max(128 * c * h * ww * 2 for c, h, ww in w4.tensor_shapes().values()) / 1e6 - 205.5) < 0.1
    assert m4["inference_peak_activations"] < 0.3 * m4["intermediates_all_kept"]
    assert abs(m4["parameters"] / 1e6 - (23.45 * 2 + 0.2)) < 0.3
    assert "total_inference_minimum" in m4 and "total_training" not in m4


def test_inference_arena_never_overlaps_live_tensors():
    """Planned activation buffers of the inference schedule: at every op the tensors alive (written earlier
    and still to be read, the op's own output, the final output) occupy disjoint byte ranges; an op's output
    never shares bytes with its operands; the arena is no larger than keeping everything and no smaller than
    the largest set of bytes alive at one op."""
    for ops, (c, h, w) in ((wl.resnet50_ops(), (3, 224, 224)), (wl.bottleneck14_ops(), (1024, 14, 14)),
                           (wl.stage2_ops(True), (256, 56, 56))):
        n = 2
        W = wl.Workload(9, "t", "bf16", n, h, w, c, ops, np.zeros((1,), np.float32), train=False)
        offset, top = W.plan_inference_arena()
        shp = W.tensor_shapes()
        nbytes = {t: n * cc * hh * ww * 2 for t, (cc, hh, ww) in shp.items()}
        assert set(offset) == set(shp) - {0} and all(o % 256 == 0 for o in offset.values())
        last = {}
        for i, o in enumerate(ops):
            last[o.inp] = i
            if getattr(o, "res", None) is not None:
                last[o.res] = i
        last[ops[-1].out] = len(ops)
        born = {o.out: i for i, o in enumerate(ops)}
        lower = 0
        for i, o in enumerate(ops):
            alive = [t for t in offset if born[t] <= i <= last.get(t, born[t])]
            assert o.out in alive and all(t in alive for t in (o.inp, getattr(o, "res", None)) if t)
            spans = sorted((offset[t], offset[t] + nbytes[t]) for t in alive)
            assert all(a[1] <= b[0] for a, b in zip(spans, spans[1:])), f"overlap at op {i}"
            assert spans[-1][1] <= top
            lower = max(lower, sum(nbytes[t] for t in alive))
        assert lower <= top <= sum(-(-b // 256) * 256 for t, b in nbytes.items() if t != 0)
        assert W.memory_plan()["inference_arena"] == top
    # ResNet-50: the arena reaches the lower bound (stem output + pooled output and the like), a sixth of all-kept
    W = wl.Workload(4, "t", "bf16", 1, 224, 224, 3, wl.resnet50_ops(), np.zeros((1,), np.float32), train=False)
    assert W.plan_inference_arena()[1] == 3612672 and W.memory_plan()["intermediates_all_kept"] == 22428672
