"""GPU parity of the five workloads, run through the layer-list sequencer (same launch configuration as
the benchmark).  Small sizes are compared element by element; the full sizes on sampled outputs that the
CPU checker computes one by one.  Every comparison is teacher-forced per block: the checker is fed the
tensors the GPU stored (so the tolerance measures kernels, not bf16 drift over depth); the end-to-end
drift of the three-block chain is reported separately.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from oracle import oracle as orc                              # noqa: E402
from paper_2205_10357_amd import binding as B, runner, tuning, workloads as wl      # noqa: E402
from tests import parity_util as pu                           # noqa: E402

TOL = 1e-2              # bf16 tensors (y, dx)
TOL_F32 = 1e-5          # float32 outputs (dW, dscale, dshift): float32 sums of exact bf16 products


def over_tolerance(worst):
    return {k: v for k, v in worst.items() if v > (TOL_F32 if k.rsplit(".", 1)[-1] in ("dW", "dscale", "dshift") else TOL)}


def host(t, images=None):
    """NHWC device tensor -> NCHW float64 (optionally only some images)."""
    if images is not None:
        t = t[torch.as_tensor(images, device=t.device)]
    return np.ascontiguousarray(np.transpose(runner.download(t), (0, 3, 1, 2)))


def desc_of(seq, o, n):
    _, h, w = seq.shapes[o.inp]
    return orc.Desc(n, h, w, o.c_in, o.c_out, o.k, o.k, o.stride, o.pad, o.relu)


def rand_points(rng, shape, count):
    return np.stack([rng.integers(0, s, size=count) for s in shape], axis=1).astype(np.int32)


def rel(got, ref):
    return pu.rel_l2(got, ref)


def grad_source(w):
    """tensor id -> tensor id whose stored gradient IS this tensor's gradient: a tensor that is only used
    as a shortcut (a projection's output) takes the tail block's masked gradient as it is."""
    src = {}
    for o in w.conv_blocks():
        if o.res is not None and not any(oo.inp == o.res for oo in w.conv_blocks()):
            src[o.res] = o.out
    return src


# ----------------------------------------------------------------- element-by-element, small sizes
def check_chain_elementwise(w):
    seq = runner.Sequencer(w, "cuda:0", retain_activations=True)
    seq.step()
    torch.cuda.synchronize()
    n = w.n
    acts = {k: host(v) for k, v in seq.act.items()}
    dacts = {k: host(v) for k, v in seq.dact.items()} if w.train else {}
    producer = {o.out: o for o in w.ops}
    alias = grad_source(w)
    worst = {}
    dx_sum = {}
    for o in w.ops:
        if o.op != "conv":
            y = orc.maxpool(acts[o.inp], o.k, o.stride, o.pad)
            assert np.array_equal(y, acts[o.out])
            continue
        p = w.params[o.layer]
        d = desc_of(seq, o, n)
        y = orc.block_fwd(d, acts[o.inp], p["W"], p["scale"], p["shift"], acts[o.res] if o.res is not None else None)
        worst[f"{o.name}.y"] = rel(acts[o.out], y)
        if not w.train:
            continue
        dy = dacts[alias.get(o.out, o.out)]
        if o.relu:
            assert np.all(dy[acts[o.out] <= 0] == 0), f"{o.name}: stored gradient not masked by its ReLU"
        need_dx = o.inp in dacts
        g = orc.block_bwd(d, dy, acts[o.inp], p["W"], acts[o.out], p["scale"], need_dx=need_dx)
        gr = seq.grads[o.layer]
        worst[f"{o.name}.dW"] = rel(np.transpose(runner.download(gr["dW"]), (0, 3, 1, 2)), g["dW"])
        worst[f"{o.name}.dscale"] = rel(runner.download(gr["dscale"]), g["dscale"])
        worst[f"{o.name}.dshift"] = rel(runner.download(gr["dshift"]), g["dshift"])
        if need_dx:
            dx_sum[o.inp] = dx_sum.get(o.inp, 0.0) + g["dx"]
        if o.res is not None:
            dx_sum[o.res] = dx_sum.get(o.res, 0.0) + dy          # shortcut: the (masked) gradient itself
    for tid, dx in dx_sum.items():
        if tid not in dacts or not any(oo.inp == tid for oo in w.conv_blocks()):
            continue
        src = producer.get(tid)
        if src is not None and src.relu:
            assert np.all(dacts[tid][acts[tid] <= 0] == 0)
            dx = np.where(acts[tid] > 0, dx, 0.0)
        worst[f"t{tid}.dx"] = rel(dacts[tid], dx)
    if w.train:
        last = w.ops[-1]
        dy_o = orc.l1_grad(acts[last.out], w.target)
        if last.relu:
            dy_o = np.where(acts[last.out] > 0, dy_o, 0.0)
        assert np.array_equal(dacts[last.out], orc.quantize_bf16(dy_o))
    bad = over_tolerance(worst)
    print(f"[parity] {w.name} N={n}: worst {max(worst.values()):.3g} over {len(worst)} tensors", flush=True)
    assert not bad, bad
    return seq, acts


def test_stem_block_full_size():
    """Workload 2 at its full size (N = 32): forward, dW, dscale, dshift; no gradient to the image."""
    w = wl.stem_bf16()
    p = w.params[0]
    case = dict(d=orc.Desc(w.n, 224, 224, 3, 64, 7, 7, 2, 3, True), bf16=True, x=w.x, w=p["W"], scale=p["scale"],
                shift=p["shift"], res=None, t=w.target)
    got = pu.gpu_block(case, need_dx=False)
    errs = pu.check_block(case, got, need_dx=False)
    print(f"[parity] stem N=32: {errs}", flush=True)


def test_bottleneck_small_elementwise_and_end_to_end_drift():
    w = wl.bottleneck14_bf16(n=4)
    seq, acts = check_chain_elementwise(w)
    # end-to-end: the checker's own chain, quantising where the GPU stores bf16 (informational bound)
    a = {0: w.x.astype(np.float64)}
    for o in w.conv_blocks():
        p = w.params[o.layer]
        d = desc_of(seq, o, w.n)
        a[o.out] = orc.quantize_bf16(orc.block_fwd(d, a[o.inp], p["W"], p["scale"], p["shift"],
                                                   a[o.res] if o.res is not None else None))
    drift = rel(acts[w.ops[-1].out], a[w.ops[-1].out])
    print(f"[parity] bottleneck end-to-end drift of y3 (bf16-quantised chain): {drift:.3g}", flush=True)
    assert drift < 2e-2


def test_stage2_small_elementwise():
    """Workload 5 topology (stride-2 block with projection + identity blocks) at N = 2, 28x28 input."""
    check_chain_elementwise(wl.stage2_train_bf16(n=2, faithful=True, hw=28))


def test_resnet50_small_elementwise():
    """Workload 4 topology (all 53 blocks + max-pool) at N = 1, 64x64 input."""
    check_chain_elementwise(wl.resnet50_infer_bf16(n=1, hw=64))


@pytest.mark.parametrize("geom", [
    dict(N=2, H=13, W=11, C=16, k=3, stride=2, pad=1),      # the stem's pool: every tap requested at once
    dict(N=1, H=9, W=10, C=8, k=3, stride=1, pad=1),
    dict(N=2, H=8, W=12, C=24, k=2, stride=2, pad=0),       # other windows: tap by tap
    dict(N=1, H=11, W=7, C=8, k=5, stride=2, pad=2),
    dict(N=1, H=7, W=9, C=12, k=3, stride=2, pad=1),        # channels not a multiple of 8: element by element
], ids=lambda g: "k{k}s{stride}p{pad}_c{C}".format(**g))
def test_maxpool_windows_bit_exact(geom):
    """The max-pool of the glue layer for several windows, strides and channel counts, bf16 and fp32: every output
    is one of the inputs, so the comparison with the CPU checker is bit for bit."""
    g = geom
    r = np.random.default_rng(77)
    x = wl.snap_to_bf16(r.standard_normal((g["N"], g["C"], g["H"], g["W"])).astype(np.float32))
    ref = orc.maxpool(x, g["k"], g["stride"], g["pad"])
    for dt, tdt in ((B.SOL_BF16, torch.bfloat16), (B.SOL_F32, torch.float32)):
        xd = torch.from_numpy(np.ascontiguousarray(np.transpose(x, (0, 2, 3, 1)))).to("cuda:0").to(tdt)
        yd = torch.full((g["N"], ref.shape[2], ref.shape[3], g["C"]), 7.0, dtype=tdt, device="cuda:0")
        B.sol_maxpool_fwd(dt, xd, yd, g["N"], g["H"], g["W"], g["C"], g["k"], g["stride"], g["pad"],
                          torch.cuda.current_stream())
        torch.cuda.synchronize()
        got = np.transpose(yd.float().cpu().numpy().astype(np.float64), (0, 3, 1, 2))
        assert np.array_equal(got, ref), (geom, dt)


# ------------------------------------------------------------------------- full sizes, sampled
def check_sampled(w, images, n_fwd=400, n_dx=300, dw_layers=(), n_dw=64, n_ch=2, seed=5):
    rng = np.random.default_rng(seed)
    seq = runner.Sequencer(w, "cuda:0", retain_activations=True)
    seq.step()
    torch.cuda.synchronize()
    images = list(images)
    nsub = len(images)
    producer = {o.out: o for o in w.ops}
    alias = grad_source(w)
    worst = {}
    sub_act = {}

    def act(tid):
        if tid not in sub_act:
            sub_act[tid] = host(seq.act[tid], images)
        return sub_act[tid]

    sub_dact = {}

    def dact(tid):
        if tid not in sub_dact:
            sub_dact[tid] = host(seq.dact[tid], images)
        return sub_dact[tid]

    dx_pts, dx_ref = {}, {}
    for o in w.ops:
        if o.op != "conv":
            assert np.array_equal(orc.maxpool(act(o.inp), o.k, o.stride, o.pad), act(o.out))
            continue
        p = w.params[o.layer]
        d = desc_of(seq, o, nsub)
        res = act(o.res) if o.res is not None else None
        pts = rand_points(rng, (nsub, o.c_out, d.Ho, d.Wo), n_fwd)
        v, y, mag = orc.fwd_points(d, act(o.inp), p["W"], p["scale"], p["shift"], res, pts)
        got = act(o.out)[tuple(pts.T)]
        worst[f"{o.name}.y"] = rel(got, y)
        if o.relu:
            band = np.abs(v) <= 2.0 ** -19 * mag
            assert not np.any(((got > 0) != (v > 0)) & ~band), f"{o.name}: ReLU mask mismatch"
        if not w.train:
            continue
        if o.inp in seq.dact:
            ip = dx_pts.setdefault(o.inp, rand_points(rng, (nsub,) + tuple(act(o.inp).shape[1:]), n_dx))
            dn = orc.Desc(nsub, d.H, d.W, d.C_in, d.C_out, d.KH, d.KW, d.stride, d.pad, False)   # dy is pre-masked
            dx_ref[o.inp] = dx_ref.get(o.inp, 0.0) + orc.dx_points(dn, dact(alias.get(o.out, o.out)), act(o.out), p["W"], p["scale"], ip)
        if o.res is not None and o.res in seq.dact and any(oo.inp == o.res for oo in w.conv_blocks()):
            ip = dx_pts.setdefault(o.res, rand_points(rng, (nsub,) + tuple(act(o.res).shape[1:]), n_dx))
            dx_ref[o.res] = dx_ref.get(o.res, 0.0) + dact(o.out)[tuple(ip.T)]
    for tid, ref in dx_ref.items():
        ip = dx_pts[tid]
        src = producer.get(tid)
        got = dact(tid)[tuple(ip.T)]
        if src is not None and src.relu:
            keep = act(tid)[tuple(ip.T)] > 0
            assert np.all(got[~keep] == 0)
            ref = np.where(keep, ref, 0.0)
        worst[f"t{tid}.dx"] = rel(got, ref)
    sub_act.clear()
    sub_dact.clear()
    # weight / affine gradients need every image: a few layers, a few outputs each
    for o in w.conv_blocks():
        if o.name not in dw_layers:
            continue
        p = w.params[o.layer]
        d = desc_of(seq, o, w.n)
        dn = orc.Desc(w.n, d.H, d.W, d.C_in, d.C_out, d.KH, d.KW, d.stride, d.pad, False)
        dy, y, x = host(seq.dact[alias.get(o.out, o.out)]), host(seq.act[o.out]), host(seq.act[o.inp])
        wp = rand_points(rng, (o.c_out, o.c_in, o.k, o.k), n_dw)
        ref = orc.dw_points(dn, dy, y, x, p["scale"], wp)
        dW = np.transpose(runner.download(seq.grads[o.layer]["dW"]), (0, 3, 1, 2))
        worst[f"{o.name}.dW"] = rel(dW[tuple(wp.T)], ref)
        ch = rng.choice(o.c_out, size=n_ch, replace=False).astype(np.int32)
        ds, db = orc.affine_grad_channels(dn, dy, y, x, p["W"], ch)
        worst[f"{o.name}.dscale"] = rel(runner.download(seq.grads[o.layer]["dscale"])[ch], ds)
        worst[f"{o.name}.dshift"] = rel(runner.download(seq.grads[o.layer]["dshift"])[ch], db)
        del dy, y, x
    bad = over_tolerance(worst)
    print(f"[parity] {w.name} N={w.n} sampled: worst {max(worst.values()):.3g} over {len(worst)} checks", flush=True)
    assert not bad, bad


def test_bottleneck_full_size_sampled():
    """Workload 3 as benchmarked (N = 64)."""
    check_sampled(wl.bottleneck14_bf16(), images=(0, 31, 63), dw_layers=("b.conv1", "b.conv2", "b.conv3"))


def test_resnet50_full_size_sampled():
    """Workload 4 (N = 128, 224x224, inference): every layer's output on sampled elements of two images."""
    check_sampled(wl.resnet50_infer_bf16(), images=(0, 64, 127), n_fwd=300)


def test_stage2_full_size_sampled():
    """Workload 5 (N = 128, training step over stage 2)."""
    check_sampled(wl.stage2_train_bf16(), images=(0, 64, 127),
                  dw_layers=("s2.b0.conv2", "s2.b0.proj", "s2.b0.conv3", "s2.b2.conv1"), n_dw=48)


@pytest.mark.parametrize("which", ["stage2_small", "bottleneck_full"])
def test_two_lane_backward_matches_one_lane(which):
    """Weight branches on a second stream (block by block behind the gradient they read): same bits.  At the
    benchmark size the kernels are long enough for a block's weight branch to still be running when the next
    block's data branch starts, which is why the second lane needs a workspace of its own."""
    w = wl.stage2_train_bf16(n=2, hw=14) if which == "stage2_small" else wl.bottleneck14_bf16()
    seq = runner.Sequencer(w, "cuda:0", retain_activations=True)
    seq.step()
    torch.cuda.synchronize()
    ref = {k: {n: t.clone() for n, t in v.items()} for k, v in seq.grads.items()}
    ref_d = {k: v.clone() for k, v in seq.dact.items()}
    assert seq._ws_side is None
    for it in range(3):
        for v in seq.grads.values():
            for t in v.values():
                t.fill_(3.0)
        torch.cuda.synchronize()
        seq.step(lanes=2)
        assert seq._ws_side is not None and seq._ws_side.data_ptr() != seq.ws.data_ptr()
        torch.cuda.synchronize()
        for k, v in ref.items():
            for n, t in v.items():
                assert torch.equal(seq.grads[k][n], t), (it, k, n)
        for c in seq._bwd_calls:
            if c["dx"] is not None:
                k = next(i for i, t in seq.dact.items() if t is c["dx"])
                assert torch.equal(seq.dact[k], ref_d[k]), (it, k)


def test_graph_replays_match_eager():
    """A captured step (two lanes: weight branches as parallel branches of the graph) replayed several times,
    with eager work and synchronisations in between, gives the eager one-lane result bit for bit every time."""
    w = wl.bottleneck14_bf16(n=8)
    seq = runner.Sequencer(w, "cuda:0", retain_activations=True)
    seq.step()
    torch.cuda.synchronize()
    ref = {k: v.clone() for k, v in seq.dact.items()}
    ref_dw = {k: v["dW"].clone() for k, v in seq.grads.items()}
    g = seq.capture()
    for it in range(4):
        for t in seq.dact.values():
            t.fill_(7.0)                      # eager work between replays
        for v in seq.grads.values():
            v["dW"].zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for k in ref:
            if any(c["dx"] is seq.dact[k] for c in seq._bwd_calls) or k == w.ops[-1].out:
                assert torch.equal(seq.dact[k], ref[k]), (it, k)
        for k in ref_dw:
            assert torch.equal(seq.grads[k]["dW"], ref_dw[k]), (it, k)


@pytest.mark.parametrize("size", ["small", "full"])
def test_inference_arena_gives_the_retained_run_bit_for_bit(size):
    """The inference version of the schedule keeps its activations in one planned arena (ranges reused after a
    tensor's last reader); its network output must equal, bit for bit, that of a run with one buffer per
    tensor, whose every layer the tests above check against the CPU checker.  Two passes: the arena is dirty
    from the first when the second starts."""
    w = wl.resnet50_infer_bf16(n=2, hw=64) if size == "small" else wl.resnet50_infer_bf16()
    kept = runner.Sequencer(w, "cuda:0", retain_activations=True)
    ref = kept.forward().clone()
    del kept
    seq = runner.Sequencer(w, "cuda:0")
    assert not seq.retain and seq.arena.numel() == w.plan_inference_arena()[1]
    assert seq.memory_report()["activation_buffers_allocated"] == seq.arena.numel()
    for _ in range(2):
        out = seq.forward()
        torch.cuda.synchronize()
        assert torch.equal(out, ref)


@pytest.mark.parametrize("size", ["small", "full"])
def test_inference_graph_replays_match_eager_and_checker(size):
    """The inference version of the schedule (nothing retained, one activation arena) captured as a HIP graph:
    every replay, with eager work and synchronisations in between, gives the eager run's bits; the eager run is
    compared with the CPU checker on sampled outputs of the network's last layer (teacher-forced on the
    retained run of the same schedule)."""
    w = wl.resnet50_infer_bf16(n=2, hw=64) if size == "small" else wl.resnet50_infer_bf16()
    seq = runner.Sequencer(w, "cuda:0")
    assert not seq.retain
    ref = seq.forward().clone()
    torch.cuda.synchronize()
    g = seq.capture(lanes=1)
    out = seq.act[w.ops[-1].out]
    for it in range(3):
        seq.arena.fill_(77)                  # eager work between the replays: the arena is dirty
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, ref), it
    seq.step_prepared()                      # the prepared sequence issues the same launches
    torch.cuda.synchronize()
    assert torch.equal(out, ref)
    del seq, g
    # the last block against the checker, fed with the tensors a retained run stored
    kept = runner.Sequencer(w, "cuda:0", retain_activations=True)
    assert torch.equal(kept.forward(), ref)
    torch.cuda.synchronize()
    o = w.conv_blocks()[-1]
    images = [0, w.n - 1]
    d = desc_of(kept, o, len(images))
    p = w.params[o.layer]
    rng = np.random.default_rng(17)
    pts = rand_points(rng, (len(images), o.c_out, d.Ho, d.Wo), 300)
    v, y, mag = orc.fwd_points(d, host(kept.act[o.inp], images), p["W"], p["scale"], p["shift"],
                               host(kept.act[o.res], images) if o.res is not None else None, pts)
    got = host(ref, images)[tuple(pts.T)]
    assert rel(got, y) < TOL
    pu.assert_elementwise_bf16("y (graph)", got, y, mag)


def test_plan_sweep_covers_strided_and_projection_layers():
    """The sweep on the stage-2 topology (stride-2 3x3, stride-2 1x1 projection, identity blocks): every distinct
    layer shape is timed for the kernels that serve it, installed plans are valid table entries, and the chain
    still matches the CPU checker under them."""
    w = wl.stage2_train_bf16(n=2, faithful=True, hw=28)
    try:
        seq = runner.Sequencer(w, "cuda:0")
        seq.step()
        report = tuning.tune(seq, iters=3, margin=0.0)
        shapes = {(o.c_in, o.c_out, o.k, o.stride, seq.shapes[o.inp][1]) for o in w.conv_blocks()}
        assert len(report) == len(shapes)
        for name, e in report.items():
            assert "fwd" in e and "wgrad" in e, name
            for kind, v in e.items():
                assert v["best_ms"] <= v["default_ms"] and (v["plan"] is None or len(v["plan"]) == 3), (name, kind)
        del seq
        check_chain_elementwise(w)
    finally:
        B.sol_clear_plans()


def test_tuned_plans_change_speed_only():
    """Time the candidate plans of the bottleneck's layers, install the winners (margin 0: whatever measured
    fastest, so that plans really are in force), and run the step again: the forward output and the input
    gradient keep their bits (they do not depend on tile shape or pipeline depth), the whole chain stays
    within tolerance of the CPU checker, and clearing the table restores the weight gradient's bits."""
    w = wl.bottleneck14_bf16(n=8)
    last = w.ops[-1].out
    try:
        seq = runner.Sequencer(w, "cuda:0")
        seq.step()
        torch.cuda.synchronize()
        y0, dx0 = seq.act[last].clone(), seq.dact[0].clone()
        dw0 = {k: v["dW"].clone() for k, v in seq.grads.items()}
        report = tuning.tune(seq, iters=3, margin=0.0)
        assert set(report) == {"b.conv1", "b.conv2", "b.conv3"}
        assert all(set(e) == {"fwd", "dgrad", "wgrad"} for e in report.values())
        installed = [B.sol_block_get_plan(seq.desc[o.layer], k) for o in w.conv_blocks() for k in range(3)]
        print("[tuning]", {n: {k: (v["plan"], round(v["default_ms"] * 1e3, 1), round(v["best_ms"] * 1e3, 1))
                              for k, v in e.items()} for n, e in report.items()}, flush=True)
        seq.step()
        torch.cuda.synchronize()
        assert torch.equal(seq.act[last], y0) and torch.equal(seq.dact[0], dx0)
        for k, v in seq.grads.items():
            assert rel(v["dW"].double().cpu().numpy(), dw0[k].double().cpu().numpy()) < 1e-5
        if any(p != (-1, 0, 0) for p in installed):
            check_chain_elementwise(w)                       # a fresh sequencer under the installed plans
        B.sol_clear_plans()
        seq2 = runner.Sequencer(w, "cuda:0")
        seq2.step()
        torch.cuda.synchronize()
        assert all(torch.equal(seq2.grads[k]["dW"], dw0[k]) for k in dw0)
    finally:
        B.sol_clear_plans()


def test_prepared_step_and_launch_trace():
    """The step recorded as a prepared sequence of the library gives the eager step's bits, and a launch trace
    of it lists the 13 launches of the bottleneck step by kind and layer, each with a plausible time."""
    w = wl.bottleneck14_bf16(n=8)
    seq = runner.Sequencer(w, "cuda:0")
    seq.step()
    torch.cuda.synchronize()
    ref = {k: v.clone() for k, v in seq.dact.items()}
    ref_g = {k: {n: t.clone() for n, t in v.items()} for k, v in seq.grads.items()}
    ref_y = seq.act[w.ops[-1].out].clone()
    for t in list(seq.dact.values()) + [t for v in seq.grads.values() for t in v.values()]:
        t.fill_(5.0)
    assert len(seq.prepared()) == 7
    B.sol_trace_start(256)
    for _ in range(3):
        seq.step_prepared()
    trace = B.sol_trace_stop(256)
    torch.cuda.synchronize()
    assert torch.equal(seq.act[w.ops[-1].out], ref_y)
    for k, v in ref.items():
        if any(c["dx"] is seq.dact[k] for c in seq._bwd_calls) or k == w.ops[-1].out:
            assert torch.equal(seq.dact[k], v), k
    for k, v in ref_g.items():
        for n, t in v.items():
            assert torch.equal(seq.grads[k][n], t), (k, n)
    # the reduction of a split weight gradient is a launch of its own or rides along with the data-gradient launch
    assert len(trace) % 3 == 0
    per_step = len(trace) // 3
    kinds = [B.sol_trace_kind_name(k) for k, _, _, _ in trace[:per_step]]
    print("[trace]", [(B.sol_trace_kind_name(k), tag, round(us, 1), round(at, 1)) for k, tag, us, at in trace[per_step:2 * per_step]], flush=True)
    assert sum(k.startswith("implicit GEMM (") for k in kinds) == 6 and kinds.count("weight-gradient GEMM (pipelined)") == 3
    riding = sum(k.endswith("+ split reduction") for k in kinds)
    assert riding + kinds.count("split reduction") == 3 and kinds.count("L1-loss gradient") == 1
    assert per_step == 13 - riding
    tags = [tag for _, tag, _, _ in trace[:per_step]]
    assert tags[:4] == [0, 1, 2, -2] and tags[4:] == sorted(tags[4:], reverse=True) and set(tags[4:]) == {0, 1, 2}
    assert all(0.5 < us < 5000 for _, _, us, _ in trace)
    starts = [at for _, _, _, at in trace]
    assert starts[0] == 0 and all(b > a for a, b in zip(starts, starts[1:]))          # one stream: launches in order
    # tracing is off again: nothing is recorded, a second stop is refused
    seq.step_prepared()
    torch.cuda.synchronize()
    import ctypes as C
    n = C.c_int32(0)
    assert B.lib().sol_trace_stop(None, 0, C.byref(n)) == -4
