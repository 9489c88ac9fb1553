"""Helpers shared by the GPU parity tests: run one block through the C-ABI and compare with the
CPU checker on the same values (teacher-forced: the checker's backward is fed the y the GPU
stored, so that the comparison measures kernels, not storage-format drift)."""
from __future__ import annotations

import numpy as np
import torch

from oracle import oracle as orc
from paper_2205_10357_amd import binding as B
from paper_2205_10357_amd import workloads as wl

TOL = {"f32": 1e-5, "bf16": 1e-2}   # max relative L2 error per output tensor
# dW, dscale and dshift are float32 in both modes: float32 sums of products that are exact in float32
# (bf16 x bf16), so they are held to the float32 tolerance whatever the storage type of the activations
TOL_F32_OUTPUTS = 1e-5


def bf16_ulp(ref: np.ndarray) -> np.ndarray:
    """Spacing of the bf16 grid at |ref| (8 significand bits; the smallest normal exponent below that)."""
    a = np.maximum(np.abs(np.asarray(ref, np.float64)), 2.0 ** -126)
    return 2.0 ** (np.floor(np.log2(a)) - 7)


def assert_elementwise_bf16(name: str, got: np.ndarray, ref: np.ndarray, mag: np.ndarray) -> None:
    """Every element, not only the norm: a stored bf16 value is the float32 result rounded once, and the
    float32 result differs from the exact one by accumulation-order noise of at most 2^-19 of the summed
    magnitudes, so |got - ref| <= 1 bf16 ulp (rounding, plus a possible step across a rounding boundary)
    + 2^-19 * mag.  A dropped row, a wrong tap or a stale element fails this long before it moves the norm."""
    got, ref, mag = (np.asarray(a, np.float64) for a in (got, ref, mag))
    bound = bf16_ulp(ref) + 2.0 ** -19 * mag
    bad = np.abs(got - ref) > bound
    assert not bad.any(), (f"{name}: {int(bad.sum())} of {bad.size} elements outside 1 ulp + 2^-19 * magnitude; worst "
                           f"{float(np.max(np.abs(got - ref) / bound)):.3g} x the bound at {np.argwhere(bad)[0].tolist()}")


def rel_l2(got: np.ndarray, ref: np.ndarray) -> float:
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    nr = float(np.linalg.norm(ref.ravel()))
    ne = float(np.linalg.norm((got - ref).ravel()))
    return ne / nr if nr > 0 else ne


def to_dev(a_nchw: np.ndarray, bf16: bool, perm=(0, 2, 3, 1)) -> torch.Tensor:
    a = np.ascontiguousarray(np.transpose(a_nchw, perm), dtype=np.float32)
    return torch.from_numpy(a).to(device="cuda", dtype=torch.bfloat16 if bf16 else torch.float32)


def vec_dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def to_host(t: torch.Tensor, perm=(0, 3, 1, 2)) -> np.ndarray:
    a = t.detach().to(device="cpu", dtype=torch.float64).numpy()
    return np.ascontiguousarray(np.transpose(a, perm)) if perm is not None else a


def make_case(seed, N, H, W, C_in, C_out, K, stride, pad, bf16=True, relu=True, res=False, x_dist="normal"):
    r = np.random.default_rng(seed)
    snap = wl.snap_to_bf16 if bf16 else (lambda a: np.asarray(a, np.float32))
    d = orc.Desc(N, H, W, C_in, C_out, K, K, stride, pad, relu)
    x = r.standard_normal((N, C_in, H, W)) if x_dist == "normal" else r.random((N, C_in, H, W))
    case = dict(
        d=d, bf16=bf16,
        x=snap(x.astype(np.float32)),
        w=snap((r.standard_normal((C_out, C_in, K, K)) * np.sqrt(2.0 / (C_in * K * K))).astype(np.float32)),
        scale=(0.5 + r.random(C_out)).astype(np.float32),
        shift=(0.1 * r.standard_normal(C_out)).astype(np.float32),
        res=snap(r.standard_normal((N, C_out, d.Ho, d.Wo)).astype(np.float32)) if res else None,
        t=snap(r.random((N, C_out, d.Ho, d.Wo)).astype(np.float32)),
    )
    return case


def gpu_block(case, need_dx=True, want_dres=False, addend=None, addend_mask=None, guard=True, accumulate=False,
              dw_init=None, dx_mask=None, premasked=False, two_calls=False):
    """Forward, L1 gradient and backward of one block on the GPU.  Returns host arrays in the
    checker's layout plus the raw device tensors."""
    d, bf16 = case["d"], case["bf16"]
    dt = B.SOL_BF16 if bf16 else B.SOL_F32
    flags = (B.SOL_RELU if d.relu else 0) | (B.SOL_DW_ACCUMULATE if accumulate else 0)
    desc = B.BlockDesc(d.N, d.H, d.W, d.C_in, d.C_out, d.KH, d.KW, d.stride, d.pad, dt, flags)
    tdt = torch.bfloat16 if bf16 else torch.float32
    x, w = to_dev(case["x"], bf16), to_dev(case["w"], bf16)
    scale, shift = vec_dev(case["scale"]), vec_dev(case["shift"])
    res = to_dev(case["res"], bf16) if case["res"] is not None else None
    t = to_dev(case["t"], bf16)

    def guarded(shape, dtype):
        """Output buffer with canary bands on both sides (detects out-of-bounds stores)."""
        n = int(np.prod(shape))
        pad = 64
        full = torch.full((n + 2 * pad,), -1536.0, dtype=dtype, device="cuda")
        return full, full[pad:pad + n].view(shape)

    y_full, y = guarded((d.N, d.Ho, d.Wo, d.C_out), tdt)
    dy_full, dy = guarded((d.N, d.Ho, d.Wo, d.C_out), tdt)
    dx_full, dx = guarded((d.N, d.H, d.W, d.C_in), tdt) if need_dx else (None, None)
    dW_full, dW = guarded((d.C_out, d.KH, d.KW, d.C_in), torch.float32)
    ds_full, dscale = guarded((d.C_out,), torch.float32)
    db_full, dshift = guarded((d.C_out,), torch.float32)
    dres_full, dres = guarded((d.N, d.Ho, d.Wo, d.C_out), tdt) if want_dres else (None, None)
    if dw_init is not None:
        dW.copy_(torch.from_numpy(np.ascontiguousarray(np.transpose(dw_init, (0, 2, 3, 1)), np.float32)).cuda())
        dscale.fill_(1.0)
        dshift.fill_(-2.0)
    # the backward call below may drop SOL_RELU (premasked): ask for the descriptor that call will carry
    bwd_desc = B.BlockDesc(d.N, d.H, d.W, d.C_in, d.C_out, d.KH, d.KW, d.stride, d.pad, dt,
                           flags & ~B.SOL_RELU) if premasked else desc
    ws_bytes = B.sol_block_workspace_bytes(bwd_desc, B.SOL_PASS_BWD)
    ws = torch.full((ws_bytes // 4 + 64,), float("nan"), dtype=torch.float32, device="cuda")   # poisoned
    ad = to_dev(addend, bf16) if addend is not None else None
    am = to_dev(addend_mask, bf16) if addend_mask is not None else None
    dxm = to_dev(dx_mask, bf16) if dx_mask is not None else None

    fws_bytes = B.sol_block_workspace_bytes(desc, B.SOL_PASS_FWD)
    fws = torch.full((fws_bytes // 4 + 64,), float("nan"), dtype=torch.float32, device="cuda") if fws_bytes else None
    B.sol_block_fwd(desc, x, w, scale, shift, res, y, fws, fws_bytes)
    B.sol_l1_loss_grad(dt, y, t, dy, y.numel(), premasked and d.relu)
    if premasked:           # gradient already masked by this block's ReLU: backward without flag and y
        desc = B.BlockDesc(d.N, d.H, d.W, d.C_in, d.C_out, d.KH, d.KW, d.stride, d.pad, dt,
                           flags & ~B.SOL_RELU)
    ymask = None if premasked else y
    if two_calls:           # weight branch on a second stream, data branch on the first, one shared workspace
        main, side = torch.cuda.current_stream(), torch.cuda.Stream()
        side.wait_stream(main)
        B.sol_block_bwd(desc, dy, x, w, ymask, None, dW, dscale, dshift, scale, None, None, None, None, ws, ws_bytes,
                        stream=side)
        if need_dx or want_dres:
            B.sol_block_bwd(desc, dy, x, w, ymask, dx, None, None, None, scale, dres, ad, am, dxm, ws, ws_bytes,
                            stream=main)
        main.wait_stream(side)
    else:
        B.sol_block_bwd(desc, dy, x, w, ymask, dx, dW, dscale, dshift, scale, dres, ad, am, dxm, ws, ws_bytes)
    torch.cuda.synchronize()

    if guard:
        for name, full, inner in (("y", y_full, y), ("dy", dy_full, dy), ("dx", dx_full, dx), ("dW", dW_full, dW),
                                  ("dscale", ds_full, dscale), ("dshift", db_full, dshift), ("dres", dres_full, dres)):
            if full is None:
                continue
            n = inner.numel()
            band = torch.cat([full[:64], full[64 + n:]]).float()
            assert bool((band == -1536.0).all()), f"canary around {name} overwritten"
    out = dict(
        y=to_host(y), dy=to_host(dy), dx=to_host(dx) if need_dx else None,
        dW=to_host(dW), dscale=to_host(dscale, None), dshift=to_host(dshift, None),
        dres=to_host(dres) if want_dres else None,
        dev=dict(y=y, dy=dy, dx=dx, dW=dW, dscale=dscale, dshift=dshift),
    )
    return out


def check_block(case, got, need_dx=True, addend=None, addend_mask=None, tol=None, dx_mask=None, premasked=False):
    """Element-by-element comparison with the checker; returns dict of relative L2 errors."""
    d, bf16 = case["d"], case["bf16"]
    tol = tol if tol is not None else TOL["bf16" if bf16 else "f32"]
    errs = {}
    y_o, z_o = orc.block_fwd(d, case["x"], case["w"], case["scale"], case["shift"], case["res"], return_z=True)
    errs["y"] = rel_l2(got["y"], y_o)
    mag = None
    if d.relu or bf16:
        mag = np.abs(case["scale"]).astype(np.float64)[None, :, None, None] * \
            orc.conv(d, np.abs(case["x"]), np.abs(case["w"])) + \
            np.abs(case["shift"]).astype(np.float64)[None, :, None, None] + \
            (np.abs(case["res"]) if case["res"] is not None else 0.0)
    if bf16:
        assert_elementwise_bf16("y", got["y"], y_o, mag)
    # ReLU mask: identical outside a band of pre-activations within fp32 accumulation noise of zero
    if d.relu:
        v = case["scale"].astype(np.float64)[None, :, None, None] * z_o + \
            case["shift"].astype(np.float64)[None, :, None, None] + (case["res"] if case["res"] is not None else 0.0)
        band = np.abs(v) <= 2.0 ** -19 * mag          # fp32 accumulation-order noise around zero
        mism = ((got["y"] > 0) != (v > 0)) & ~band
        assert not mism.any(), f"{int(mism.sum())} ReLU mask mismatches outside the rounding band"
        assert not np.any(np.signbit(got["y"])), "ReLU output has a negative zero or negative value"
        errs["mask_band"] = int(band.sum())
    # loss gradient: exact function of the stored y
    dy_o = orc.l1_grad(got["y"], case["t"])
    if premasked and d.relu:
        dy_o = np.where(got["y"] > 0, dy_o, 0.0)
    if bf16:
        dy_o = orc.quantize_bf16(dy_o)
    else:
        dy_o = dy_o.astype(np.float32).astype(np.float64)
    assert np.array_equal(got["dy"], dy_o), "L1 gradient differs"
    g = orc.block_bwd(d, got["dy"], case["x"], case["w"], got["y"], case["scale"], need_dx=need_dx, need_dres=True)
    if need_dx:
        dx_o = g["dx"]
        if addend is not None:
            dx_o = dx_o + (np.where(addend_mask > 0, addend, 0.0) if addend_mask is not None else addend)
        if dx_mask is not None:
            assert np.all(got["dx"][dx_mask <= 0] == 0), "dx not exactly zero where the mask is <= 0"
            dx_o = np.where(dx_mask > 0, dx_o, 0.0)
        errs["dx"] = rel_l2(got["dx"], dx_o)
        if bf16:
            # element by element against the same definition with the weights the data gradient multiplies:
            # scale[co] * W rounded once to bf16 (product taken in float32, as on the GPU)
            wf = wl.snap_to_bf16(case["scale"].astype(np.float32)[:, None, None, None] * case["w"].astype(np.float32))
            one = np.ones(d.C_out)
            dn = orc.Desc(d.N, d.H, d.W, d.C_in, d.C_out, d.KH, d.KW, d.stride, d.pad, False)
            gm = g["dres"]                                           # the masked gradient
            ref = orc.block_bwd(dn, gm, case["x"], wf, got["y"], one)["dx"]
            dmag = orc.block_bwd(dn, np.abs(gm), case["x"], np.abs(wf), got["y"], one)["dx"]
            if addend is not None:
                a = np.where(addend_mask > 0, addend, 0.0) if addend_mask is not None else addend
                ref, dmag = ref + a, dmag + np.abs(a)
            if dx_mask is not None:
                ref, dmag = np.where(dx_mask > 0, ref, 0.0), np.where(dx_mask > 0, dmag, 0.0)
            assert_elementwise_bf16("dx", got["dx"], ref, dmag)
    errs["dW"] = rel_l2(got["dW"], g["dW"])
    errs["dscale"] = rel_l2(got["dscale"], g["dscale"])
    errs["dshift"] = rel_l2(got["dshift"], g["dshift"])
    if got.get("dres") is not None:
        assert np.array_equal(got["dres"], g["dres"]), "dres is not bit-exact"
        errs["dres"] = 0.0
    f32_out = ("dW", "dscale", "dshift")
    bad = {k: v for k, v in errs.items() if k != "mask_band" and v > (min(tol, TOL_F32_OUTPUTS) if k in f32_out else tol)}
    assert not bad, f"relative L2 above {tol}: {bad} (all: {errs})"
    return errs
