"""Pins of the CPU checker against facts that do not depend on it.

The paper gives no worked numbers for this path, so every pin is a closed form, an
invariant, a special case that reduces to a library routine (numpy matmul, torch's CPU
float64 conv2d + autograd), finite differences, or a hand-derived example stored under
tests/golden/.
"""
import os

import numpy as np
import pytest

from oracle import oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rng(seed):
    return np.random.default_rng(seed)


def rand_block(seed, N=2, H=7, W=6, C_in=3, C_out=4, KH=3, KW=3, stride=1, pad=1, relu=True, res=False):
    r = rng(seed)
    d = orc.Desc(N, H, W, C_in, C_out, KH, KW, stride, pad, relu)
    x = r.standard_normal((N, C_in, H, W))
    w = r.standard_normal((C_out, C_in, KH, KW)) * 0.3
    scale = 0.5 + r.random(C_out)
    shift = 0.1 * r.standard_normal(C_out)
    rs = r.standard_normal((N, C_out, d.Ho, d.Wo)) if res else None
    return d, x, w, scale, shift, rs


# ------------------------------------------------------------------ convolution forward
@pytest.mark.parametrize("H,W,KH,KW,stride,pad", [(5, 5, 3, 3, 1, 1), (7, 6, 3, 3, 2, 1), (9, 8, 7, 7, 2, 3),
                                                  (6, 7, 1, 1, 1, 0), (8, 8, 1, 1, 2, 0), (6, 5, 3, 2, 1, 1)])
def test_all_ones_counts_in_bounds_taps(H, W, KH, KW, stride, pad):
    C_in, C_out, N = 3, 2, 2
    d = orc.Desc(N, H, W, C_in, C_out, KH, KW, stride, pad, False)
    z = orc.conv(d, np.ones((N, C_in, H, W)), np.ones((C_out, C_in, KH, KW)))

    def count(o, size, k):
        lo = o * stride - pad
        return len([t for t in range(k) if 0 <= lo + t < size])

    expect = np.array([[count(ho, H, KH) * count(wo, W, KW) * C_in for wo in range(d.Wo)] for ho in range(d.Ho)],
                      dtype=np.float64)
    assert z.shape == (N, C_out, d.Ho, d.Wo)
    for n in range(N):
        for co in range(C_out):
            assert np.array_equal(z[n, co], expect)


@pytest.mark.parametrize("kh0,kw0", [(1, 1), (0, 0), (2, 1), (0, 2)])
def test_delta_weight_shifts_without_flip(kh0, kw0):
    """w = delta at tap (kh0,kw0) on the channel diagonal: z[ho,wo] = x[ho-p+kh0, wo-p+kw0]
    (cross-correlation: a flipped kernel would shift the other way)."""
    N, C, H, W, k, p = 2, 3, 6, 5, 3, 1
    d = orc.Desc(N, H, W, C, C, k, k, 1, p, False)
    x = rng(1).standard_normal((N, C, H, W))
    w = np.zeros((C, C, k, k))
    for c in range(C):
        w[c, c, kh0, kw0] = 1.0
    z = orc.conv(d, x, w)
    xp = np.pad(x, ((0, 0), (0, 0), (p, p), (p, p)))
    expect = xp[:, :, kh0:kh0 + H, kw0:kw0 + W]
    assert np.array_equal(z, expect)


def test_1x1_is_a_matrix_product():
    N, C_in, C_out, H, W = 3, 5, 7, 4, 6
    d = orc.Desc(N, H, W, C_in, C_out, 1, 1, 1, 0, False)
    r = rng(2)
    x = r.standard_normal((N, C_in, H, W))
    w = r.standard_normal((C_out, C_in, 1, 1))
    z = orc.conv(d, x, w)
    expect = np.einsum("oc,nchw->nohw", w[:, :, 0, 0], x)        # BLAS-backed contraction
    np.testing.assert_allclose(z, expect, rtol=1e-13, atol=1e-13)


def test_stride2_is_subsampled_stride1():
    d1, x, w, *_ = rand_block(3, H=9, W=11, stride=1, pad=1, relu=False)
    d2 = orc.Desc(d1.N, d1.H, d1.W, d1.C_in, d1.C_out, 3, 3, 2, 1, False)
    z1, z2 = orc.conv(d1, x, w), orc.conv(d2, x, w)
    assert np.array_equal(z2, z1[:, :, ::2, ::2][:, :, :d2.Ho, :d2.Wo])


def test_linearity_in_x_and_w():
    d, x, w, *_ = rand_block(4, stride=2, relu=False)
    r = rng(5)
    x2, w2 = r.standard_normal(x.shape), r.standard_normal(w.shape)
    np.testing.assert_allclose(orc.conv(d, 2 * x - 3 * x2, w), 2 * orc.conv(d, x, w) - 3 * orc.conv(d, x2, w),
                               rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(orc.conv(d, x, w + 0.5 * w2), orc.conv(d, x, w) + 0.5 * orc.conv(d, x, w2),
                               rtol=1e-12, atol=1e-12)


def test_translation_equivariance_in_the_interior():
    N, C, H, W = 1, 2, 12, 12
    d = orc.Desc(N, H, W, C, 3, 3, 3, 1, 1, False)
    r = rng(6)
    x = np.zeros((N, C, H, W))
    x[:, :, 3:7, 3:7] = r.standard_normal((N, C, 4, 4))
    w = r.standard_normal((3, C, 3, 3))
    z = orc.conv(d, x, w)
    zs = orc.conv(d, np.roll(x, (2, 3), axis=(2, 3)), w)
    np.testing.assert_allclose(zs, np.roll(z, (2, 3), axis=(2, 3)), rtol=0, atol=1e-14)


# ---------------------------------------------------------- affine / residual / ReLU
def test_identity_affine_no_flags_is_pure_conv():
    d, x, w, *_ = rand_block(7, relu=False)
    y = orc.block_fwd(d, x, w, np.ones(d.C_out), np.zeros(d.C_out))
    assert np.array_equal(y, orc.conv(d, x, w))


def test_relu_invariants_and_affine_per_channel():
    d, x, w, scale, shift, res = rand_block(8, res=True)
    y, z = orc.block_fwd(d, x, w, scale, shift, res, return_z=True)
    v = scale[None, :, None, None] * z + shift[None, :, None, None] + res
    assert np.all(y >= 0)
    assert np.array_equal(y == 0, v <= 0)
    assert np.array_equal(y[v > 0], v[v > 0])
    assert not np.any(np.signbit(y))
    dn = orc.Desc(d.N, d.H, d.W, d.C_in, d.C_out, d.KH, d.KW, d.stride, d.pad, False)
    assert np.array_equal(orc.block_fwd(dn, x, w, scale, shift, res), v)


def test_cancelling_residual_gives_zero():
    d, x, w, scale, shift, _ = rand_block(9)
    z = orc.conv(d, x, w)
    res = -(scale[None, :, None, None] * z + shift[None, :, None, None])
    assert np.array_equal(orc.block_fwd(d, x, w, scale, shift, res), np.zeros_like(z))


def test_hand_example_from_golden_file():
    vals = {}
    with open(os.path.join(GOLDEN, "hand_example_2x2.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            k, *v = line.split()
            vals[k] = np.array([float(t) for t in v])
    d = orc.Desc(1, 3, 3, 1, 1, 2, 2, 1, 0, True)
    x = np.arange(1.0, 10.0).reshape(1, 1, 3, 3)
    w = np.array([[1.0, 0.0], [0.0, -1.0]]).reshape(1, 1, 2, 2)
    scale, shift = np.array([2.0]), np.array([10.0])
    res = np.array([[-1.0, -2.0], [-3.0, 5.0]]).reshape(1, 1, 2, 2)
    y = orc.block_fwd(d, x, w, scale, shift, res)
    assert np.array_equal(y.ravel(), vals["y"])
    g = orc.block_bwd(d, np.ones((1, 1, 2, 2)), x, w, y, scale, need_dres=True)
    assert np.array_equal(g["dshift"], vals["dshift"])
    assert np.array_equal(g["dscale"], vals["dscale"])
    assert np.array_equal(g["dW"].ravel(), vals["dw"])
    assert np.array_equal(g["dx"].ravel(), vals["dx"])
    assert np.array_equal(g["dres"].ravel(), np.array([1.0, 0.0, 0.0, 1.0]))


# ------------------------------------------------------------------------- L1 loss
def test_l1_gradient_properties():
    r = rng(10)
    y, t = r.random((2, 3, 4, 5)), r.random((2, 3, 4, 5))
    t.flat[7] = y.flat[7]                                   # exercises sign(0) = 0
    dy = orc.l1_grad(y, t)
    inv = 1.0 / y.size
    assert dy.flat[7] == 0.0
    ne = y != t
    assert np.array_equal(np.abs(dy[ne]), np.full(ne.sum(), inv))
    assert np.array_equal(np.sign(dy), np.sign(y - t))
    assert np.abs(dy).sum() <= 1.0 + 1e-15
    assert abs(orc.l1_loss(y, t) - np.mean(np.abs(y - t))) < 1e-15


# ------------------------------------------------------------------------ backward
CASES = [dict(), dict(stride=2, H=9, W=8), dict(KH=1, KW=1, pad=0), dict(KH=1, KW=1, pad=0, stride=2, H=8, W=8),
         dict(KH=7, KW=7, pad=3, stride=2, H=11, W=10, C_in=3, C_out=2), dict(res=True), dict(relu=False),
         dict(KH=3, KW=2, pad=1, H=6, W=7)]


@pytest.mark.parametrize("kw", CASES)
def test_block_matches_library_conv_and_autograd(kw):
    """Special case "the whole block is a library routine": torch CPU float64 conv2d + autograd."""
    torch = pytest.importorskip("torch")
    d, x, w, scale, shift, res = rand_block(11, **kw)
    tx = torch.tensor(x, requires_grad=True)
    tw = torch.tensor(w, requires_grad=True)
    ts = torch.tensor(scale, requires_grad=True)
    tb = torch.tensor(shift, requires_grad=True)
    tz = torch.nn.functional.conv2d(tx, tw, None, stride=d.stride, padding=d.pad)
    tv = ts[None, :, None, None] * tz + tb[None, :, None, None]
    tr = None
    if res is not None:
        tr = torch.tensor(res, requires_grad=True)
        tv = tv + tr
    ty = torch.relu(tv) if d.relu else tv
    tt = torch.tensor(rng(12).random(tuple(ty.shape)))
    loss = torch.nn.functional.l1_loss(ty, tt)
    loss.backward()

    y = orc.block_fwd(d, x, w, scale, shift, res)
    np.testing.assert_allclose(y, ty.detach().numpy(), rtol=1e-12, atol=1e-12)
    assert abs(orc.l1_loss(y, tt.numpy()) - float(loss.detach())) < 1e-14
    dy = orc.l1_grad(y, tt.numpy())
    g = orc.block_bwd(d, dy, x, w, y, scale, need_dres=True)
    np.testing.assert_allclose(g["dx"], tx.grad.numpy(), rtol=1e-11, atol=1e-14)
    np.testing.assert_allclose(g["dW"], tw.grad.numpy(), rtol=1e-11, atol=1e-14)
    np.testing.assert_allclose(g["dscale"], ts.grad.numpy(), rtol=1e-11, atol=1e-14)
    np.testing.assert_allclose(g["dshift"], tb.grad.numpy(), rtol=1e-11, atol=1e-14)
    if tr is not None:
        np.testing.assert_allclose(g["dres"], tr.grad.numpy(), rtol=1e-12, atol=1e-15)


@pytest.mark.parametrize("kw", [dict(), dict(stride=2, H=9, W=8), dict(res=True), dict(KH=1, KW=1, pad=0)])
def test_central_finite_differences(kw):
    """d/dtheta of Phi = sum(dy * y) with dy frozen, for every parameter kind."""
    for seed in range(13, 1013, 100):          # first seed whose pre-activations all stay clear of 0
        d, x, w, scale, shift, res = rand_block(seed, **kw)
        y, z = orc.block_fwd(d, x, w, scale, shift, res, return_z=True)
        v = scale[None, :, None, None] * z + shift[None, :, None, None] + (res if res is not None else 0.0)
        if np.min(np.abs(v)) > 1e-3:           # no pre-activation changes sign under h = 1e-6
            break
    else:
        raise AssertionError("no seed keeps every pre-activation away from zero")
    r = rng(14)
    dy = r.standard_normal(y.shape)
    g = orc.block_bwd(d, dy, x, w, y, scale)

    def phi(x_, w_, s_, b_):
        return float(np.sum(dy * orc.block_fwd(d, x_, w_, s_, b_, res)))

    h = 1e-6
    for name, arr, grad in (("x", x, g["dx"]), ("W", w, g["dW"]), ("scale", scale, g["dscale"]),
                            ("shift", shift, g["dshift"])):
        for flat in r.choice(arr.size, size=min(6, arr.size), replace=False):
            hi, lo = arr.copy(), arr.copy()
            hi.flat[flat] += h
            lo.flat[flat] -= h
            args_hi = dict(x=x, W=w, scale=scale, shift=shift)
            args_lo = dict(args_hi)
            args_hi[name], args_lo[name] = hi, lo
            fd = (phi(args_hi["x"], args_hi["W"], args_hi["scale"], args_hi["shift"]) -
                  phi(args_lo["x"], args_lo["W"], args_lo["scale"], args_lo["shift"])) / (2 * h)
            assert abs(fd - grad.flat[flat]) <= 1e-7 * max(1.0, abs(fd)), (name, flat, fd, grad.flat[flat])


@pytest.mark.parametrize("kw", [dict(), dict(stride=2, H=10, W=9), dict(KH=7, KW=7, pad=3, stride=2, H=12, W=12)])
def test_adjoint_identities(kw):
    """<gs, conv(dx', w)> = <dx, dx'>  and  <gs, conv(x, dw')> = <dW, dw'>."""
    d, x, w, scale, shift, _ = rand_block(15, **kw)
    r = rng(16)
    y = orc.block_fwd(d, x, w, scale, shift)
    dy = r.standard_normal(y.shape)
    g = orc.block_bwd(d, dy, x, w, y, scale)
    gs = np.where(y > 0, dy, 0.0) * scale[None, :, None, None]
    px, pw = r.standard_normal(x.shape), r.standard_normal(w.shape)
    lhs_x, rhs_x = np.sum(gs * orc.conv(d, px, w)), np.sum(g["dx"] * px)
    lhs_w, rhs_w = np.sum(gs * orc.conv(d, x, pw)), np.sum(g["dW"] * pw)
    assert abs(lhs_x - rhs_x) <= 1e-11 * max(1.0, abs(lhs_x))
    assert abs(lhs_w - rhs_w) <= 1e-11 * max(1.0, abs(lhs_w))


def test_masked_gradient_is_exact_and_dscale_identity():
    d, x, w, scale, shift, res = rand_block(17, res=True)
    y = orc.block_fwd(d, x, w, scale, shift, res)
    dy = rng(18).standard_normal(y.shape)
    g = orc.block_bwd(d, dy, x, w, y, scale, need_dres=True)
    assert np.array_equal(g["dres"][y > 0], dy[y > 0])
    assert np.all(g["dres"][y == 0] == 0)
    # dscale[co] = sum_k w[co,k] * dW[co,k] / scale[co]
    ident = np.sum(w * g["dW"], axis=(1, 2, 3)) / scale
    np.testing.assert_allclose(g["dscale"], ident, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(g["dshift"], g["dres"].sum(axis=(0, 2, 3)), rtol=1e-12, atol=1e-14)


def test_bottleneck_chain_residual_routing():
    """Three chained blocks with an identity shortcut; W3 = 0 gives y3 = relu(shift3 + x) and the
    gradient that reaches x through the shortcut alone is g3."""
    r = rng(19)
    N, C, Cm, H = 2, 8, 4, 5
    x = r.standard_normal((N, C, H, H))
    d1 = orc.Desc(N, H, H, C, Cm, 1, 1, 1, 0, True)
    d2 = orc.Desc(N, H, H, Cm, Cm, 3, 3, 1, 1, True)
    d3 = orc.Desc(N, H, H, Cm, C, 1, 1, 1, 0, True)
    w1, w2 = r.standard_normal((Cm, C, 1, 1)), r.standard_normal((Cm, Cm, 3, 3))
    w3 = np.zeros((C, Cm, 1, 1))
    s = [0.5 + r.random(c) for c in (Cm, Cm, C)]
    b = [0.1 * r.standard_normal(c) for c in (Cm, Cm, C)]
    y1 = orc.block_fwd(d1, x, w1, s[0], b[0])
    y2 = orc.block_fwd(d2, y1, w2, s[1], b[1])
    y3 = orc.block_fwd(d3, y2, w3, s[2], b[2], x)
    assert np.array_equal(y3, np.maximum(b[2][None, :, None, None] + x, 0.0))
    dy3 = r.standard_normal(y3.shape)
    g3 = orc.block_bwd(d3, dy3, y2, w3, y3, s[2], need_dres=True)
    assert np.all(g3["dx"] == 0)
    g2 = orc.block_bwd(d2, g3["dx"], y1, w2, y2, s[1])
    g1 = orc.block_bwd(d1, g2["dx"], x, w1, y1, s[0])
    dx_total = g1["dx"] + g3["dres"]
    assert np.array_equal(dx_total, np.where(y3 > 0, dy3, 0.0))


# ------------------------------------------------------------------ single-output forms
@pytest.mark.parametrize("kw", [dict(res=True), dict(stride=2, H=9, W=8), dict(KH=1, KW=1, pad=0, stride=2, H=8, W=8)])
def test_point_functions_agree_with_full_loops(kw):
    d, x, w, scale, shift, res = rand_block(20, **kw)
    r = rng(21)
    y, z = orc.block_fwd(d, x, w, scale, shift, res, return_z=True)
    dy = r.standard_normal(y.shape)
    g = orc.block_bwd(d, dy, x, w, y, scale)

    def pts(shape, k=40):
        return np.stack([r.integers(0, s, size=k) for s in shape], axis=1)

    p = pts(y.shape)
    v, yy, mag = orc.fwd_points(d, x, w, scale, shift, res, p)
    np.testing.assert_allclose(yy, y[tuple(p.T)], rtol=1e-13, atol=1e-14)
    assert np.all(mag >= np.abs(v) - 1e-12)
    p = pts(x.shape)
    np.testing.assert_allclose(orc.dx_points(d, dy, y, w, scale, p), g["dx"][tuple(p.T)], rtol=1e-12, atol=1e-13)
    p = pts(w.shape)
    np.testing.assert_allclose(orc.dw_points(d, dy, y, x, scale, p), g["dW"][tuple(p.T)], rtol=1e-12, atol=1e-13)
    ch = np.arange(d.C_out)
    ds, db = orc.affine_grad_channels(d, dy, y, x, w, ch)
    np.testing.assert_allclose(ds, g["dscale"], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(db, g["dshift"], rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("kw", [dict(res=True), dict(stride=2, H=9, W=8, relu=True), dict(KH=7, KW=7, pad=3, stride=2, H=12, W=11),
                                dict(KH=1, KW=1, pad=0, stride=1, relu=False)])
def test_point_pre_activation_and_rounding_magnitude_against_library(kw):
    """The single-output forward returns the pre-activation v (negative ones included) and the magnitude
    |scale| * sum|x*w| + |shift| + |r| that sets the width of the rounding band in the full-size mask checks.
    Both are pinned to torch's CPU float64 conv2d: v on the signed operands, the magnitude as the same
    convolution of the absolute values (a magnitude that is too large would silently widen the band, one
    that is too small would flag legitimate roundings; >= |v| alone pins neither)."""
    torch = pytest.importorskip("torch")
    d, x, w, scale, shift, res = rand_block(24, **kw)
    r = rng(25)
    p = np.stack([r.integers(0, s, size=60) for s in (d.N, d.C_out, d.Ho, d.Wo)], axis=1)
    v, y, mag = orc.fwd_points(d, x, w, scale, shift, res, p)

    def tconv(a, b):
        return torch.nn.functional.conv2d(torch.tensor(a), torch.tensor(b), stride=d.stride, padding=d.pad).numpy()

    sc, sh = scale[None, :, None, None], shift[None, :, None, None]
    v_ref = sc * tconv(x, w) + sh + (res if res is not None else 0.0)
    mag_ref = np.abs(sc) * tconv(np.abs(x), np.abs(w)) + np.abs(sh) + (np.abs(res) if res is not None else 0.0)
    assert (v_ref[tuple(p.T)] < 0).any() and (v_ref[tuple(p.T)] > 0).any()
    np.testing.assert_allclose(v, v_ref[tuple(p.T)], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(mag, mag_ref[tuple(p.T)], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(y, np.maximum(v_ref, 0.0)[tuple(p.T)] if d.relu else v_ref[tuple(p.T)], rtol=1e-12, atol=1e-13)
    # a negative scale must enter the magnitude by its absolute value
    v2, _, mag2 = orc.fwd_points(d, x, w, -scale, shift, res, p)
    mag2_ref = np.abs(sc) * tconv(np.abs(x), np.abs(w)) + np.abs(sh) + (np.abs(res) if res is not None else 0.0)
    np.testing.assert_allclose(mag2, mag2_ref[tuple(p.T)], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(v2, (-sc * tconv(x, w) + sh + (res if res is not None else 0.0))[tuple(p.T)], rtol=1e-12, atol=1e-13)


def test_maxpool_matches_library():
    torch = pytest.importorskip("torch")
    x = rng(22).standard_normal((2, 3, 9, 10))
    y = orc.maxpool(x, 3, 2, 1)
    ty = torch.nn.functional.max_pool2d(torch.tensor(x), 3, 2, 1).numpy()
    assert np.array_equal(y, ty)


# ------------------------------------------------------------------- bf16 quantiser
def test_bf16_rounding_hand_cases():
    q = orc.bf16_rne
    assert q(1.0) == 1.0 and q(-0.0) == 0.0 and np.signbit(q(-0.0))
    assert q(1.0 + 2.0 ** -8) == 1.0                        # tie -> even (down)
    assert q(1.0 + 3 * 2.0 ** -8) == 1.0 + 2.0 ** -6        # tie -> even (up)
    assert q(1.0 + 2.0 ** -8 + 2.0 ** -40) == 1.0 + 2.0 ** -7   # just above a tie; float32 would lose it
    assert q(1.0 + 2.0 ** -9) == 1.0
    assert q(2.0 - 2.0 ** -9) == 2.0                        # carry into the exponent
    assert q(-(1.0 + 3 * 2.0 ** -8)) == -(1.0 + 2.0 ** -6)
    max_bf16 = (2.0 - 2.0 ** -7) * 2.0 ** 127
    assert q(max_bf16) == max_bf16
    assert q(max_bf16 * (1 + 2.0 ** -10)) == max_bf16
    assert np.isinf(q(2.0 ** 128 * (1 - 2.0 ** -12)))
    assert q(2.0 ** -133) == 2.0 ** -133 and q(2.0 ** -134) == 0.0 and q(3 * 2.0 ** -134) == 2.0 ** -132


def test_bf16_rounding_matches_library_cast_and_is_idempotent():
    torch = pytest.importorskip("torch")
    r = rng(23)
    a32 = np.concatenate([r.standard_normal(20000).astype(np.float32) * np.float32(10.0) ** r.integers(-20, 20, 20000),
                          np.float32(1.0) + np.arange(-300, 300, dtype=np.float32) * np.float32(2.0 ** -10)])
    a32 = a32.astype(np.float32)
    q = orc.quantize_bf16(a32.astype(np.float64))
    lib = torch.from_numpy(a32).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(q, lib)
    assert np.array_equal(orc.quantize_bf16(q), q)
