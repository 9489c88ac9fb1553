"""ctypes front-end of the CPU checker in oracle.c (test infrastructure only).

All arrays are C-contiguous float64; activations ``[N, C, H, W]``, weights
``[C_out, C_in, KH, KW]``.  The functions only marshal arguments: the arithmetic is the
plain loops in oracle.c, which follow the block definition implied by steps 1-3 of the
paper's training loop (section "SOL principle").
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import numpy as np

from . import build as _build

_LIB = None


class _Desc(C.Structure):
    _fields_ = [(k, C.c_int) for k in
                ("N", "H", "W", "C_in", "C_out", "KH", "KW", "stride", "pad", "relu")]


@dataclass(frozen=True)
class Desc:
    N: int
    H: int
    W: int
    C_in: int
    C_out: int
    KH: int
    KW: int
    stride: int
    pad: int
    relu: bool

    @property
    def Ho(self) -> int:
        return (self.H + 2 * self.pad - self.KH) // self.stride + 1

    @property
    def Wo(self) -> int:
        return (self.W + 2 * self.pad - self.KW) // self.stride + 1

    def c(self) -> _Desc:
        return _Desc(self.N, self.H, self.W, self.C_in, self.C_out, self.KH, self.KW,
                     self.stride, self.pad, int(self.relu))


_DP = C.POINTER(C.c_double)
_IP = C.POINTER(C.c_int)


def lib():
    global _LIB
    if _LIB is None:
        path = _build.LIB
        if (not os.path.exists(path)) or os.path.getmtime(path) < os.path.getmtime(_build.SRC):
            _build.build()
        _LIB = C.CDLL(path)
        _LIB.orc_bf16_rne.restype = C.c_double
        _LIB.orc_bf16_rne.argtypes = [C.c_double]
        _LIB.orc_l1_loss.restype = C.c_double
        _LIB.orc_now.restype = C.c_double
        _LIB.orc_num_threads.restype = C.c_int
    return _LIB


def _p(a: Optional[np.ndarray]):
    if a is None:
        return None
    assert a.dtype == np.float64 and a.flags.c_contiguous
    return a.ctypes.data_as(_DP)


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _idx(idx) -> np.ndarray:
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    assert idx.ndim == 2 and idx.shape[1] == 4
    return idx


def num_threads() -> int:
    return int(lib().orc_num_threads())


def conv(d: Desc, x, w) -> np.ndarray:
    x, w = _f64(x), _f64(w)
    assert x.shape == (d.N, d.C_in, d.H, d.W) and w.shape == (d.C_out, d.C_in, d.KH, d.KW)
    z = np.empty((d.N, d.C_out, d.Ho, d.Wo))
    dc = d.c()
    lib().orc_conv(C.byref(dc), _p(x), _p(w), _p(z))
    return z


def block_fwd(d: Desc, x, w, scale, shift, res=None, return_z: bool = False):
    x, w, scale, shift = _f64(x), _f64(w), _f64(scale), _f64(shift)
    assert x.shape == (d.N, d.C_in, d.H, d.W) and w.shape == (d.C_out, d.C_in, d.KH, d.KW)
    assert scale.shape == (d.C_out,) and shift.shape == (d.C_out,)
    y = np.empty((d.N, d.C_out, d.Ho, d.Wo))
    z = np.empty_like(y) if return_z else None
    if res is not None:
        res = _f64(res)
        assert res.shape == y.shape
    dc = d.c()
    lib().orc_block_fwd(C.byref(dc), _p(x), _p(w), _p(scale), _p(shift), _p(res), _p(z), _p(y))
    return (y, z) if return_z else y


def l1_loss(y, t) -> float:
    y, t = _f64(y), _f64(t)
    assert y.shape == t.shape
    return float(lib().orc_l1_loss(_p(y), _p(t), C.c_long(y.size)))


def l1_grad(y, t) -> np.ndarray:
    y, t = _f64(y), _f64(t)
    assert y.shape == t.shape
    dy = np.empty_like(y)
    lib().orc_l1_grad(_p(y), _p(t), C.c_long(y.size), _p(dy))
    return dy


def block_bwd(d: Desc, dy, x, w, y, scale, need_dx: bool = True, need_dres: bool = False):
    """Returns dict(dx, dW, dscale, dshift, dres); dx / dres are None when not requested."""
    dy, x, w, y, scale = _f64(dy), _f64(x), _f64(w), _f64(y), _f64(scale)
    assert x.shape == (d.N, d.C_in, d.H, d.W) and w.shape == (d.C_out, d.C_in, d.KH, d.KW)
    assert dy.shape == (d.N, d.C_out, d.Ho, d.Wo) and y.shape == dy.shape
    dx = np.empty_like(x) if need_dx else None
    dres = np.empty_like(dy) if need_dres else None
    dw = np.empty_like(w)
    dscale, dshift = np.empty(d.C_out), np.empty(d.C_out)
    dc = d.c()
    lib().orc_block_bwd(C.byref(dc), _p(dy), _p(x), _p(w), _p(y), _p(scale), _p(dx), _p(dw),
                        _p(dscale), _p(dshift), _p(dres))
    return {"dx": dx, "dW": dw, "dscale": dscale, "dshift": dshift, "dres": dres}


def maxpool(x, k: int = 3, stride: int = 2, pad: int = 1) -> np.ndarray:
    x = _f64(x)
    n, c, h, w = x.shape
    ho, wo = (h + 2 * pad - k) // stride + 1, (w + 2 * pad - k) // stride + 1
    y = np.empty((n, c, ho, wo))
    lib().orc_maxpool(n, c, h, w, k, stride, pad, _p(x), _p(y))
    return y


def bf16_rne(v: float) -> float:
    return float(lib().orc_bf16_rne(C.c_double(v)))


def quantize_bf16(a) -> np.ndarray:
    a = _f64(a)
    out = np.empty_like(a)
    lib().orc_quantize_bf16(_p(a), _p(out), C.c_long(a.size))
    return out


def fwd_points(d: Desc, x, w, scale, shift, res, idx):
    """idx rows (n, co, ho, wo) -> (v, y, magnitude)."""
    x, w, scale, shift = _f64(x), _f64(w), _f64(scale), _f64(shift)
    assert x.shape == (d.N, d.C_in, d.H, d.W) and w.shape == (d.C_out, d.C_in, d.KH, d.KW)
    if res is not None:
        res = _f64(res)
        assert res.shape == (d.N, d.C_out, d.Ho, d.Wo)
    idx = _idx(idx)
    n = idx.shape[0]
    v, y, mag = np.empty(n), np.empty(n), np.empty(n)
    dc = d.c()
    lib().orc_fwd_points(C.byref(dc), _p(x), _p(w), _p(scale), _p(shift), _p(res), C.c_long(n),
                         idx.ctypes.data_as(_IP), _p(v), _p(y), _p(mag))
    return v, y, mag


def dx_points(d: Desc, dy, y, w, scale, idx) -> np.ndarray:
    """idx rows (n, ci, hi, wi)."""
    dy, y, w, scale = _f64(dy), _f64(y), _f64(w), _f64(scale)
    assert dy.shape == (d.N, d.C_out, d.Ho, d.Wo) and y.shape == dy.shape
    idx = _idx(idx)
    out = np.empty(idx.shape[0])
    dc = d.c()
    lib().orc_dx_points(C.byref(dc), _p(dy), _p(y), _p(w), _p(scale), C.c_long(idx.shape[0]),
                        idx.ctypes.data_as(_IP), _p(out))
    return out


def dw_points(d: Desc, dy, y, x, scale, idx) -> np.ndarray:
    """idx rows (co, ci, kh, kw)."""
    dy, y, x, scale = _f64(dy), _f64(y), _f64(x), _f64(scale)
    assert dy.shape == (d.N, d.C_out, d.Ho, d.Wo) and x.shape == (d.N, d.C_in, d.H, d.W)
    idx = _idx(idx)
    out = np.empty(idx.shape[0])
    dc = d.c()
    lib().orc_dw_points(C.byref(dc), _p(dy), _p(y), _p(x), _p(scale), C.c_long(idx.shape[0]),
                        idx.ctypes.data_as(_IP), _p(out))
    return out


def affine_grad_channels(d: Desc, dy, y, x, w, channels):
    """(dscale, dshift) of the listed output channels."""
    dy, y, x, w = _f64(dy), _f64(y), _f64(x), _f64(w)
    ch = np.ascontiguousarray(channels, dtype=np.int32)
    ds, db = np.empty(ch.size), np.empty(ch.size)
    dc = d.c()
    lib().orc_affine_grad_channels(C.byref(dc), _p(dy), _p(y), _p(x), _p(w), C.c_long(ch.size),
                                   ch.ctypes.data_as(_IP), _p(ds), _p(db))
    return ds, db


def now() -> float:
    return float(lib().orc_now())
