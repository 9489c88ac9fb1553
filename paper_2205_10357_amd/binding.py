"""ctypes binding of libsol_block.so: the same entry points as include/sol_block.h.

Argument marshalling only.  Every buffer argument may be a torch tensor (its
``data_ptr()`` is used), any object with ``data_ptr()``, or an integer device address.
There is no fallback: if the compiled library is missing, importing a symbol raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

SOL_F32, SOL_BF16 = 0, 1
SOL_RELU, SOL_DW_ACCUMULATE = 1, 2
SOL_PASS_FWD, SOL_PASS_BWD = 0, 1
SOL_PLAN_FWD, SOL_PLAN_DGRAD, SOL_PLAN_WGRAD = 0, 1, 2

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libsol_block.so")
EXPORTS = ("sol_block_fwd", "sol_block_bwd", "sol_block_workspace_bytes", "sol_status_string",
           "sol_l1_loss_grad", "sol_maxpool_fwd", "sol_block_set_plan", "sol_block_get_plan", "sol_clear_plans",
           "sol_reload_overrides", "sol_block_bwd_noalloc", "sol_block_bwd_noalloc_limit",
           "sol_sequence_create", "sol_sequence_destroy", "sol_sequence_length", "sol_sequence_add_fwd",
           "sol_sequence_add_bwd", "sol_sequence_add_l1_loss_grad", "sol_sequence_add_maxpool", "sol_sequence_run",
           "sol_trace_start", "sol_trace_tag", "sol_trace_stop", "sol_trace_kind_name")

_lib = None


class SolError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: status {status} ({sol_status_string(status)})")


class _CDesc(C.Structure):
    _fields_ = [("N", C.c_int32), ("H", C.c_int32), ("W", C.c_int32), ("C_in", C.c_int32),
                ("C_out", C.c_int32), ("KH", C.c_int32), ("KW", C.c_int32),
                ("stride", C.c_int32), ("pad", C.c_int32), ("dtype", C.c_int32), ("flags", C.c_uint32)]


class _CTraceEntry(C.Structure):
    _fields_ = [("kind", C.c_int32), ("tag", C.c_int32), ("us", C.c_float), ("start_us", C.c_float)]


class _CPlan(C.Structure):
    _fields_ = [("tile", C.c_int32), ("stages", C.c_int32), ("splits", C.c_int32)]


@dataclass(frozen=True)
class BlockDesc:
    N: int
    H: int
    W: int
    C_in: int
    C_out: int
    KH: int
    KW: int
    stride: int
    pad: int
    dtype: int = SOL_BF16
    flags: int = SOL_RELU

    @property
    def Ho(self) -> int:
        return (self.H + 2 * self.pad - self.KH) // self.stride + 1

    @property
    def Wo(self) -> int:
        return (self.W + 2 * self.pad - self.KW) // self.stride + 1

    def c(self) -> _CDesc:
        return _CDesc(self.N, self.H, self.W, self.C_in, self.C_out, self.KH, self.KW, self.stride,
                      self.pad, self.dtype, self.flags)


def lib():
    """Load the compiled library (raises if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with "
                               "`python -m paper_2205_10357_amd.build` (there is no fallback path)")
        l = C.CDLL(LIB_PATH)
        vp, fp = C.c_void_p, C.c_void_p
        l.sol_block_fwd.restype = C.c_int
        l.sol_block_fwd.argtypes = [C.POINTER(_CDesc), vp, vp, fp, fp, vp, vp, vp, C.c_size_t, vp]
        l.sol_block_bwd.restype = C.c_int
        l.sol_block_bwd.argtypes = [C.POINTER(_CDesc), vp, vp, vp, vp, vp, fp, fp, fp, fp, vp, vp, vp, vp, vp,
                                    C.c_size_t, vp]
        l.sol_block_bwd_noalloc.restype = C.c_int
        l.sol_block_bwd_noalloc.argtypes = [C.POINTER(_CDesc), vp, vp, vp, vp, vp, fp, fp, fp, fp, vp, vp, vp, vp, vp]
        l.sol_block_bwd_noalloc_limit.restype = C.c_size_t
        l.sol_block_bwd_noalloc_limit.argtypes = []
        i32 = C.c_int32
        l.sol_sequence_create.restype = vp
        l.sol_sequence_create.argtypes = []
        l.sol_sequence_destroy.restype = None
        l.sol_sequence_destroy.argtypes = [vp]
        l.sol_sequence_length.restype = i32
        l.sol_sequence_length.argtypes = [vp]
        l.sol_sequence_add_fwd.restype = C.c_int
        l.sol_sequence_add_fwd.argtypes = [vp, C.POINTER(_CDesc), vp, vp, fp, fp, vp, vp, vp, C.c_size_t, i32]
        l.sol_sequence_add_bwd.restype = C.c_int
        l.sol_sequence_add_bwd.argtypes = [vp, C.POINTER(_CDesc), vp, vp, vp, vp, vp, fp, fp, fp, fp, vp, vp, vp, vp, vp,
                                           C.c_size_t, i32]
        l.sol_sequence_add_l1_loss_grad.restype = C.c_int
        l.sol_sequence_add_l1_loss_grad.argtypes = [vp, i32, vp, vp, vp, C.c_int64, i32, i32]
        l.sol_sequence_add_maxpool.restype = C.c_int
        l.sol_sequence_add_maxpool.argtypes = [vp, i32, vp, vp] + [i32] * 8
        l.sol_sequence_run.restype = C.c_int
        l.sol_sequence_run.argtypes = [vp, i32, i32, vp]
        l.sol_trace_start.restype = C.c_int
        l.sol_trace_start.argtypes = [i32]
        l.sol_trace_tag.restype = None
        l.sol_trace_tag.argtypes = [i32]
        l.sol_trace_stop.restype = C.c_int
        l.sol_trace_stop.argtypes = [C.POINTER(_CTraceEntry), i32, C.POINTER(i32)]
        l.sol_trace_kind_name.restype = C.c_char_p
        l.sol_trace_kind_name.argtypes = [i32]
        l.sol_block_workspace_bytes.restype = C.c_size_t
        l.sol_block_workspace_bytes.argtypes = [C.POINTER(_CDesc), C.c_int]
        l.sol_status_string.restype = C.c_char_p
        l.sol_status_string.argtypes = [C.c_int]
        l.sol_l1_loss_grad.restype = C.c_int
        l.sol_l1_loss_grad.argtypes = [C.c_int32, vp, vp, vp, C.c_int64, C.c_int32, vp]
        l.sol_maxpool_fwd.restype = C.c_int
        l.sol_maxpool_fwd.argtypes = [C.c_int32, vp, vp] + [C.c_int32] * 7 + [vp]
        l.sol_block_set_plan.restype = C.c_int
        l.sol_block_set_plan.argtypes = [C.POINTER(_CDesc), C.c_int, C.POINTER(_CPlan)]
        l.sol_block_get_plan.restype = C.c_int
        l.sol_block_get_plan.argtypes = [C.POINTER(_CDesc), C.c_int, C.POINTER(_CPlan)]
        l.sol_clear_plans.restype = None
        l.sol_clear_plans.argtypes = []
        l.sol_reload_overrides.restype = None
        l.sol_reload_overrides.argtypes = []
        _lib = l
    return _lib


def _ptr(a) -> Optional[int]:
    if a is None:
        return None
    if isinstance(a, int):
        return a
    if hasattr(a, "data_ptr"):
        return int(a.data_ptr())
    raise TypeError(f"cannot take a device address from {type(a)!r}")


def _nbytes(a) -> int:
    if a is None:
        return 0
    return int(a.numel() * a.element_size())


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return int(torch.cuda.current_stream().cuda_stream) or None
    if isinstance(stream, int):
        return stream or None
    return int(stream.cuda_stream) or None


def _cdesc(desc) -> _CDesc:
    return desc.c() if isinstance(desc, BlockDesc) else desc


def sol_status_string(status: int) -> str:
    return lib().sol_status_string(int(status)).decode()


def sol_block_set_plan(desc, which: int, plan: Optional[tuple], check: bool = True) -> int:
    """plan: (tile, stages, splits) or None to remove the installed plan."""
    d = _cdesc(desc)
    if plan is None:
        st = lib().sol_block_set_plan(C.byref(d), int(which), None)
    else:
        cp = _CPlan(int(plan[0]), int(plan[1]), int(plan[2]))
        st = lib().sol_block_set_plan(C.byref(d), int(which), C.byref(cp))
    if check and st != 0:
        raise SolError(st, "sol_block_set_plan")
    return st


def sol_block_get_plan(desc, which: int) -> tuple:
    d, cp = _cdesc(desc), _CPlan()
    st = lib().sol_block_get_plan(C.byref(d), int(which), C.byref(cp))
    if st != 0:
        raise SolError(st, "sol_block_get_plan")
    return (cp.tile, cp.stages, cp.splits)


def sol_clear_plans() -> None:
    lib().sol_clear_plans()


def sol_reload_overrides() -> None:
    lib().sol_reload_overrides()


def sol_block_workspace_bytes(desc, pass_: int) -> int:
    d = _cdesc(desc)
    return int(lib().sol_block_workspace_bytes(C.byref(d), int(pass_)))


def sol_block_fwd(desc, x, W, scale, shift, residual, y, ws=None, ws_bytes: Optional[int] = None, stream=None,
                  check: bool = True) -> int:
    d = _cdesc(desc)
    nb = _nbytes(ws) if ws_bytes is None else ws_bytes
    st = lib().sol_block_fwd(C.byref(d), _ptr(x), _ptr(W), _ptr(scale), _ptr(shift), _ptr(residual), _ptr(y),
                             _ptr(ws), nb, _stream(stream))
    if check and st != 0:
        raise SolError(st, "sol_block_fwd")
    return st


def sol_block_bwd(desc, dy, x, W, y, dx, dW, dscale, dshift, scale, dres=None, dx_addend=None,
                  dx_addend_mask=None, dx_mask=None, ws=None, ws_bytes: Optional[int] = None, stream=None,
                  check: bool = True) -> int:
    d = _cdesc(desc)
    nb = _nbytes(ws) if ws_bytes is None else ws_bytes
    st = lib().sol_block_bwd(C.byref(d), _ptr(dy), _ptr(x), _ptr(W), _ptr(y), _ptr(dx), _ptr(dW), _ptr(dscale),
                             _ptr(dshift), _ptr(scale), _ptr(dres), _ptr(dx_addend), _ptr(dx_addend_mask),
                             _ptr(dx_mask), _ptr(ws), nb, _stream(stream))
    if check and st != 0:
        raise SolError(st, "sol_block_bwd")
    return st


def sol_block_bwd_noalloc(desc, dy, x, W, y, dx, dW, dscale, dshift, scale, dres=None, dx_addend=None,
                          dx_addend_mask=None, dx_mask=None, stream=None, check: bool = True) -> int:
    d = _cdesc(desc)
    st = lib().sol_block_bwd_noalloc(C.byref(d), _ptr(dy), _ptr(x), _ptr(W), _ptr(y), _ptr(dx), _ptr(dW),
                                     _ptr(dscale), _ptr(dshift), _ptr(scale), _ptr(dres), _ptr(dx_addend),
                                     _ptr(dx_addend_mask), _ptr(dx_mask), _stream(stream))
    if check and st != 0:
        raise SolError(st, "sol_block_bwd_noalloc")
    return st


def sol_block_bwd_noalloc_limit() -> int:
    return int(lib().sol_block_bwd_noalloc_limit())


def sol_l1_loss_grad(dtype: int, y, t, dy, numel: int, mask_by_y: bool = False, stream=None,
                     check: bool = True) -> int:
    st = lib().sol_l1_loss_grad(int(dtype), _ptr(y), _ptr(t), _ptr(dy), int(numel), int(bool(mask_by_y)),
                                _stream(stream))
    if check and st != 0:
        raise SolError(st, "sol_l1_loss_grad")
    return st


def sol_maxpool_fwd(dtype: int, x, y, N: int, H: int, W: int, Cc: int, k: int, stride: int, pad: int, stream=None,
                    check: bool = True) -> int:
    st = lib().sol_maxpool_fwd(int(dtype), _ptr(x), _ptr(y), N, H, W, Cc, k, stride, pad, _stream(stream))
    if check and st != 0:
        raise SolError(st, "sol_maxpool_fwd")
    return st


class Sequence:
    """A prepared list of block calls (sol_sequence_*): record once, run with one call per pass."""

    def __init__(self):
        self._h = lib().sol_sequence_create()
        if not self._h:
            raise MemoryError("sol_sequence_create")
        self._keep = []                      # the recorded buffers must outlive the runs

    def __del__(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.sol_sequence_destroy(self._h)
            self._h = None

    def __len__(self) -> int:
        return int(lib().sol_sequence_length(self._h))

    def _ok(self, st: int, where: str) -> None:
        if st != 0:
            raise SolError(st, where)

    def add_fwd(self, desc, x, W, scale, shift, residual, y, ws=None, ws_bytes: Optional[int] = None, tag: int = 0):
        d = _cdesc(desc)
        nb = _nbytes(ws) if ws_bytes is None else ws_bytes
        self._keep.append((x, W, scale, shift, residual, y, ws))
        self._ok(lib().sol_sequence_add_fwd(self._h, C.byref(d), _ptr(x), _ptr(W), _ptr(scale), _ptr(shift),
                                            _ptr(residual), _ptr(y), _ptr(ws), nb, int(tag)), "sol_sequence_add_fwd")

    def add_bwd(self, desc, dy, x, W, y, dx, dW, dscale, dshift, scale, dres=None, dx_addend=None,
                dx_addend_mask=None, dx_mask=None, ws=None, ws_bytes: Optional[int] = None, tag: int = 0):
        d = _cdesc(desc)
        nb = _nbytes(ws) if ws_bytes is None else ws_bytes
        self._keep.append((dy, x, W, y, dx, dW, dscale, dshift, scale, dres, dx_addend, dx_addend_mask, dx_mask, ws))
        self._ok(lib().sol_sequence_add_bwd(self._h, C.byref(d), _ptr(dy), _ptr(x), _ptr(W), _ptr(y), _ptr(dx),
                                            _ptr(dW), _ptr(dscale), _ptr(dshift), _ptr(scale), _ptr(dres),
                                            _ptr(dx_addend), _ptr(dx_addend_mask), _ptr(dx_mask), _ptr(ws), nb,
                                            int(tag)), "sol_sequence_add_bwd")

    def add_l1_loss_grad(self, dtype: int, y, t, dy, numel: int, mask_by_y: bool = False, tag: int = 0):
        self._keep.append((y, t, dy))
        self._ok(lib().sol_sequence_add_l1_loss_grad(self._h, int(dtype), _ptr(y), _ptr(t), _ptr(dy), int(numel),
                                                     int(bool(mask_by_y)), int(tag)), "sol_sequence_add_l1_loss_grad")

    def add_maxpool(self, dtype: int, x, y, N: int, H: int, W: int, Cc: int, k: int, stride: int, pad: int,
                    tag: int = 0):
        self._keep.append((x, y))
        self._ok(lib().sol_sequence_add_maxpool(self._h, int(dtype), _ptr(x), _ptr(y), N, H, W, Cc, k, stride, pad,
                                                int(tag)), "sol_sequence_add_maxpool")

    def run(self, first: int = 0, count: Optional[int] = None, stream=None, check: bool = True) -> int:
        n = len(self) - first if count is None else count
        st = lib().sol_sequence_run(self._h, int(first), int(n), _stream(stream))
        if check and st != 0:
            raise SolError(st, "sol_sequence_run")
        return st


def sol_trace_start(capacity: int = 4096) -> None:
    st = lib().sol_trace_start(int(capacity))
    if st != 0:
        raise SolError(st, "sol_trace_start")


def sol_trace_tag(tag: int) -> None:
    lib().sol_trace_tag(int(tag))


def sol_trace_stop(capacity: int = 4096):
    """-> list of (kind, tag, execution microseconds, start microseconds since the first launch) in launch order."""
    buf = (_CTraceEntry * capacity)()
    n = C.c_int32(0)
    st = lib().sol_trace_stop(buf, int(capacity), C.byref(n))
    if st != 0:
        raise SolError(st, "sol_trace_stop")
    return [(int(buf[i].kind), int(buf[i].tag), float(buf[i].us), float(buf[i].start_us))
            for i in range(min(n.value, capacity))]


def sol_trace_kind_name(kind: int) -> str:
    return lib().sol_trace_kind_name(int(kind)).decode()
