"""Thin ctypes binding of libfno.so: argument marshalling only.

Every function has the name of the C entry point it calls (include/fno.h) and hands it the
device pointers of torch tensors; all arithmetic happens in the HIP kernels.  torch is used
for device memory and the current stream, nothing else.  If libfno.so is missing the first
call raises: there is no fallback.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfno.so")

FNO_OK, FNO_EINVAL, FNO_EUNSUPPORTED, FNO_ENOSPC, FNO_EHIP = 0, -1, -2, -3, -4
FNO_ACT_IDENTITY, FNO_ACT_GELU = 0, 1
FNO_OP_SPECTRAL_CONV_FWD, FNO_OP_SPECTRAL_CONV_BWD, FNO_OP_BLOCK_FWD, FNO_OP_BLOCK_BWD = 0, 1, 2, 3
FNO_FLAG_MSE_TARGET = 1
FNO_FLAG_ACCUMULATE_GRADS = 2
FNO_FLAG_TABLES_READY = 4
FNO_STATIC_SCRATCH_BYTES = 64 << 20

EXPORTS = [
    "fno_workspace_bytes", "fno_plan_tables", "fno_mode_indices", "fno_spectral_conv_fwd", "fno_spectral_conv_bwd",
    "fno_block_fwd", "fno_block_bwd", "fno_pointwise_linear", "fno_pointwise_mlp2", "fno_time_lift",
    "fno_rel_l2_workspace_bytes", "fno_rel_l2_loss", "fno_adam_step",
    "fno_pointwise_bwd_workspace_bytes", "fno_pointwise_linear_bwd", "fno_pointwise_mlp2_bwd",
    "fno_time_lift_bwd_workspace_bytes", "fno_time_lift_bwd",
    "fno_spectral_conv_fwd_static",
    "fno_status_string", "fno_timing_enable", "fno_timing_read",
]

STAGE_NAMES = ["tz_fwd", "y_fwd", "x_fwd", "mix", "x_inv", "y_inv", "zt_inv", "mix_bwd", "bwd_pointwise"]


class FnoDesc(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("c_in", ctypes.c_int32), ("c_out", ctypes.c_int32),
                ("grid", ctypes.c_int32 * 4), ("modes", ctypes.c_int32 * 4),
                ("mode_rule", ctypes.c_int32), ("activation", ctypes.c_int32),
                ("flags", ctypes.c_int32)]


class FnoError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"libfno status {status}: {text}")
        self.status = status


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()')")
        l = ctypes.CDLL(LIB_PATH)
        l.fno_status_string.restype = ctypes.c_char_p
        l.fno_status_string.argtypes = [ctypes.c_int]
        for name in EXPORTS:
            if name != "fno_status_string":
                getattr(l, name).restype = ctypes.c_int
        _lib = l
    return _lib


def make_desc(batch: int, c_in: int, c_out: int, grid: Sequence[int], modes: Sequence[int],
              mode_rule: int = 0, activation: int = FNO_ACT_GELU, flags: int = 0) -> FnoDesc:
    return FnoDesc(batch, c_in, c_out, (ctypes.c_int32 * 4)(*grid), (ctypes.c_int32 * 4)(*modes),
                   mode_rule, activation, flags)


def _check(status: int) -> None:
    if status != FNO_OK:
        raise FnoError(status, lib().fno_status_string(status).decode())


def _ptr(t: Optional[torch.Tensor], dtype=torch.float32, name: str = "tensor"):
    if t is None:
        return ctypes.c_void_p(0)
    if not t.is_cuda:
        raise ValueError(f"{name} must live on the GPU")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    want = (dtype, torch.complex64) if dtype == torch.float32 else (dtype,)
    if t.dtype not in want:
        raise ValueError(f"{name} has dtype {t.dtype}")
    return ctypes.c_void_p(t.data_ptr())


def _sizes(desc: FnoDesc):
    """(grid points, kept modes) per (batch, channel) slab, from the library's own mode lists."""
    npts = 1
    for n in desc.grid:
        npts *= int(n)
    kept = 1
    for axis in range(4):
        n = ctypes.c_int32(0)
        _check(lib().fno_mode_indices(ctypes.byref(desc), ctypes.c_int(axis), None, ctypes.byref(n)))
        kept *= int(n.value)
    return npts, kept


def _expect(t: Optional[torch.Tensor], name: str, numel: int) -> None:
    """A tensor handed to the kernels must hold exactly the elements the descriptor implies: the
    kernels index by the descriptor alone, and a short buffer would be read or written out of bounds."""
    if t is None:
        return
    have = t.numel() * (2 if t.dtype == torch.complex64 else 1)
    if have != numel:
        raise ValueError(f"{name} holds {have} floats, the descriptor implies {numel}")


def _check_layer_tensors(desc, *, x=None, y=None, R=None, xhat=None, W=None, b=None, extra_in=(), extra_out=()):
    npts, kept = _sizes(desc)
    B_, ci, co = int(desc.batch), int(desc.c_in), int(desc.c_out)
    _expect(x, "x", B_ * ci * npts)
    _expect(y, "output", B_ * co * npts)
    _expect(R, "R", 2 * ci * co * kept)
    _expect(xhat, "xhat", 2 * B_ * ci * kept)
    _expect(W, "W", co * ci)
    _expect(b, "b", co)
    for name, t in extra_in:
        _expect(t, name, B_ * ci * npts)
    for name, t in extra_out:
        _expect(t, name, B_ * co * npts)


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def fno_status_string(status: int) -> str:
    return lib().fno_status_string(status).decode()


def fno_workspace_bytes(desc: FnoDesc, op: int) -> int:
    n = ctypes.c_size_t(0)
    _check(lib().fno_workspace_bytes(ctypes.byref(desc), ctypes.c_int(op), ctypes.byref(n)))
    return int(n.value)


def fno_plan_tables(desc: FnoDesc, op: int, ws) -> None:
    p, n = _ws(ws)
    _check(lib().fno_plan_tables(ctypes.byref(desc), ctypes.c_int(op), p, n, _stream()))


def fno_mode_indices(desc: FnoDesc, axis: int) -> list[int]:
    n = ctypes.c_int32(0)
    _check(lib().fno_mode_indices(ctypes.byref(desc), ctypes.c_int(axis), None, ctypes.byref(n)))
    buf = (ctypes.c_int32 * max(n.value, 1))()
    _check(lib().fno_mode_indices(ctypes.byref(desc), ctypes.c_int(axis), buf, ctypes.byref(n)))
    return [int(buf[i]) for i in range(n.value)]


def kept_counts(desc: FnoDesc) -> tuple:
    """Number of kept modes per axis (x, y, z, t): the lengths of the library's mode lists."""
    return tuple(len(fno_mode_indices(desc, axis)) for axis in range(4))


def alloc_workspace(desc: FnoDesc, op: int, device="cuda") -> torch.Tensor:
    """A byte tensor of the size the op asks for (torch allocations are 256-byte aligned)."""
    return torch.empty(max(fno_workspace_bytes(desc, op), 256), dtype=torch.uint8, device=device)


def _ws(ws: torch.Tensor):
    if not ws.is_cuda or ws.dtype != torch.uint8:
        raise ValueError("workspace must be a uint8 GPU tensor")
    return ctypes.c_void_p(ws.data_ptr()), ctypes.c_size_t(ws.numel())


def fno_spectral_conv_fwd(desc, x, R, y, xhat_save, ws) -> None:
    _check_layer_tensors(desc, x=x, y=y, R=R, xhat=xhat_save)
    p, n = _ws(ws)
    _check(lib().fno_spectral_conv_fwd(ctypes.byref(desc), _ptr(x, name="x"), _ptr(R, name="R"),
                                       _ptr(y, name="y"), _ptr(xhat_save, name="xhat_save"),
                                       p, n, _stream()))


def fno_spectral_conv_fwd_static(desc, x, R, y, xhat_save) -> None:
    _check_layer_tensors(desc, x=x, y=y, R=R, xhat=xhat_save)
    _check(lib().fno_spectral_conv_fwd_static(ctypes.byref(desc), _ptr(x, name="x"), _ptr(R, name="R"),
                                              _ptr(y, name="y"), _ptr(xhat_save, name="xhat_save"),
                                              _stream()))


def fno_spectral_conv_bwd(desc, x, xhat_saved, R, gy, gx, gR, ws) -> None:
    _check_layer_tensors(desc, x=x, y=gy, R=R, xhat=xhat_saved, extra_in=(("gx", gx),))
    _expect(gR, "gR", R.numel() * 2 if R is not None else 0)
    p, n = _ws(ws)
    _check(lib().fno_spectral_conv_bwd(ctypes.byref(desc), _ptr(x, name="x"),
                                       _ptr(xhat_saved, name="xhat_saved"), _ptr(R, name="R"),
                                       _ptr(gy, name="gy"), _ptr(gx, name="gx"), _ptr(gR, name="gR"),
                                       p, n, _stream()))


def fno_block_fwd(desc, x, R, W, b, out, z_save, xhat_save, ws) -> None:
    _check_layer_tensors(desc, x=x, y=out, R=R, xhat=xhat_save, W=W, b=b, extra_out=(("z_save", z_save),))
    p, n = _ws(ws)
    _check(lib().fno_block_fwd(ctypes.byref(desc), _ptr(x, name="x"), _ptr(R, name="R"),
                               _ptr(W, name="W"), _ptr(b, name="b"), _ptr(out, name="out"),
                               _ptr(z_save, name="z_save"), _ptr(xhat_save, name="xhat_save"),
                               p, n, _stream()))


def fno_block_bwd(desc, x, R, W, z_saved, xhat_saved, gout, gx, gR, gW, gb, ws) -> None:
    _check_layer_tensors(desc, x=x, y=gout, R=R, xhat=xhat_saved, W=W, b=gb,
                         extra_in=(("gx", gx),), extra_out=(("z_saved", z_saved),))
    _expect(gR, "gR", R.numel() * 2 if R is not None else 0)
    _expect(gW, "gW", W.numel() if W is not None else 0)
    p, n = _ws(ws)
    _check(lib().fno_block_bwd(ctypes.byref(desc), _ptr(x, name="x"), _ptr(R, name="R"),
                               _ptr(W, name="W"), _ptr(z_saved, name="z_saved"),
                               _ptr(xhat_saved, name="xhat_saved"), _ptr(gout, name="gout"),
                               _ptr(gx, name="gx"), _ptr(gR, name="gR"), _ptr(gW, name="gW"),
                               _ptr(gb, name="gb"), p, n, _stream()))


def fno_pointwise_linear(batch, c_in, c_out, npoints, x, W, bias, y) -> None:
    _check(lib().fno_pointwise_linear(ctypes.c_int32(batch), ctypes.c_int32(c_in), ctypes.c_int32(c_out),
                                      ctypes.c_int64(npoints), _ptr(x, name="x"), _ptr(W, name="W"),
                                      _ptr(bias, name="bias"), _ptr(y, name="y"), _stream()))


def fno_time_lift(batch, c_in, c_out, nspace, nt, a, Wt, bt, Wc, bc, out) -> None:
    _check(lib().fno_time_lift(ctypes.c_int32(batch), ctypes.c_int32(c_in), ctypes.c_int32(c_out),
                               ctypes.c_int64(nspace), ctypes.c_int32(nt), _ptr(a, name="a"),
                               _ptr(Wt, name="Wt"), _ptr(bt, name="bt"), _ptr(Wc, name="Wc"),
                               _ptr(bc, name="bc"), _ptr(out, name="out"), _stream()))


def fno_time_lift_bwd_workspace_bytes(c_in, c_out, nt) -> int:
    n = ctypes.c_size_t(0)
    _check(lib().fno_time_lift_bwd_workspace_bytes(ctypes.c_int32(c_in), ctypes.c_int32(c_out), ctypes.c_int32(nt),
                                                   ctypes.byref(n)))
    return int(n.value)


def fno_time_lift_bwd(batch, c_in, c_out, nspace, nt, a, Wt, bt, Wc, g, gWt, gbt, gWc, gbc, ws) -> None:
    _check(lib().fno_time_lift_bwd(ctypes.c_int32(batch), ctypes.c_int32(c_in), ctypes.c_int32(c_out),
                                   ctypes.c_int64(nspace), ctypes.c_int32(nt), _ptr(a, name="a"),
                                   _ptr(Wt, name="Wt"), _ptr(bt, name="bt"), _ptr(Wc, name="Wc"),
                                   _ptr(g, name="g"), _ptr(gWt, name="gWt"), _ptr(gbt, name="gbt"),
                                   _ptr(gWc, name="gWc"), _ptr(gbc, name="gbc"), _ptr(ws, name="ws"),
                                   ctypes.c_size_t(ws.numel() * ws.element_size()), _stream()))


def fno_pointwise_bwd_workspace_bytes(c_in, hidden, c_out) -> int:
    n = ctypes.c_size_t(0)
    _check(lib().fno_pointwise_bwd_workspace_bytes(ctypes.c_int32(c_in), ctypes.c_int32(hidden),
                                                   ctypes.c_int32(c_out), ctypes.byref(n)))
    return int(n.value)


def fno_pointwise_linear_bwd(batch, c_in, c_out, npoints, x, W, g, gx, gW, gb, ws) -> None:
    _check(lib().fno_pointwise_linear_bwd(ctypes.c_int32(batch), ctypes.c_int32(c_in), ctypes.c_int32(c_out),
                                          ctypes.c_int64(npoints), _ptr(x, name="x"), _ptr(W, name="W"),
                                          _ptr(g, name="g"), _ptr(gx, name="gx"), _ptr(gW, name="gW"),
                                          _ptr(gb, name="gb"), _ptr(ws, name="ws"),
                                          ctypes.c_size_t(ws.numel() * ws.element_size()), _stream()))


def fno_pointwise_mlp2_bwd(batch, c_in, hidden, c_out, npoints, x, W1, b1, W2, g, gx, gW1, gb1, gW2, gb2, ws) -> None:
    _check(lib().fno_pointwise_mlp2_bwd(ctypes.c_int32(batch), ctypes.c_int32(c_in), ctypes.c_int32(hidden),
                                        ctypes.c_int32(c_out), ctypes.c_int64(npoints), _ptr(x, name="x"),
                                        _ptr(W1, name="W1"), _ptr(b1, name="b1"), _ptr(W2, name="W2"),
                                        _ptr(g, name="g"), _ptr(gx, name="gx"), _ptr(gW1, name="gW1"),
                                        _ptr(gb1, name="gb1"), _ptr(gW2, name="gW2"), _ptr(gb2, name="gb2"),
                                        _ptr(ws, name="ws"), ctypes.c_size_t(ws.numel() * ws.element_size()),
                                        _stream()))


def fno_rel_l2_workspace_bytes() -> int:
    n = ctypes.c_size_t(0)
    _check(lib().fno_rel_l2_workspace_bytes(ctypes.byref(n)))
    return int(n.value)


def fno_rel_l2_loss(n, pred, target, loss, grad, ws) -> None:
    _check(lib().fno_rel_l2_loss(ctypes.c_int64(n), _ptr(pred, name="pred"), _ptr(target, name="target"),
                                 _ptr(loss, name="loss"), _ptr(grad, name="grad"), _ptr(ws, name="ws"),
                                 ctypes.c_size_t(ws.numel() * ws.element_size()), _stream()))


def fno_adam_step(n, param, grad, m, v, lr, beta1, beta2, eps, step) -> None:
    _check(lib().fno_adam_step(ctypes.c_int64(n), _ptr(param, name="param"), _ptr(grad, name="grad"),
                               _ptr(m, name="m"), _ptr(v, name="v"), ctypes.c_double(lr), ctypes.c_double(beta1),
                               ctypes.c_double(beta2), ctypes.c_double(eps), ctypes.c_int32(step), _stream()))


def fno_pointwise_mlp2(batch, c_in, hidden, c_out, npoints, x, W1, b1, W2, b2, y) -> None:
    _check(lib().fno_pointwise_mlp2(ctypes.c_int32(batch), ctypes.c_int32(c_in), ctypes.c_int32(hidden),
                                    ctypes.c_int32(c_out), ctypes.c_int64(npoints), _ptr(x, name="x"),
                                    _ptr(W1, name="W1"), _ptr(b1, name="b1"), _ptr(W2, name="W2"),
                                    _ptr(b2, name="b2"), _ptr(y, name="y"), _stream()))


FNO_TIMING_ALL = -1


def fno_timing_enable(stages) -> None:
    """True: every stage; False: off; else stage names (as in STAGE_NAMES) to time alone."""
    if stages is True:
        mask = FNO_TIMING_ALL
    elif not stages:
        mask = 0
    else:
        mask = 0
        for name in stages:
            mask |= 1 << STAGE_NAMES.index(name)
    _check(lib().fno_timing_enable(ctypes.c_int(mask)))


def fno_timing_read(capacity: int = 8192):
    """List of (stage name, milliseconds) in launch order since the last read."""
    stages = (ctypes.c_int32 * capacity)()
    ms = (ctypes.c_float * capacity)()
    n = ctypes.c_int32(0)
    _check(lib().fno_timing_read(stages, ms, ctypes.c_int32(capacity), ctypes.byref(n)))
    return [(STAGE_NAMES[stages[i]], float(ms[i])) for i in range(n.value)]
