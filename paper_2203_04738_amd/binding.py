"""ctypes binding of libmgrit_gru.so: argument marshalling only.

Each function has the name and argument order of the C entry point declared in
include/mgrit_gru.h.  Tensors are torch CUDA tensors (PyTorch is used here for
device memory and streams only); they are passed as raw device pointers, the
current torch stream is passed as the stream argument, and a negative return
code raises MgritGruError.  There is no fallback: without the built library, or
with a tensor that is not a contiguous CUDA tensor of the expected dtype, the
call fails.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_NAME = "libmgrit_gru.so"


class MgritGruError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {mgrit_gru_strerror(code)} ({code})")


class MgritGruCfg(ctypes.Structure):
    """Mirror of ``mgrit_gru_cfg``."""

    _fields_ = [(n, ctypes.c_int32) for n in (
        "T", "B", "D", "H", "cf", "levels", "iters", "fine_relax", "propagator", "dtype", "flags")]

    def __init__(self, T, B, D, H, cf=1, levels=1, iters=1, fine_relax=1, propagator=0, dtype=0,
                 flags=0):
        super().__init__(T, B, D, H, cf, levels, iters, fine_relax, propagator, dtype, flags)


MGRIT_F32, MGRIT_BF16, MGRIT_F32_BF16X3 = 0, 1, 2   # cfg.dtype
MGRIT_REUSE_PROJECTION = 1
MGRIT_KEEP_COEFFS = 2
MGRIT_REUSE_COEFFS = 4
MGRIT_ZERO_ADJOINT_GUESS = 8
MGRIT_ZERO_STATE_GUESS = 16
_lib = None


def lib_path() -> str:
    return os.path.join(_HERE, _LIB_NAME)


def lib() -> ctypes.CDLL:
    """Load the built library (built by ``paper_2203_04738_amd/build.py`` or
    ``__graft_entry__.build()``); building is attempted only if no library exists."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        from . import build as _build
        _build.build(verbose=False)
    L = ctypes.CDLL(path)
    vp, sz, fp = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p
    cfgp = ctypes.POINTER(MgritGruCfg)
    L.mgrit_gru_workspace_bytes.argtypes = [cfgp, ctypes.POINTER(sz)]
    L.gru_serial_scan.argtypes = [cfgp, vp, vp, fp, fp, vp, fp, fp, vp, sz, vp]
    L.mgrit_gru_forward.argtypes = [cfgp, vp, vp, fp, fp, vp, fp, fp, fp, vp, sz, vp]
    L.gru_serial_scan_backward.argtypes = [cfgp, vp, vp, fp, fp, vp, fp, fp, fp, fp, fp, fp, fp,
                                           vp, sz, vp]
    L.mgrit_gru_backward.argtypes = [cfgp, vp, vp, fp, fp, vp, fp, fp, fp, fp, fp, fp, fp, fp,
                                     vp, sz, vp]
    L.gru_serial_scan_backward_steps.argtypes = [cfgp, vp, vp, fp, fp, vp, fp, fp, fp, fp, fp, fp,
                                                 fp, fp, vp, sz, vp]
    L.mgrit_gru_backward_steps.argtypes = [cfgp, vp, vp, fp, fp, vp, fp, fp, fp, fp, fp, fp, fp,
                                           fp, fp, vp, sz, vp]
    cf = ctypes.c_float
    L.ode_serial_scan.argtypes = [cfgp, cf, fp, fp, fp, fp, fp, fp, vp, sz, vp]
    L.mgrit_ode_forward.argtypes = [cfgp, cf, fp, fp, fp, fp, fp, fp, fp, vp, sz, vp]
    L.mgrit_gru_strerror.argtypes = [ctypes.c_int]
    L.mgrit_gru_strerror.restype = ctypes.c_char_p
    L.mgrit_gru_profile_enable.argtypes = [ctypes.c_int]
    L.mgrit_gru_profile_read.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_int64),
                                         ctypes.POINTER(ctypes.c_double),
                                         ctypes.POINTER(ctypes.c_double),
                                         ctypes.POINTER(ctypes.c_double)]
    L.mgrit_gru_profile_read_shape.argtypes = [ctypes.c_int, ctypes.c_int64, ctypes.c_int,
                                               ctypes.POINTER(ctypes.c_int64),
                                               ctypes.POINTER(ctypes.c_double),
                                               ctypes.POINTER(ctypes.c_double),
                                               ctypes.POINTER(ctypes.c_double)]
    for name in ("mgrit_gru_workspace_bytes", "gru_serial_scan", "mgrit_gru_forward",
                 "gru_serial_scan_backward", "mgrit_gru_backward",
                 "gru_serial_scan_backward_steps", "mgrit_gru_backward_steps",
                 "ode_serial_scan", "mgrit_ode_forward", "mgrit_gru_profile_enable", "mgrit_gru_profile_read_shape",
                 "mgrit_gru_profile_read"):
        getattr(L, name).restype = ctypes.c_int
    _lib = L
    return L


def mgrit_gru_strerror(code: int) -> str:
    return lib().mgrit_gru_strerror(int(code)).decode()


def _ptr(t, name: str, dtype=None) -> Optional[int]:
    """Device pointer of a contiguous CUDA tensor (None passes NULL)."""
    if t is None:
        return None
    import torch
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name}: expected a CUDA tensor")
    if not t.is_contiguous():
        raise ValueError(f"{name}: tensor must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name}: expected dtype {dtype}, got {t.dtype}")
    return t.data_ptr()


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


def _in_dtype(cfg: MgritGruCfg):
    import torch
    return torch.bfloat16 if cfg.dtype == 1 else torch.float32


def _check(rc: int, where: str) -> None:
    if rc != 0:
        raise MgritGruError(rc, where)


def mgrit_gru_workspace_bytes(cfg: MgritGruCfg) -> int:
    n = ctypes.c_size_t(0)
    _check(lib().mgrit_gru_workspace_bytes(ctypes.byref(cfg), ctypes.byref(n)),
           "mgrit_gru_workspace_bytes")
    return int(n.value)


def gru_serial_scan(cfg, W, U, b_i, b_h, x, h0, h_out, workspace) -> None:
    import torch
    f32, dt = torch.float32, _in_dtype(cfg)
    _check(lib().gru_serial_scan(
        ctypes.byref(cfg), _ptr(W, "W", dt), _ptr(U, "U", dt), _ptr(b_i, "b_i", f32),
        _ptr(b_h, "b_h", f32), _ptr(x, "x", dt), _ptr(h0, "h0", f32), _ptr(h_out, "h_out", f32),
        _ptr(workspace, "workspace"), workspace.numel() * workspace.element_size(), _stream()),
        "gru_serial_scan")


def mgrit_gru_forward(cfg, W, U, b_i, b_h, x, h0, h_inout, resnorm_out, workspace) -> None:
    import torch
    f32, dt = torch.float32, _in_dtype(cfg)
    _check(lib().mgrit_gru_forward(
        ctypes.byref(cfg), _ptr(W, "W", dt), _ptr(U, "U", dt), _ptr(b_i, "b_i", f32),
        _ptr(b_h, "b_h", f32), _ptr(x, "x", dt), _ptr(h0, "h0", f32),
        _ptr(h_inout, "h_inout", f32), _ptr(resnorm_out, "resnorm_out", f32),
        _ptr(workspace, "workspace"), workspace.numel() * workspace.element_size(), _stream()),
        "mgrit_gru_forward")


def gru_serial_scan_backward(cfg, W, U, b_i, b_h, x, h, dL_dhT, w_out, dW, dU, db_i, db_h,
                             workspace) -> None:
    import torch
    f32, dt = torch.float32, _in_dtype(cfg)
    _check(lib().gru_serial_scan_backward(
        ctypes.byref(cfg), _ptr(W, "W", dt), _ptr(U, "U", dt), _ptr(b_i, "b_i", f32),
        _ptr(b_h, "b_h", f32), _ptr(x, "x", dt), _ptr(h, "h", f32), _ptr(dL_dhT, "dL_dhT", f32),
        _ptr(w_out, "w_out", f32), _ptr(dW, "dW", f32), _ptr(dU, "dU", f32),
        _ptr(db_i, "db_i", f32), _ptr(db_h, "db_h", f32),
        _ptr(workspace, "workspace"), workspace.numel() * workspace.element_size(), _stream()),
        "gru_serial_scan_backward")


def mgrit_gru_backward(cfg, W, U, b_i, b_h, x, h, dL_dhT, w_inout, resnorm_out, dW, dU, db_i,
                       db_h, workspace) -> None:
    import torch
    f32, dt = torch.float32, _in_dtype(cfg)
    _check(lib().mgrit_gru_backward(
        ctypes.byref(cfg), _ptr(W, "W", dt), _ptr(U, "U", dt), _ptr(b_i, "b_i", f32),
        _ptr(b_h, "b_h", f32), _ptr(x, "x", dt), _ptr(h, "h", f32), _ptr(dL_dhT, "dL_dhT", f32),
        _ptr(w_inout, "w_inout", f32), _ptr(resnorm_out, "resnorm_out", f32),
        _ptr(dW, "dW", f32), _ptr(dU, "dU", f32), _ptr(db_i, "db_i", f32), _ptr(db_h, "db_h", f32),
        _ptr(workspace, "workspace"), workspace.numel() * workspace.element_size(), _stream()),
        "mgrit_gru_backward")


def gru_serial_scan_backward_steps(cfg, W, U, b_i, b_h, x, h, dL_dh, w_out, dW, dU, db_i, db_h,
                                   dx, workspace) -> None:
    import torch
    f32, dt = torch.float32, _in_dtype(cfg)
    _check(lib().gru_serial_scan_backward_steps(
        ctypes.byref(cfg), _ptr(W, "W", dt), _ptr(U, "U", dt), _ptr(b_i, "b_i", f32),
        _ptr(b_h, "b_h", f32), _ptr(x, "x", dt), _ptr(h, "h", f32), _ptr(dL_dh, "dL_dh", f32),
        _ptr(w_out, "w_out", f32), _ptr(dW, "dW", f32), _ptr(dU, "dU", f32),
        _ptr(db_i, "db_i", f32), _ptr(db_h, "db_h", f32), _ptr(dx, "dx", f32),
        _ptr(workspace, "workspace"), workspace.numel() * workspace.element_size(), _stream()),
        "gru_serial_scan_backward_steps")


def mgrit_gru_backward_steps(cfg, W, U, b_i, b_h, x, h, dL_dh, w_inout, resnorm_out, dW, dU,
                             db_i, db_h, dx, workspace) -> None:
    import torch
    f32, dt = torch.float32, _in_dtype(cfg)
    _check(lib().mgrit_gru_backward_steps(
        ctypes.byref(cfg), _ptr(W, "W", dt), _ptr(U, "U", dt), _ptr(b_i, "b_i", f32),
        _ptr(b_h, "b_h", f32), _ptr(x, "x", dt), _ptr(h, "h", f32), _ptr(dL_dh, "dL_dh", f32),
        _ptr(w_inout, "w_inout", f32), _ptr(resnorm_out, "resnorm_out", f32),
        _ptr(dW, "dW", f32), _ptr(dU, "dU", f32), _ptr(db_i, "db_i", f32), _ptr(db_h, "db_h", f32),
        _ptr(dx, "dx", f32),
        _ptr(workspace, "workspace"), workspace.numel() * workspace.element_size(), _stream()),
        "mgrit_gru_backward_steps")


def ode_serial_scan(cfg, dt, A, Bw, b, d, h0, h_out, workspace) -> None:
    import torch
    f32 = torch.float32
    _check(lib().ode_serial_scan(
        ctypes.byref(cfg), float(dt), _ptr(A, "A", f32), _ptr(Bw, "Bw", f32), _ptr(b, "b", f32),
        _ptr(d, "d", f32), _ptr(h0, "h0", f32), _ptr(h_out, "h_out", f32),
        _ptr(workspace, "workspace"), workspace.numel() * workspace.element_size(), _stream()),
        "ode_serial_scan")


def mgrit_ode_forward(cfg, dt, A, Bw, b, d, h0, h_inout, resnorm_out, workspace) -> None:
    import torch
    f32 = torch.float32
    _check(lib().mgrit_ode_forward(
        ctypes.byref(cfg), float(dt), _ptr(A, "A", f32), _ptr(Bw, "Bw", f32), _ptr(b, "b", f32),
        _ptr(d, "d", f32), _ptr(h0, "h0", f32), _ptr(h_inout, "h_inout", f32),
        _ptr(resnorm_out, "resnorm_out", f32),
        _ptr(workspace, "workspace"), workspace.numel() * workspace.element_size(), _stream()),
        "mgrit_ode_forward")


def mgrit_gru_profile_enable(on: bool) -> None:
    _check(lib().mgrit_gru_profile_enable(1 if on else 0), "mgrit_gru_profile_enable")


def mgrit_gru_profile_read_shape(kind: int, rows: int = -1, mode: int = -1):
    """(launches, total_ms, flops, bytes) of the launches of a step kernel class that advance
    `rows` rows in epilogue mode `mode` (negative: any); clears what it returns."""
    n = ctypes.c_int64(0)
    ms, fl, by = ctypes.c_double(0), ctypes.c_double(0), ctypes.c_double(0)
    _check(lib().mgrit_gru_profile_read_shape(kind, rows, mode, ctypes.byref(n), ctypes.byref(ms),
                                              ctypes.byref(fl), ctypes.byref(by)),
           "mgrit_gru_profile_read_shape")
    return int(n.value), float(ms.value), float(fl.value), float(by.value)


def mgrit_gru_profile_read(kind: int):
    """Returns (launches, total_ms, flops, bytes) of the kernel class and clears it."""
    n = ctypes.c_int64(0)
    ms, fl, by = ctypes.c_double(0), ctypes.c_double(0), ctypes.c_double(0)
    _check(lib().mgrit_gru_profile_read(kind, ctypes.byref(n), ctypes.byref(ms), ctypes.byref(fl),
                                        ctypes.byref(by)), "mgrit_gru_profile_read")
    return int(n.value), float(ms.value), float(fl.value), float(by.value)
