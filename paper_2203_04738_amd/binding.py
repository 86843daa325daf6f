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


MGRIT_F32, MGRIT_BF16, MGRIT_F32_BF16X3, MGRIT_BF16_STATE2 = 0, 1, 2, 3   # cfg.dtype
MGRIT_REUSE_PROJECTION = 1
MGRIT_KEEP_COEFFS = 2
MGRIT_REUSE_COEFFS = 4
MGRIT_ZERO_ADJOINT_GUESS = 8
MGRIT_ZERO_STATE_GUESS = 16
MGRIT_STATIC_SCRATCH_BYTES = 64 << 20     # workspace limit of mgrit_gru_forward_static
MGRIT_E_STATE = -9
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
    L.mgrit_gru_forward_static.argtypes = [cfgp, vp, vp, fp, fp, vp, fp, fp, fp, vp]
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
    L.mgrit_lstm_workspace_bytes.argtypes = [cfgp, ctypes.POINTER(sz)]
    L.lstm_serial_scan.argtypes = [cfgp, fp, fp, fp, fp, fp, fp, fp, vp, sz, vp]
    L.mgrit_lstm_forward.argtypes = [cfgp, fp, fp, fp, fp, fp, fp, fp, fp, vp, sz, vp]
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
                 "mgrit_gru_forward_static",
                 "gru_serial_scan_backward", "mgrit_gru_backward",
                 "gru_serial_scan_backward_steps", "mgrit_gru_backward_steps",
                 "ode_serial_scan", "mgrit_ode_forward", "mgrit_lstm_workspace_bytes",
                 "lstm_serial_scan", "mgrit_lstm_forward", "mgrit_gru_profile_enable", "mgrit_gru_profile_read_shape",
                 "mgrit_gru_profile_read"):
        getattr(L, name).restype = ctypes.c_int
    _lib = L
    return L


def mgrit_gru_strerror(code: int) -> str:
    return lib().mgrit_gru_strerror(int(code)).decode()


class _Arg:
    """One tensor argument and what cfg implies about it."""

    def __init__(self, t, name, dtype=None, shape=None, min_numel=None):
        self.t, self.name, self.dtype, self.shape, self.min_numel = t, name, dtype, shape, min_numel


def _marshal(args):
    """Device pointers of contiguous CUDA tensors (None passes NULL; plain values pass through).
    The C ABI takes plain pointers and cannot know buffer sizes, so the size of every tensor is
    compared with what cfg implies here: `shape` must match exactly, `min_numel` is a lower
    bound.  All sizes are checked first (ValueError), then dtype, layout and device
    (TypeError / ValueError); nothing is launched unless every argument passes."""
    import torch
    for a in args:
        if not isinstance(a, _Arg) or a.t is None:
            continue
        if not isinstance(a.t, torch.Tensor):
            raise TypeError(f"{a.name}: expected a CUDA tensor")
        if a.shape is not None and tuple(a.t.shape) != tuple(a.shape):
            raise ValueError(f"{a.name}: expected shape {tuple(a.shape)}, got {tuple(a.t.shape)}")
        if a.min_numel is not None and a.t.numel() < a.min_numel:
            raise ValueError(f"{a.name}: expected at least {a.min_numel} elements, "
                             f"got {a.t.numel()}")
    out = []
    for a in args:
        if not isinstance(a, _Arg):
            out.append(a)
        elif a.t is None:
            out.append(None)
        else:
            if a.dtype is not None and a.t.dtype != a.dtype:
                raise TypeError(f"{a.name}: expected dtype {a.dtype}, got {a.t.dtype}")
            if not a.t.is_contiguous():
                raise ValueError(f"{a.name}: tensor must be contiguous")
            if not a.t.is_cuda:
                raise TypeError(f"{a.name}: expected a CUDA tensor")
            out.append(a.t.data_ptr())
    return out


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


def _check(rc: int, where: str) -> None:
    if rc != 0:
        raise MgritGruError(rc, where)


def _call(name: str, cfg, *args) -> None:
    """Checks and marshals the arguments, then calls entry point `name` on the current stream."""
    ptrs = _marshal(args)
    _check(getattr(lib(), name)(ctypes.byref(cfg), *ptrs, _stream()), name)


def mgrit_gru_workspace_bytes(cfg: MgritGruCfg) -> int:
    n = ctypes.c_size_t(0)
    _check(lib().mgrit_gru_workspace_bytes(ctypes.byref(cfg), ctypes.byref(n)),
           "mgrit_gru_workspace_bytes")
    return int(n.value)


def _f32():
    import torch
    return torch.float32


def _params(cfg, W, U, b_i, b_h, x):
    """The five arguments every GRU entry point starts with."""
    import torch
    f32 = torch.float32
    dt = torch.bfloat16 if cfg.dtype in (MGRIT_BF16, MGRIT_BF16_STATE2) else f32
    T, B, D, H = cfg.T, cfg.B, cfg.D, cfg.H
    return (_Arg(W, "W", dt, (3 * H, D)), _Arg(U, "U", dt, (3 * H, H)),
            _Arg(b_i, "b_i", f32, (3 * H,)), _Arg(b_h, "b_h", f32, (3 * H,)),
            _Arg(x, "x", dt, (T, B, D)))


def _grads(cfg, dW, dU, db_i, db_h):
    f32, D, H = _f32(), cfg.D, cfg.H
    return (_Arg(dW, "dW", f32, (3 * H, D)), _Arg(dU, "dU", f32, (3 * H, H)),
            _Arg(db_i, "db_i", f32, (3 * H,)), _Arg(db_h, "db_h", f32, (3 * H,)))


def _workspace(workspace):
    """Workspace pointer and its size in bytes (the library compares the size with cfg)."""
    n = 0 if workspace is None else workspace.numel() * workspace.element_size()
    return _Arg(workspace, "workspace"), ctypes.c_size_t(n)


def _state(cfg, t, name):
    return _Arg(t, name, _f32(), (cfg.T + 1, cfg.B, cfg.H))


def _row(cfg, t, name):
    return _Arg(t, name, _f32(), (cfg.B, cfg.H))


def _res(cfg, t):
    return _Arg(t, "resnorm_out", _f32(), min_numel=cfg.iters)


def _dx(cfg, t):
    return _Arg(t, "dx", _f32(), (cfg.T, cfg.B, cfg.D))


def gru_serial_scan(cfg, W, U, b_i, b_h, x, h0, h_out, workspace) -> None:
    _call("gru_serial_scan", cfg, *_params(cfg, W, U, b_i, b_h, x), _row(cfg, h0, "h0"),
          _state(cfg, h_out, "h_out"), *_workspace(workspace))


def _check_declared_zero(cfg, flag, tensor, rows, what):
    """Opt-in check of a zero-guess declaration (environment MGRIT_CHECK_ZERO_GUESS=1): the
    library trusts MGRIT_ZERO_STATE_GUESS / MGRIT_ZERO_ADJOINT_GUESS; with the variable set the
    binding looks at the rows the flag declares zero before the call (this reads the tensor
    back, so it synchronises; meant for debugging a harness, not for timed runs)."""
    if not (cfg.flags & flag) or os.environ.get("MGRIT_CHECK_ZERO_GUESS") != "1":
        return
    import torch
    if tensor is not None and tensor.is_cuda and int(torch.count_nonzero(tensor[rows])) != 0:
        raise ValueError(f"{what}: declared zero by the flags, but holds non-zero values")


def mgrit_gru_forward(cfg, W, U, b_i, b_h, x, h0, h_inout, resnorm_out, workspace) -> None:
    _check_declared_zero(cfg, MGRIT_ZERO_STATE_GUESS, h_inout, slice(1, None), "h_inout rows 1..T")
    _call("mgrit_gru_forward", cfg, *_params(cfg, W, U, b_i, b_h, x), _row(cfg, h0, "h0"),
          _state(cfg, h_inout, "h_inout"), _res(cfg, resnorm_out), *_workspace(workspace))


def mgrit_gru_forward_static(cfg, W, U, b_i, b_h, x, h0, h_inout, resnorm_out) -> None:
    _call("mgrit_gru_forward_static", cfg, *_params(cfg, W, U, b_i, b_h, x), _row(cfg, h0, "h0"),
          _state(cfg, h_inout, "h_inout"), _res(cfg, resnorm_out))


def gru_serial_scan_backward(cfg, W, U, b_i, b_h, x, h, dL_dhT, w_out, dW, dU, db_i, db_h,
                             workspace) -> None:
    _call("gru_serial_scan_backward", cfg, *_params(cfg, W, U, b_i, b_h, x), _state(cfg, h, "h"),
          _row(cfg, dL_dhT, "dL_dhT"), _state(cfg, w_out, "w_out"),
          *_grads(cfg, dW, dU, db_i, db_h), *_workspace(workspace))


def mgrit_gru_backward(cfg, W, U, b_i, b_h, x, h, dL_dhT, w_inout, resnorm_out, dW, dU, db_i,
                       db_h, workspace) -> None:
    _check_declared_zero(cfg, MGRIT_ZERO_ADJOINT_GUESS, w_inout, slice(0, -1), "w_inout rows 0..T-1")
    _call("mgrit_gru_backward", cfg, *_params(cfg, W, U, b_i, b_h, x), _state(cfg, h, "h"),
          _row(cfg, dL_dhT, "dL_dhT"), _state(cfg, w_inout, "w_inout"), _res(cfg, resnorm_out),
          *_grads(cfg, dW, dU, db_i, db_h), *_workspace(workspace))


def gru_serial_scan_backward_steps(cfg, W, U, b_i, b_h, x, h, dL_dh, w_out, dW, dU, db_i, db_h,
                                   dx, workspace) -> None:
    _call("gru_serial_scan_backward_steps", cfg, *_params(cfg, W, U, b_i, b_h, x),
          _state(cfg, h, "h"), _state(cfg, dL_dh, "dL_dh"), _state(cfg, w_out, "w_out"),
          *_grads(cfg, dW, dU, db_i, db_h), _dx(cfg, dx), *_workspace(workspace))


def mgrit_gru_backward_steps(cfg, W, U, b_i, b_h, x, h, dL_dh, w_inout, resnorm_out, dW, dU,
                             db_i, db_h, dx, workspace) -> None:
    _check_declared_zero(cfg, MGRIT_ZERO_ADJOINT_GUESS, w_inout, slice(0, -1), "w_inout rows 0..T-1")
    _check_declared_zero(cfg, MGRIT_ZERO_ADJOINT_GUESS, dL_dh, slice(0, -1), "dL_dh rows 0..T-1")
    _call("mgrit_gru_backward_steps", cfg, *_params(cfg, W, U, b_i, b_h, x), _state(cfg, h, "h"),
          _state(cfg, dL_dh, "dL_dh"), _state(cfg, w_inout, "w_inout"), _res(cfg, resnorm_out),
          *_grads(cfg, dW, dU, db_i, db_h), _dx(cfg, dx), *_workspace(workspace))


def _ode_params(cfg, dt, A, Bw, b, d):
    f32 = _f32()
    T, B, D, H = cfg.T, cfg.B, cfg.D, cfg.H
    return (ctypes.c_float(float(dt)), _Arg(A, "A", f32, (H, H)), _Arg(Bw, "Bw", f32, (H, D)),
            _Arg(b, "b", f32, (H,)), _Arg(d, "d", f32, (T, B, D)))


def ode_serial_scan(cfg, dt, A, Bw, b, d, h0, h_out, workspace) -> None:
    _call("ode_serial_scan", cfg, *_ode_params(cfg, dt, A, Bw, b, d), _row(cfg, h0, "h0"),
          _state(cfg, h_out, "h_out"), *_workspace(workspace))


def mgrit_ode_forward(cfg, dt, A, Bw, b, d, h0, h_inout, resnorm_out, workspace) -> None:
    _call("mgrit_ode_forward", cfg, *_ode_params(cfg, dt, A, Bw, b, d), _row(cfg, h0, "h0"),
          _state(cfg, h_inout, "h_inout"), _res(cfg, resnorm_out), *_workspace(workspace))


def mgrit_lstm_workspace_bytes(cfg: MgritGruCfg) -> int:
    n = ctypes.c_size_t(0)
    _check(lib().mgrit_lstm_workspace_bytes(ctypes.byref(cfg), ctypes.byref(n)),
           "mgrit_lstm_workspace_bytes")
    return int(n.value)


def _lstm_params(cfg, W, U, b_i, b_h, x):
    f32 = _f32()
    T, B, D, H = cfg.T, cfg.B, cfg.D, cfg.H
    return (_Arg(W, "W", f32, (4 * H, D)), _Arg(U, "U", f32, (4 * H, H)),
            _Arg(b_i, "b_i", f32, (4 * H,)), _Arg(b_h, "b_h", f32, (4 * H,)),
            _Arg(x, "x", f32, (T, B, D)))


def lstm_serial_scan(cfg, W, U, b_i, b_h, x, u0, u_out, workspace) -> None:
    f32 = _f32()
    _call("lstm_serial_scan", cfg, *_lstm_params(cfg, W, U, b_i, b_h, x),
          _Arg(u0, "u0", f32, (cfg.B, 2 * cfg.H)),
          _Arg(u_out, "u_out", f32, (cfg.T + 1, cfg.B, 2 * cfg.H)), *_workspace(workspace))


def mgrit_lstm_forward(cfg, W, U, b_i, b_h, x, u0, u_inout, resnorm_out, workspace) -> None:
    f32 = _f32()
    _call("mgrit_lstm_forward", cfg, *_lstm_params(cfg, W, U, b_i, b_h, x),
          _Arg(u0, "u0", f32, (cfg.B, 2 * cfg.H)),
          _Arg(u_inout, "u_inout", f32, (cfg.T + 1, cfg.B, 2 * cfg.H)), _res(cfg, resnorm_out),
          *_workspace(workspace))


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
