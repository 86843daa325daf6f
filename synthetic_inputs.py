"""Seeded synthetic inputs for the MGRIT-GRU workloads.

This module only draws random tensors (shapes, value distributions and the
rounding of inputs to a storage type).  It holds none of the method's
arithmetic: no GRU cell, no relaxation, no projection.  Both the CPU oracle's
tests and the HIP path's tests/bench take their inputs from here so that the two
sides see bit-identical host arrays.

Draw order (fixed, from ``numpy.random.default_rng(seed)``):
    x, W, U, b_i, b_h, h0, dL_dhT, W_o, b_o, labels
Gate order in the stacked 3H dimension is r, z, n (Eq. 1 of the paper).

The public-benchmark inputs the paper trains on (HMDB51 ResNet features,
UCI-HAR accelerometer traces) are not available here; these seeded tensors of
the same shapes stand in for them.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, Optional

import numpy as np


@dataclass(frozen=True)
class Workload:
    """One named configuration: sizes, MGRIT hierarchy and value recipe."""

    name: str
    T: int
    B: int
    D: int
    H: int
    cf: int
    levels: int
    fwd_iters: int
    bwd_iters: int
    dtype: str = "fp32"          # "fp32" | "bf16" (x, W, U rounded to bf16)
    x_dist: str = "normal"       # "normal" | "normal0.1" | "relu_normal"
    w_dist: str = "xavier"       # "xavier" | "normal0.1"
    n_classes: int = 51
    seed: int = 0

    def twin(self, coarsest_steps: int = 8) -> "Workload":
        """Reduced twin: same B, D, H, cf, levels; T = coarsest_steps*cf^(levels-1)."""
        T = coarsest_steps * self.cf ** (self.levels - 1)
        return replace(self, name=self.name + "-twin", T=T)


# The five benchmark configurations, in order (C1..C5).
WORKLOADS: Dict[str, Workload] = {
    "C1": Workload("C1", T=64, B=2, D=16, H=32, cf=4, levels=2, fwd_iters=3, bwd_iters=3,
                   x_dist="normal0.1", w_dist="normal0.1"),
    "C2": Workload("C2", T=1024, B=16, D=512, H=256, cf=4, levels=2, fwd_iters=8, bwd_iters=0),
    "C3": Workload("C3", T=2048, B=32, D=1024, H=512, cf=4, levels=3, fwd_iters=2, bwd_iters=2),
    "C4": Workload("C4", T=4096, B=8, D=2048, H=1024, cf=8, levels=3, fwd_iters=2, bwd_iters=1,
                   dtype="bf16", x_dist="relu_normal"),
    "C5": Workload("C5", T=16384, B=4, D=1024, H=1024, cf=4, levels=4, fwd_iters=2, bwd_iters=2),
    # Shape of the paper's HMDB51 experiment (Sec. 4: 128 time steps, batch 100, 1000
    # features, hidden size 1000, cf = 4, 3 levels, 2 forward / 1 backward iterations);
    # used with two stacked layers.  Not one of the five benchmark configurations.
    "P1": Workload("P1", T=128, B=100, D=1000, H=1000, cf=4, levels=3, fwd_iters=2, bwd_iters=1,
                   x_dist="relu_normal"),
}


def layer_workload(wl: Workload, layer: int) -> Workload:
    """Workload whose draw gives the parameters of layer `layer` (0-based) of a stack
    built on `wl`: layers above the first read H features (the states of the layer
    below) and use their own seed; the x of their draw is not used."""
    if layer == 0:
        return wl
    return replace(wl, name=f"{wl.name}-layer{layer + 1}", D=wl.H, seed=wl.seed + 1000 * layer)


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even); result stays fp32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    bits = a.view(np.uint32).astype(np.uint64)
    lsb = (bits >> 16) & 1
    rounded = ((bits + 0x7FFF + lsb) >> 16) << 16
    return rounded.astype(np.uint32).view(np.float32).reshape(a.shape)


def to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Upper 16 bits of already bf16-representable fp32 values, as uint16."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) >> 16).astype(np.uint16).reshape(a.shape)


def _xavier(rng: np.random.Generator, fan_out: int, fan_in: int, n_gates: int) -> np.ndarray:
    # Per gate matrix [fan_out, fan_in] ~ U(+-sqrt(6/(fan_in+fan_out))), gates stacked on rows.
    bound = np.sqrt(6.0 / (fan_in + fan_out))
    return rng.uniform(-bound, bound, size=(n_gates * fan_out, fan_in))


def make_inputs(wl: Workload, seed: Optional[int] = None) -> Dict[str, np.ndarray]:
    """Draw every tensor of a workload.  All arrays are C-contiguous float32
    (labels int64).  For ``dtype == "bf16"`` x, W and U hold bf16-representable
    values (so an fp64 oracle and a bf16 kernel read the same numbers)."""
    rng = np.random.default_rng(wl.seed if seed is None else seed)
    T, B, D, H = wl.T, wl.B, wl.D, wl.H

    if wl.x_dist == "normal":
        x = rng.standard_normal((T, B, D))
    elif wl.x_dist == "normal0.1":
        x = 0.1 * rng.standard_normal((T, B, D))
    elif wl.x_dist == "relu_normal":
        x = np.maximum(rng.standard_normal((T, B, D)), 0.0)
    else:
        raise ValueError(wl.x_dist)

    if wl.w_dist == "xavier":
        W = _xavier(rng, H, D, 3)
        U = _xavier(rng, H, H, 3)
        b_i = np.zeros(3 * H)
        b_h = np.zeros(3 * H)
    elif wl.w_dist == "normal0.1":
        W = 0.1 * rng.standard_normal((3 * H, D))
        U = 0.1 * rng.standard_normal((3 * H, H))
        b_i = 0.1 * rng.standard_normal(3 * H)
        b_h = 0.1 * rng.standard_normal(3 * H)
    else:
        raise ValueError(wl.w_dist)

    h0 = np.zeros((B, H))
    dL_dhT = rng.standard_normal((B, H)) / np.sqrt(H)
    W_o = _xavier(rng, wl.n_classes, H, 1)
    b_o = np.zeros(wl.n_classes)
    labels = rng.integers(0, wl.n_classes, size=B)

    out = {
        "x": x, "W": W, "U": U, "b_i": b_i, "b_h": b_h, "h0": h0,
        "dL_dhT": dL_dhT, "W_o": W_o, "b_o": b_o,
    }
    out = {k: np.ascontiguousarray(v, dtype=np.float32) for k, v in out.items()}
    if wl.dtype == "bf16":
        for k in ("x", "W", "U"):
            out[k] = round_to_bf16(out[k])
    out["labels"] = labels.astype(np.int64)
    return out


def random_small(seed: int, T: int, B: int, D: int, H: int, scale: float = 0.5,
                 h0_random: bool = True) -> Dict[str, np.ndarray]:
    """Small dense random problem (all parameters and h0 nonzero) for oracle
    pins and edge-case parity tests."""
    rng = np.random.default_rng(seed)
    d = {
        "x": rng.standard_normal((T, B, D)),
        "W": scale * rng.standard_normal((3 * H, D)),
        "U": scale * rng.standard_normal((3 * H, H)),
        "b_i": scale * rng.standard_normal(3 * H),
        "b_h": scale * rng.standard_normal(3 * H),
        "h0": (rng.standard_normal((B, H)) if h0_random else np.zeros((B, H))),
        "dL_dhT": rng.standard_normal((B, H)),
    }
    return {k: np.ascontiguousarray(v, dtype=np.float32) for k, v in d.items()}


def random_ode(seed: int, T: int, B: int, D: int, H: int, scale: Optional[float] = None,
               h0_random: bool = True) -> Dict[str, np.ndarray]:
    """Inputs of the demonstration ODE (appendix, Eq. 17): data d[T,B,D] ~ N(0,1),
    randomly selected time-independent weights A[H,H], Bw[H,D] and bias b[H]
    (N(0,1) scaled by `scale`, default 1/sqrt(fan-in)), initial state h0[B,H].
    Draw order: d, A, Bw, b, h0."""
    rng = np.random.default_rng(seed)
    sa = scale if scale is not None else 1.0 / np.sqrt(H)
    sb = scale if scale is not None else 1.0 / np.sqrt(D)
    out = {
        "d": rng.standard_normal((T, B, D)),
        "A": sa * rng.standard_normal((H, H)),
        "Bw": sb * rng.standard_normal((H, D)),
        "b": 0.5 * rng.standard_normal(H),
        "h0": (rng.standard_normal((B, H)) if h0_random else np.zeros((B, H))),
    }
    return {k: np.ascontiguousarray(v, dtype=np.float32) for k, v in out.items()}


# ---------------------------------------------------------------------------
# Synthetic classification task for the training loop (Alg. 3 of the paper)
# ---------------------------------------------------------------------------
# Stands in for the UCI-HAR traces (128 steps x 9 channels, 6 classes), which are not
# available here: the label of a sequence is a fixed function of its inputs, so a GRU can
# learn it.  Inputs and labels only; none of the method's arithmetic.

@dataclass(frozen=True)
class ClassificationTask:
    T: int = 128
    B: int = 100
    D: int = 12            # input width seen by the GRU (channels padded with zeros)
    channels: int = 9
    classes: int = 6
    seed: int = 0

    def readout(self) -> np.ndarray:
        return np.random.default_rng(self.seed).standard_normal(
            (self.classes, self.channels)).astype(np.float32)

    def batch(self, index: int):
        """Batch `index`: x[T,B,D] float32 ~ N(0,1) in the first `channels` columns, labels[B] =
        argmax_c sum_t 0.97^(T-t) <readout_c, x_t> (recent steps weigh more)."""
        r = np.random.default_rng(1000 + index)
        x = np.zeros((self.T, self.B, self.D), dtype=np.float32)
        x[:, :, :self.channels] = r.standard_normal((self.T, self.B, self.channels))
        decay = (0.97 ** np.arange(self.T - 1, -1, -1)).astype(np.float32)
        score = np.einsum("t,tbd,cd->bc", decay, x[:, :, :self.channels], self.readout())
        return x, np.argmax(score, axis=1).astype(np.int64)


def init_stack(seed: int, D: int, H: int, classes: int, layers: int):
    """Xavier-uniform parameters of a stack of GRU layers and a linear head, zero biases.
    Returns (params, head): params[j] = [W, U, b_i, b_h] (layer 0 reads D features, the others
    H), head = [W_o[classes,H], b_o[classes]]; all float32."""
    r = np.random.default_rng(seed)
    params = []
    for j in range(layers):
        Dj = D if j == 0 else H
        params.append([_xavier(r, H, Dj, 3).astype(np.float32), _xavier(r, H, H, 3).astype(np.float32),
                       np.zeros(3 * H, dtype=np.float32), np.zeros(3 * H, dtype=np.float32)])
    head = [_xavier(r, classes, H, 1).astype(np.float32), np.zeros(classes, dtype=np.float32)]
    return params, head


def random_lstm(seed: int, T: int, B: int, D: int, H: int, scale: float = 0.5,
                u0_random: bool = True) -> Dict[str, np.ndarray]:
    """Small dense random LSTM problem: x[T,B,D], W[4H,D], U[4H,H], b_i[4H], b_h[4H] (gate order
    i, f, g, o) and the initial state pair u0[B,2H] = (h_0 | c_0)."""
    rng = np.random.default_rng(seed)
    d = {
        "x": rng.standard_normal((T, B, D)),
        "W": scale * rng.standard_normal((4 * H, D)),
        "U": scale * rng.standard_normal((4 * H, H)),
        "b_i": scale * rng.standard_normal(4 * H),
        "b_h": scale * rng.standard_normal(4 * H),
        "u0": (0.5 * rng.standard_normal((B, 2 * H)) if u0_random else np.zeros((B, 2 * H))),
    }
    return {k: np.ascontiguousarray(v, dtype=np.float32) for k, v in d.items()}


def make_lstm_inputs(wl: Workload, seed: Optional[int] = None) -> Dict[str, np.ndarray]:
    """LSTM inputs at the sizes of a workload: x as in make_inputs, Xavier-uniform weights per
    gate matrix (four gates), zero biases, zero initial state pair."""
    rng = np.random.default_rng(wl.seed if seed is None else seed)
    T, B, D, H = wl.T, wl.B, wl.D, wl.H
    x = rng.standard_normal((T, B, D))
    if wl.x_dist == "relu_normal":
        x = np.maximum(x, 0.0)
    out = {"x": x, "W": _xavier(rng, H, D, 4), "U": _xavier(rng, H, H, 4),
           "b_i": np.zeros(4 * H), "b_h": np.zeros(4 * H), "u0": np.zeros((B, 2 * H))}
    return {k: np.ascontiguousarray(v, dtype=np.float32) for k, v in out.items()}
