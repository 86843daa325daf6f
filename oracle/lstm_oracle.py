"""CPU oracle for the MGRIT forward solve over an LSTM layer (the extension the paper's conclusion
names without giving equations).

TEST INFRASTRUCTURE ONLY (see mgrit_gru_oracle.py): float64 numpy; only tests, the smoke check
and the bench's CPU leg may import it.

The paper derives its Implicit GRU (Sec. 3.3, Eq. 15/16) by reading the cell as a forward-Euler
step of an ODE whose decay term is stiff, and taking that term implicitly.  The same steps for the
LSTM cell, which is NOT in the paper ("parity unpinned" against it; the pins are a library LSTM
for the explicit step with step size 1, the defining implicit equations, the common ODE limit,
closed forms, and the propagator-independent properties of the cycle):

  gates at (x_t, h_{t-1}):   i, f, o = sigmoid(.), g = tanh(.)   of  P + U h + b_h   (order i, f, g, o)
  standard cell:             c_t = f c_{t-1} + i g,           h_t = o tanh(c_t)
  as an ODE (step 1 of):     dc/dt = -(1 - f) c + i g,        dh/dt = -h + o tanh(c)
  explicit step, size gamma: c' = c + gamma (-(1-f) c + i g), h' = h + gamma (-h + o tanh(c'))
  implicit in the decay:     c' = (c + gamma i g) / (1 + gamma (1-f)),
                             h' = (h + gamma o tanh(c')) / (1 + gamma)

The state of the time integration is the pair (h, c); state arrays are [(T+1), B, 2H] with h in
columns 0..H-1 and c in columns H..2H-1.  Level l uses gamma = cf^l and the inputs of its own
points (Sec. 3.1, 3.3), exactly as for the GRU; the cycle is mgrit_gru_oracle.v_cycle.
"""
from __future__ import annotations

import numpy as np

from . import mgrit_gru_oracle as orc

IMPLICIT = 0
CLASSIC = 1


def lstm_gates(P, h, U, b_h):
    """i, f, g, o at (x_t through P = W x_t + b_i, h = h_{t-1}); stacked order i, f, g, o."""
    H = h.shape[-1]
    a = P + orc._rows_times(h, U.T) + b_h
    i = orc.sigmoid(a[..., :H])
    f = orc.sigmoid(a[..., H:2 * H])
    g = np.tanh(a[..., 2 * H:3 * H])
    o = orc.sigmoid(a[..., 3 * H:])
    return i, f, g, o


def lstm_phi(gamma, P, u, U, b_h, propagator=IMPLICIT):
    """One step (h', c') = Phi_gamma(x_t, (h, c)) on states u[..., 2H] = (h | c)."""
    H = u.shape[-1] // 2
    h, c = u[..., :H], u[..., H:]
    i, f, g, o = lstm_gates(P, h, U, b_h)
    if propagator == IMPLICIT:
        c_new = (c + gamma * i * g) / (1.0 + gamma * (1.0 - f))
        h_new = (h + gamma * o * np.tanh(c_new)) / (1.0 + gamma)
    elif propagator == CLASSIC:
        c_new = c + gamma * (-(1.0 - f) * c + i * g)
        h_new = h + gamma * (-h + o * np.tanh(c_new))
    else:
        raise ValueError("unknown propagator")
    return np.concatenate([h_new, c_new], axis=-1)


def lstm_serial_scan(W, U, b_i, b_h, x, u0, propagator=IMPLICIT, gamma=1.0):
    """u_t = Phi_gamma(x_t, u_{t-1}), t = 1..T; u0[B,2H].  Returns u[(T+1),B,2H]."""
    W, U, b_i, b_h, x, u0 = map(orc._f64, (W, U, b_i, b_h, x, u0))
    P = orc.input_projection(W, b_i, x)
    T = x.shape[0]
    u = np.empty((T + 1,) + u0.shape)
    u[0] = u0
    for t in range(1, T + 1):
        u[t] = lstm_phi(gamma, P[t - 1], u[t - 1], U, b_h, propagator)
    return u


def mgrit_lstm_forward(W, U, b_i, b_h, x, u0, u_init, cf, levels, iters, fine_relax_fcf=True,
                       propagator=IMPLICIT, keep_iterates=False):
    """`iters` applications of the cycle of Alg. 2 (recursive, Remark 2) to the iterate
    u_init[(T+1),B,2H]; row 0 is overwritten with u0.  Returns (u, resnorms[, iterates])."""
    W, U, b_i, b_h, x, u0 = map(orc._f64, (W, U, b_i, b_h, x, u0))
    T = x.shape[0]
    orc._check_hierarchy(T, cf, levels)
    P = orc.input_projection(W, b_i, x)

    def step(l, ks, v):
        return lstm_phi(float(cf ** l), P[ks * cf ** l - 1], v, U, b_h, propagator)

    u = orc._f64(u_init).copy()
    u[0] = u0
    g0 = np.zeros_like(u)
    resnorms, iterates = [], []
    for _ in range(iters):
        u = orc.v_cycle(step, cf, levels, 0, u, g0, fine_relax_fcf, resnorms)
        if keep_iterates:
            iterates.append(u.copy())
    return (u, resnorms, iterates) if keep_iterates else (u, resnorms)
