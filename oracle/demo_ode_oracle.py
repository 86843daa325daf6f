"""CPU oracle for MGRIT forward propagation of the paper's demonstration ODE.

TEST INFRASTRUCTURE ONLY (same rules as mgrit_gru_oracle.py: float64, plain,
imported by tests, the smoke check and the bench's cpu_baseline leg only).

The ODE (appendix "Why does MGRIT work?", Eq. 17):

    dh/dt = -h/2 + sigmoid(A h + B d(t) + b)

with hidden state h in R^H, user data d(t) in R^D and time-independent A[H,H],
B[H,D], b[H].  The paper uses it for forward propagation only; so does this file.

Readings (the appendix names the equation and prints one residual history, not
the discretisation):
* time integrator: forward Euler, one step per data sample,
      Phi_dt(h_{t-1}; d_t) = h_{t-1} + dt * (-h_{t-1}/2 + sigmoid(A h_{t-1} + B d_t + b));
* level l of the hierarchy rediscretises with step size cf^l * dt and the data of
  its own points (injection), the rule Sec. 3.3 gives for the GRU;
* dt is an argument; the demonstration's parameter "alpha" is not defined in the
  text and is not modelled.
Against the printed residual history only the rate per cycle can be compared
(random weights, integrator not stated): values "parity unpinned" there.  Pinned by
closed forms, the exact solution of the ODE in the limit dt -> 0, and MGRIT's
exactness properties in tests/test_oracle_pins_ode.py.

Layout as for the GRU oracle: d[T,B,D] row t-1 holds d_t; h[(T+1),B,H] row t holds
h_t, row 0 the initial condition.
"""
from __future__ import annotations

import numpy as np

from .mgrit_gru_oracle import _check_hierarchy, _f64, sigmoid, v_cycle


def ode_projection(Bw, b, d):
    """P[t-1] = B d_t + b for every sample: the part of the sigmoid's argument that
    does not depend on the state (Eq. 17)."""
    return _f64(d) @ _f64(Bw).T + _f64(b)


def ode_phi(dt, P_rows, h, A):
    """One forward-Euler step of Eq. 17 with step size dt from states h[...,H],
    given P_rows = B d + b of the points stepped to."""
    return h + dt * (-0.5 * h + sigmoid(h @ A.T + P_rows))


def ode_serial_scan(A, Bw, b, d, h0, dt):
    """Sequential propagation h_t = Phi_dt(h_{t-1}; d_t), t = 1..T."""
    A, h0 = _f64(A), _f64(h0)
    P = ode_projection(Bw, b, d)
    T = P.shape[0]
    h = np.zeros((T + 1,) + h0.shape)
    h[0] = h0
    for t in range(1, T + 1):
        h[t] = ode_phi(dt, P[t - 1], h[t - 1], A)
    return h


def ode_fine_residual(A, Bw, b, d, h, dt):
    """r_t = h_t - Phi_dt(h_{t-1}; d_t), t = 1..T (zero for the serial solution)."""
    A, h = _f64(A), _f64(h)
    P = ode_projection(Bw, b, d)
    return h[1:] - ode_phi(dt, P, h[:-1], A)


def ode_mgrit_forward(A, Bw, b, d, h0, h_init, dt, cf, levels, iters,
                      fine_relax_fcf=True, keep_iterates=False):
    """`iters` MGRIT cycles (Alg. 2, recursive per Remark 2) on the iterate
    h_init[(T+1),B,H] with Phi of level l = forward Euler at step cf^l * dt.
    Returns (h, resnorms[, iterates]) like mgrit_forward of the GRU oracle."""
    A, h0 = _f64(A), _f64(h0)
    P = ode_projection(Bw, b, d)
    T = P.shape[0]
    _check_hierarchy(T, cf, levels)

    def step(l, ks, v):
        return ode_phi(dt * float(cf ** l), P[ks * cf ** l - 1], v, A)

    h = _f64(h_init).copy()
    h[0] = h0
    g0 = np.zeros_like(h)
    resnorms, iterates = [], []
    for _ in range(iters):
        h = v_cycle(step, cf, levels, 0, h, g0, fine_relax_fcf, resnorms)
        if keep_iterates:
            iterates.append(h.copy())
    if keep_iterates:
        return h, resnorms, iterates
    return h, resnorms
