"""Pins for the demonstration-ODE oracle (appendix, Eq. 17; no GPU).

None of them re-types the oracle's step and compares it with itself: they use the
closed form of the recurrence without coupling, the exact solution of the ODE, a
library ODE integrator on the equation written out here, and the properties MGRIT
has for any propagator (fixed point, exactness front, convergence to the serial
propagation).
"""
import os

import numpy as np
import pytest
from scipy.integrate import solve_ivp

from oracle import demo_ode_oracle as ode
from synthetic_inputs import random_ode


GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rel(a, b):
    return np.max(np.abs(a - b)) / max(np.max(np.abs(b)), 1e-300)


def test_uncoupled_recurrence_has_the_geometric_closed_form():
    """A = 0, B = 0: h_t = c^t h_0 + 2 s (1 - c^t), c = 1 - dt/2, s = sigmoid(b):
    pins the decay term -h/2, the sign of the source and the bias."""
    T, B, D, H, dt = 40, 2, 3, 5, 0.3
    p = random_ode(3, T, B, D, H)
    h = ode.ode_serial_scan(np.zeros((H, H)), np.zeros((H, D)), p["b"], p["d"], p["h0"], dt)
    s = 1.0 / (1.0 + np.exp(-p["b"].astype(np.float64)))
    c = 1.0 - dt / 2
    for t in (0, 1, 7, T):
        want = c ** t * p["h0"].astype(np.float64) + 2.0 * s * (1.0 - c ** t)
        assert _rel(h[t], want) < 1e-13


def test_serial_scan_converges_to_the_ode_solution_at_first_order():
    """Constant data: a library integrator solves dh/dt = -h/2 + sigmoid(A h + B d + b),
    written out here with A acting on h as a matrix-vector product; the scan's error
    at the final time halves when the step halves.  Pins the orientation of A and B
    (both non-symmetric / non-square) and the step-size factor."""
    B, D, H, tend = 1, 3, 4, 2.0
    p = random_ode(5, 1, B, D, H, scale=0.8)
    A, Bw, b = (p[k].astype(np.float64) for k in ("A", "Bw", "b"))
    d0 = p["d"][0, 0].astype(np.float64)
    h0 = p["h0"][0].astype(np.float64)

    def rhs(t, h):
        return -0.5 * h + 1.0 / (1.0 + np.exp(-(A @ h + Bw @ d0 + b)))

    ref = solve_ivp(rhs, (0.0, tend), h0, rtol=1e-12, atol=1e-14).y[:, -1]
    errs = []
    for n in (64, 128, 256):
        d = np.broadcast_to(p["d"][0:1], (n, B, D))
        h = ode.ode_serial_scan(A, Bw, b, d, p["h0"], tend / n)
        errs.append(np.max(np.abs(h[n, 0] - ref)))
    assert errs[0] < 2e-2
    assert 1.8 < errs[0] / errs[1] < 2.2 and 1.8 < errs[1] / errs[2] < 2.2


def test_time_dependent_data_enters_at_the_point_stepped_to():
    """Row t-1 of d drives the step into point t: changing d_t leaves h_0..h_{t-1}
    untouched and changes h_t."""
    T, B, D, H = 12, 2, 3, 4
    p = random_ode(7, T, B, D, H)
    h = ode.ode_serial_scan(p["A"], p["Bw"], p["b"], p["d"], p["h0"], 0.25)
    d2 = p["d"].copy()
    d2[6] += 1.0                                   # d_7
    h2 = ode.ode_serial_scan(p["A"], p["Bw"], p["b"], d2, p["h0"], 0.25)
    assert np.array_equal(h[:7], h2[:7])
    assert np.max(np.abs(h[7] - h2[7])) > 1e-3


def test_residual_of_the_serial_solution_is_zero():
    T, B, D, H = 16, 2, 3, 4
    p = random_ode(9, T, B, D, H)
    h = ode.ode_serial_scan(p["A"], p["Bw"], p["b"], p["d"], p["h0"], 0.2)
    r = ode.ode_fine_residual(p["A"], p["Bw"], p["b"], p["d"], h, 0.2)
    assert np.max(np.abs(r)) == 0.0
    h[5] += 0.1
    r = ode.ode_fine_residual(p["A"], p["Bw"], p["b"], p["d"], h, 0.2)
    assert np.max(np.abs(r[4])) > 0.05 and np.max(np.abs(r[5])) > 1e-3
    assert np.max(np.abs(np.delete(r, (4, 5), axis=0))) == 0.0


@pytest.mark.parametrize("cf,levels,fcf", [(4, 2, True), (4, 2, False), (2, 4, True), (4, 3, True)])
def test_mgrit_reaches_the_serial_propagation_and_has_the_exactness_front(cf, levels, fcf):
    """MGRIT with any propagator is exact at the first k*cf points after k cycles
    (F-relaxation; FCF doubles the front) and reproduces the serial propagation after
    T/cf cycles; the serial solution is a fixed point with zero residual."""
    T, B, D, H, dt = 32, 2, 3, 6, 0.25
    p = random_ode(13, T, B, D, H)
    ser = ode.ode_serial_scan(p["A"], p["Bw"], p["b"], p["d"], p["h0"], dt)
    init = np.zeros((T + 1, B, H))
    n_it = T // cf
    h, res, its = ode.ode_mgrit_forward(p["A"], p["Bw"], p["b"], p["d"], p["h0"], init, dt, cf,
                                        levels, n_it, fine_relax_fcf=fcf, keep_iterates=True)
    assert _rel(h, ser) < 1e-13
    for k, hk in enumerate(its[:4], start=1):
        front = min(T, k * cf * (2 if fcf else 1))
        assert _rel(hk[:front + 1], ser[:front + 1]) < 1e-13
    # contraction well before the front arrives
    assert res[1] < 0.5 * res[0] and res[2] < 0.5 * res[1]
    h2, res2 = ode.ode_mgrit_forward(p["A"], p["Bw"], p["b"], p["d"], p["h0"], ser, dt, cf, levels,
                                     1, fine_relax_fcf=fcf)
    assert _rel(h2, ser) < 1e-14 and res2[0] < 1e-13


def test_one_level_is_the_serial_scan_and_residuals_fall_fast_for_small_steps():
    """levels = 1 is sequential propagation.  With a small step the two-level cycle
    reduces the residual by more than an order of magnitude per cycle, the behaviour
    the appendix's printed history shows (its weights are random, so only the rate is
    comparable)."""
    T, B, D, H, dt = 128, 1, 10, 10, 1.0 / 16
    p = random_ode(17, T, B, D, H, h0_random=False)
    ser = ode.ode_serial_scan(p["A"], p["Bw"], p["b"], p["d"], p["h0"], dt)
    h1, _ = ode.ode_mgrit_forward(p["A"], p["Bw"], p["b"], p["d"], p["h0"],
                                  np.zeros((T + 1, B, H)), dt, 4, 1, 1)
    assert _rel(h1, ser) < 1e-14
    _, res = ode.ode_mgrit_forward(p["A"], p["Bw"], p["b"], p["d"], p["h0"],
                                   np.zeros((T + 1, B, H)), dt, 4, 2, 5)
    for a, bb in zip(res[:-1], res[1:]):
        assert bb < a / 10.0


def test_two_level_rate_is_that_of_the_printed_history():
    """The appendix prints the residuals of eight two-level cycles on this ODE at its
    defaults (dimension 10, 128 steps): about 1.9 digits per cycle.  The values depend on
    the random weights by the paper's own statement and the integrator is a reading, so
    only the rate is compared, loosely (tests/golden/two_level_demo_residuals.txt)."""
    rows = [l.split() for l in open(os.path.join(GOLDEN, "two_level_demo_residuals.txt"))
            if l.strip() and not l.startswith("#")]
    paper_rate = np.mean(np.diff(np.log10([float(r[2]) for r in rows])))
    T, B, D, H = 128, 1, 10, 10
    p = random_ode(0, T, B, D, H, h0_random=False)
    _, res = ode.ode_mgrit_forward(p["A"], p["Bw"], p["b"], p["d"], p["h0"],
                                   np.zeros((T + 1, B, H)), 1.0 / 16, 4, 2, 8)
    res = np.array(res)
    rate = np.mean(np.diff(np.log10(res[res > 1e-14])))
    assert rate < -1.0 and abs(rate - paper_rate) < 1.0, (rate, paper_rate)
