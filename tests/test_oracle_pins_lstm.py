"""Pins of the LSTM oracle (no GPU).  The implicit LSTM step is this build's derivation (the
paper names the extension only), so the pins are: a library LSTM for the explicit step of size 1,
the defining implicit equations, the common ODE limit of both steps, closed forms that show each
level's step size, and the propagator-independent properties of the cycle."""
import numpy as np
import pytest
import torch

from oracle import lstm_oracle as lo
from oracle import mgrit_gru_oracle as orc
from synthetic_inputs import random_lstm


def _P(d):
    return d["W"], d["U"], d["b_i"], d["b_h"]


def test_explicit_step_of_size_one_is_the_library_lstm():
    T, B, D, H = 7, 3, 5, 4
    d = random_lstm(3, T, B, D, H)
    lstm = torch.nn.LSTM(D, H, num_layers=1, bias=True, batch_first=False).double()
    with torch.no_grad():
        lstm.weight_ih_l0.copy_(torch.from_numpy(d["W"]).double())
        lstm.weight_hh_l0.copy_(torch.from_numpy(d["U"]).double())
        lstm.bias_ih_l0.copy_(torch.from_numpy(d["b_i"]).double())
        lstm.bias_hh_l0.copy_(torch.from_numpy(d["b_h"]).double())
        h0 = torch.from_numpy(d["u0"][:, :H]).double()[None]
        c0 = torch.from_numpy(d["u0"][:, H:]).double()[None]
        out, (hT, cT) = lstm(torch.from_numpy(d["x"]).double(), (h0, c0))
    u = lo.lstm_serial_scan(*_P(d), d["x"], d["u0"], propagator=lo.CLASSIC)
    assert np.allclose(u[1:, :, :H], out.numpy(), rtol=0, atol=1e-13)
    assert np.allclose(u[-1, :, H:], cT[0].numpy(), rtol=0, atol=1e-13)


@pytest.mark.parametrize("gamma", [1.0, 4.0, 16.0])
def test_implicit_step_satisfies_its_defining_equations(gamma):
    """(1 + gamma (1-f)) c' = c + gamma i g  and  (1 + gamma) h' = h + gamma o tanh(c'), with the
    gates at (x_t, h_{t-1}); the gates are pinned by the library LSTM above."""
    H = 5
    d = random_lstm(5, 1, 4, 6, H)
    P = orc.input_projection(d["W"], d["b_i"], d["x"])[0]
    u = d["u0"].astype(np.float64)
    U, b_h = d["U"].astype(np.float64), d["b_h"].astype(np.float64)
    un = lo.lstm_phi(gamma, P, u, U, b_h, lo.IMPLICIT)
    i, f, g, o = lo.lstm_gates(P, u[:, :H], U, b_h)
    assert np.allclose((1 + gamma * (1 - f)) * un[:, H:], u[:, H:] + gamma * i * g, atol=1e-13)
    assert np.allclose((1 + gamma) * un[:, :H], u[:, :H] + gamma * o * np.tanh(un[:, H:]), atol=1e-13)


@pytest.mark.parametrize("prop", [lo.IMPLICIT, lo.CLASSIC])
def test_both_steps_are_consistent_with_the_same_ode(prop):
    """(Phi_gamma(u) - u)/gamma -> (-h + o tanh(c), -(1-f) c + i g) as gamma -> 0."""
    H = 6
    d = random_lstm(7, 1, 3, 4, H)
    P = orc.input_projection(d["W"], d["b_i"], d["x"])[0]
    u = d["u0"].astype(np.float64)
    U, b_h = d["U"].astype(np.float64), d["b_h"].astype(np.float64)
    i, f, g, o = lo.lstm_gates(P, u[:, :H], U, b_h)
    rhs = np.concatenate([-u[:, :H] + o * np.tanh(u[:, H:]), -(1 - f) * u[:, H:] + i * g], axis=-1)
    gm = 1e-7
    assert np.allclose((lo.lstm_phi(gm, P, u, U, b_h, prop) - u) / gm, rhs, atol=1e-6)


@pytest.mark.parametrize("cf,levels", [(3, 2), (3, 3), (4, 3)])
@pytest.mark.parametrize("prop", [lo.IMPLICIT, lo.CLASSIC])
def test_level_step_size_shows_in_the_decay_of_a_zero_weight_problem(cf, levels, prop):
    """All weights and biases zero: i = f = o = 1/2, g = 0, so c' = c / (1 + gamma/2) (implicit) or
    c (1 - gamma/2) (explicit) whatever h is.  After one cycle from a zero guess the cell half of
    the iterate decays, from point 3 of every level on, by that level's factor with gamma = cf^l
    (Sec. 3.3) -- see the GRU pin of the same name for why."""
    T, B, D, H = 6 * cf ** (levels - 1), 2, 3, 4
    rng = np.random.default_rng(9)
    z4 = np.zeros(4 * H)
    W, U = np.zeros((4 * H, D)), np.zeros((4 * H, H))
    x = rng.standard_normal((T, B, D))
    u0 = np.concatenate([rng.standard_normal((B, H)), 1.0 + rng.random((B, H))], axis=-1)
    u, _ = lo.mgrit_lstm_forward(W, U, z4, z4, x, u0, np.zeros((T + 1, B, 2 * H)), cf, levels, 1,
                                 propagator=prop)
    c = u[:, :, H:]
    checked = 0
    for l in range(levels):
        s = cf ** l
        fac = 1.0 / (1.0 + s / 2.0) if prop == lo.IMPLICIT else 1.0 - s / 2.0
        for k in range(3, T // s + 1):
            if l < levels - 1 and k % cf == 0:
                continue
            assert np.allclose(c[k * s] / c[(k - 1) * s], fac, rtol=1e-12, atol=0), (l, k)
            checked += 1
    assert checked > levels


def test_one_level_and_cf1_reproduce_the_serial_scan():
    d = random_lstm(1, 16, 2, 3, 4)
    us = lo.lstm_serial_scan(*_P(d), d["x"], d["u0"])
    z = np.zeros_like(us)
    assert np.array_equal(lo.mgrit_lstm_forward(*_P(d), d["x"], d["u0"], z, 4, 1, 1)[0], us)
    assert np.allclose(lo.mgrit_lstm_forward(*_P(d), d["x"], d["u0"], z, 1, 2, 1)[0], us, atol=1e-14)


@pytest.mark.parametrize("fcf", [False, True])
@pytest.mark.parametrize("levels", [2, 3])
def test_exactness_front_fixed_point_and_convergence(fcf, levels):
    cf = 2
    T = 8 * cf ** (levels - 1)
    d = random_lstm(11, T, 2, 3, 4)
    us = lo.lstm_serial_scan(*_P(d), d["x"], d["u0"])
    z = np.zeros_like(us)
    _, res, its = lo.mgrit_lstm_forward(*_P(d), d["x"], d["u0"], z, cf, levels, T // cf,
                                        fine_relax_fcf=fcf, keep_iterates=True)
    for i, u in enumerate(its, start=1):
        front = min((i + 1) * cf - 1, T)
        assert np.allclose(u[:front + 1], us[:front + 1], rtol=0, atol=1e-12), i
    assert np.allclose(its[-1], us, rtol=0, atol=1e-12)
    u, r = lo.mgrit_lstm_forward(*_P(d), d["x"], d["u0"], us, cf, levels, 1, fine_relax_fcf=fcf)
    assert np.allclose(u, us, atol=1e-13) and r[0] < 1e-12


def test_single_interval_fcf_converges_in_one_cycle():
    """cf = T: FC-relaxation propagates exactly over the only interval, so one cycle gives the
    serial solution whatever the coarse level does."""
    T, cf = 6, 6
    d = random_lstm(13, T, 2, 3, 4)
    us = lo.lstm_serial_scan(*_P(d), d["x"], d["u0"])
    u, _ = lo.mgrit_lstm_forward(*_P(d), d["x"], d["u0"], np.zeros_like(us), cf, 2, 1)
    assert np.allclose(u, us, atol=1e-13)


@pytest.mark.parametrize("T,cf,levels,fcf", [(36, 3, 3, True), (32, 2, 4, True), (48, 4, 3, False)])
@pytest.mark.parametrize("prop", [lo.IMPLICIT, lo.CLASSIC])
def test_cell_half_of_the_cycle_on_an_affine_problem_equals_dense_linear_algebra(T, cf, levels, fcf,
                                                                                 prop):
    """With U = 0 the gates depend on x alone and the cell recurrence is affine and independent
    of h: c' = a c + beta with a = 1/(1 + gamma (1-f)), beta = gamma i g / (1 + gamma (1-f))
    (implicit) or a = 1 - gamma (1-f), beta = gamma i g (explicit); f and i g are read off a
    library LSTM cell (c' = f c + i g: slope and intercept in c).  Level l uses gamma = cf^l and
    the inputs x_{k cf^l}; coarse levels relax with FCF.  The cell half of the oracle's iterates
    must equal the cycle of Alg. 2 done by dense solves (helpers of the GRU pin file)."""
    from test_oracle_pins import _dense_cycle, _level_matrix
    B, D, H = 2, 3, 3
    d = random_lstm(17, T, B, D, H, scale=0.7)
    d["U"][:] = 0.0
    cell = torch.nn.LSTMCell(D, H).double()
    with torch.no_grad():
        cell.weight_ih.copy_(torch.from_numpy(d["W"]).double())
        cell.weight_hh.zero_()
        cell.bias_ih.copy_(torch.from_numpy(d["b_i"]).double())
        cell.bias_hh.copy_(torch.from_numpy(d["b_h"]).double())
        x = torch.from_numpy(d["x"]).double().reshape(T * B, D)
        zz = torch.zeros(T * B, H, dtype=torch.float64)
        c_at0 = cell(x, (zz, zz))[1]
        c_at1 = cell(x, (zz, torch.ones_like(zz)))[1]
    f = (c_at1 - c_at0).reshape(T, B, H).numpy()
    ig = c_at0.reshape(T, B, H).numpy()
    m = B * H
    As, betas = [], []
    for l in range(levels):
        g = float(cf ** l)
        idx = np.arange(1, T // cf ** l + 1) * cf ** l - 1
        fl, igl = f[idx].reshape(-1, m), ig[idx].reshape(-1, m)
        if prop == lo.IMPLICIT:
            a, beta = 1.0 / (1.0 + g * (1.0 - fl)), g * igl / (1.0 + g * (1.0 - fl))
        else:
            a, beta = 1.0 - g * (1.0 - fl), g * igl
        As.append(_level_matrix([np.diag(ak) for ak in a]))
        betas.append(beta)
    c0 = d["u0"][:, H:].astype(np.float64)
    b0 = np.concatenate([c0.ravel(), betas[0].ravel()])
    u = np.zeros((T + 1) * m)
    u[:m] = c0.ravel()
    _, _, its = lo.mgrit_lstm_forward(*_P(d), d["x"], d["u0"], np.zeros((T + 1, B, 2 * H)), cf,
                                      levels, 3, fine_relax_fcf=fcf, propagator=prop,
                                      keep_iterates=True)
    for it in range(3):
        u = _dense_cycle(As, 0, u, b0, cf, fcf, m)
        want = its[it][:, :, H:].reshape(-1)
        assert np.max(np.abs(u - want)) <= 1e-12 * max(1.0, np.max(np.abs(want))), it
