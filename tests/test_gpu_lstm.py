"""Parity of the HIP path with the CPU oracle for the LSTM step behind the forward MGRIT cycle:
serial propagation and every MGRIT iterate of the state pair (h | c), element by element on the
same seeded inputs, fp32 bar max|gpu - oracle| / max|oracle| <= 1e-5; residual norms to 1e-4
relative plus the fp32 rounding floor."""
import numpy as np
import pytest
import torch

import paper_2203_04738_amd as mg
from oracle import lstm_oracle as lo
from paper_2203_04738_amd.binding import MgritGruCfg
from synthetic_inputs import WORKLOADS, make_lstm_inputs, random_lstm

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOL = 1e-5


def _rel(a, b):
    a = np.asarray(a, dtype=np.float64)
    assert np.all(np.isfinite(a))
    return float(np.max(np.abs(a - b)) / max(np.max(np.abs(b)), 1e-30))


def _P(d):
    return d["W"], d["U"], d["b_i"], d["b_h"]


class LstmRun:
    def __init__(self, d, cf=1, levels=1, fine_relax=1, propagator=0):
        self.t = {k: torch.from_numpy(v).to(DEV) for k, v in d.items()}
        self.T, self.B, self.D = d["x"].shape
        self.H = d["U"].shape[1]
        self.kw = dict(cf=cf, levels=levels, fine_relax=fine_relax, propagator=propagator)
        self.ws = torch.empty(mg.mgrit_lstm_workspace_bytes(self.cfg(64)), dtype=torch.uint8,
                              device=DEV)

    def cfg(self, iters=1):
        return MgritGruCfg(self.T, self.B, self.D, self.H, iters=iters, **self.kw)

    def _p(self):
        t = self.t
        return t["W"], t["U"], t["b_i"], t["b_h"], t["x"], t["u0"]

    def serial(self):
        u = torch.full((self.T + 1, self.B, 2 * self.H), float("nan"), device=DEV)
        mg.lstm_serial_scan(self.cfg(), *self._p(), u, self.ws)
        torch.cuda.synchronize()
        return u.cpu().numpy()

    def iterates(self, iters, per_call=1, u_init=None):
        u = torch.zeros(self.T + 1, self.B, 2 * self.H, device=DEV)
        if u_init is not None:
            u.copy_(torch.from_numpy(np.ascontiguousarray(u_init, dtype=np.float32)))
        its, norms, done = [], [], 0
        while done < iters:
            n = min(per_call, iters - done)
            res = torch.full((n,), float("nan"), device=DEV)
            mg.mgrit_lstm_forward(self.cfg(n), *self._p(), u, res, self.ws)
            torch.cuda.synchronize()
            its.append(u.cpu().numpy().copy())
            norms += res.cpu().numpy().tolist()
            done += n
        return its, norms


# sizes: few-row and tile kernels, several tiles and ragged tails in rows and columns
SERIAL_CASES = [
    # T, B, D, H
    (9, 1, 4, 4),          # smallest widths
    (33, 3, 12, 20),       # ragged everything, few rows
    (17, 70, 24, 72),      # 64 x 64 tiles with tails (K-split 32 x 32 tiles below 128 workgroups)
    (6, 300, 40, 136),     # several row tiles, ragged columns
    (3, 1100, 16, 520),    # 128-row tiles of eight waves, ragged rows and columns
]


@pytest.mark.parametrize("prop", [lo.IMPLICIT, lo.CLASSIC])
@pytest.mark.parametrize("T,B,D,H", SERIAL_CASES)
def test_serial_propagation_matches_the_oracle(T, B, D, H, prop):
    d = random_lstm(21, T, B, D, H, scale=0.3)
    got = LstmRun(d, propagator=prop).serial()
    want = lo.lstm_serial_scan(*_P(d), d["x"], d["u0"], propagator=prop)
    assert _rel(got, want) <= TOL
    # both halves on their own scale
    assert _rel(got[:, :, :H], want[:, :, :H]) <= TOL
    assert _rel(got[:, :, H:], want[:, :, H:]) <= TOL


HIERARCHIES = [
    # T, B, D, H, cf, levels, fcf
    (64, 2, 16, 32, 4, 2, 1),
    (64, 2, 16, 32, 4, 2, 0),
    (96, 5, 24, 40, 4, 3, 1),      # ragged widths, three levels
    (64, 3, 8, 12, 2, 4, 1),       # four levels
    (54, 4, 8, 16, 3, 3, 1),       # cf = 3
    (16, 2, 8, 8, 1, 2, 1),        # cf = 1: one cycle is the serial scan
    (64, 40, 16, 72, 8, 2, 1),     # tile kernels on level 0 (320 rows), few rows on level 1
    (32, 300, 16, 136, 4, 2, 1),   # 128-row tiles on level 0, 64-row tiles on level 1
]


@pytest.mark.parametrize("T,B,D,H,cf,levels,fcf", HIERARCHIES)
def test_every_mgrit_iterate_and_residual_norm(T, B, D, H, cf, levels, fcf):
    d = random_lstm(31, T, B, D, H, scale=0.3)
    run = LstmRun(d, cf=cf, levels=levels, fine_relax=fcf)
    its, norms = run.iterates(3)
    _, rres, rits = lo.mgrit_lstm_forward(*_P(d), d["x"], d["u0"], np.zeros((T + 1, B, 2 * H)), cf,
                                          levels, 3, fine_relax_fcf=bool(fcf), keep_iterates=True)
    for i in range(3):
        assert _rel(its[i], rits[i]) <= TOL, i
        assert abs(norms[i] - rres[i]) <= 1e-4 * rres[i] + 2e-6 * np.sqrt(T), i
    # several cycles in one call give the same iterate as one cycle per call
    its2, norms2 = run.iterates(3, per_call=3)
    assert _rel(its2[-1], rits[-1]) <= TOL
    for a, b in zip(norms2, rres):
        assert abs(a - b) <= 1e-4 * b + 2e-6 * np.sqrt(T)


def test_classic_step_cycle_and_convergence_to_the_serial_scan():
    T, B, D, H, cf, levels = 32, 3, 8, 16, 2, 3
    d = random_lstm(41, T, B, D, H, scale=0.3)
    # explicit step: two levels, so that the coarse step size (2) stays where the explicit step
    # does not amplify (a factor 1 - gamma on h; on deeper levels every cycle multiplies rounding
    # differences by |1 - gamma| per coarse step and an element-wise comparison says nothing)
    # (... and a short sequence: with step size 2 the factor on h is -1, rounding differences
    # neither grow nor decay along the coarse level)
    dc = random_lstm(41, 16, B, D, H, scale=0.3)
    run = LstmRun(dc, cf=cf, levels=2, propagator=lo.CLASSIC)
    its, _ = run.iterates(2)
    _, _, rits = lo.mgrit_lstm_forward(*_P(dc), dc["x"], dc["u0"], np.zeros((17, B, 2 * H)), cf,
                                       2, 2, propagator=lo.CLASSIC, keep_iterates=True)
    for a, b in zip(its, rits):
        assert _rel(a, b) <= TOL
    run_i = LstmRun(d, cf=cf, levels=levels)
    its, norms = run_i.iterates(T // cf)
    assert _rel(its[-1], run_i.serial()) <= 2e-6
    assert norms[-1] <= 1e-4 * norms[0]
    # the serial solution is a fixed point of the cycle
    us = lo.lstm_serial_scan(*_P(d), d["x"], d["u0"])
    fp, fn = run_i.iterates(1, u_init=us)
    assert _rel(fp[-1], us) <= TOL and fn[0] <= 1e-4


@pytest.mark.timeout(600)
def test_full_size_solve_follows_sampled_batch_elements():
    """Sizes of the training-step workload (T = 2048, B = 32, D = 1024, H = 512, cf = 4, three
    levels, two cycles): the oracle follows the first and the last batch element over every
    time step and both cycles (batch elements never interact)."""
    wl = WORKLOADS["C3"]
    d = make_lstm_inputs(wl)
    run = LstmRun(d, cf=wl.cf, levels=wl.levels)
    bs = [0, wl.B - 1]
    _, _, rits = lo.mgrit_lstm_forward(d["W"], d["U"], d["b_i"], d["b_h"],
                                       np.ascontiguousarray(d["x"][:, bs]), d["u0"][bs],
                                       np.zeros((wl.T + 1, 2, 2 * wl.H)), wl.cf, wl.levels, 2,
                                       keep_iterates=True)
    its, _ = run.iterates(2)
    for i in range(2):
        assert _rel(its[i][:, bs], rits[i]) <= TOL, i
    its2, _ = run.iterates(2, per_call=2)
    assert _rel(its2[-1][:, bs], rits[-1]) <= TOL
    us = run.serial()
    rs = lo.lstm_serial_scan(d["W"], d["U"], d["b_i"], d["b_h"], np.ascontiguousarray(d["x"][:, bs]),
                             d["u0"][bs])
    assert _rel(us[:, bs], rs) <= TOL
