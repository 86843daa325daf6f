"""Parity of the entry points for a loss on every state (source term in the adjoint
recurrence), the input gradients dL/dx and a two-layer stack built from them, against
the CPU oracle, element by element, through the C ABI.  Same bars as the other
parity tests: fp32 path 1e-5, bf16-input path 2e-2 (and the 1e-4 the operand split
is expected to reach), max|gpu - oracle| / max|oracle| per tensor."""
import numpy as np
import pytest

from oracle import mgrit_gru_oracle as orc
from synthetic_inputs import WORKLOADS, make_inputs, random_small, round_to_bf16

pytestmark = pytest.mark.gpu

TOL = 1e-5
TOL_BF16 = 2e-2
TIGHT_BF16 = 1e-4
NAMES = ("w", "dW", "dU", "db_i", "db_h", "dx")


@pytest.fixture(scope="module")
def gh():
    import gpu_harness
    return gpu_harness


def _P(d):
    return d["W"], d["U"], d["b_i"], d["b_h"]


def _source(seed, T, B, H, scale=0.3):
    """Seeded dL/dh_t for every t (row 0 included: a loss may depend on h_0)."""
    return (scale * np.random.default_rng(seed).standard_normal((T + 1, B, H))).astype(np.float32)


@pytest.mark.parametrize("prop", [orc.IMPLICIT, orc.CLASSIC])
@pytest.mark.parametrize("shape", [(13, 3, 20, 36), (5, 1, 4, 4), (9, 70, 132, 12), (6, 40, 260, 136)])
def test_serial_backward_with_source_and_dx_ragged_shapes(gh, prop, shape):
    T, B, D, H = shape
    d = random_small(500 + H, T, B, D, H, scale=0.3)
    src = _source(H, T, B, H)
    h = orc.serial_scan(*_P(d), d["x"], d["h0"], prop).astype(np.float32)
    ref = orc.serial_bptt_steps(*_P(d), d["x"], h, src, prop)
    got = gh.GpuRun(d, propagator=prop).serial_backward_steps(h, src)
    for name, g, r in zip(NAMES, got, ref):
        assert gh.rel_err(g, r) <= TOL, name


def test_source_that_is_zero_except_at_T_reproduces_the_terminal_entry_point(gh):
    T, B, D, H = 24, 3, 20, 36
    d = random_small(77, T, B, D, H, scale=0.3)
    src = np.zeros((T + 1, B, H), dtype=np.float32)
    src[T] = d["dL_dhT"]
    h = orc.serial_scan(*_P(d), d["x"], d["h0"]).astype(np.float32)
    run = gh.GpuRun(d, cf=4, levels=2)
    a = run.serial_backward(h)
    b = run.serial_backward_steps(h, src, want_dx=False)
    for u, v in zip(a, b):
        assert np.array_equal(u, v)
    ia, _, ga = run.backward_iterates(h, 2)
    ib, _, gb = run.backward_steps_iterates(h, src, 2, want_dx=False)
    for u, v in zip(ia + list(ga), ib + list(gb)):
        assert np.array_equal(u, v)


def test_zero_guess_flag_with_a_source_that_is_zero_below_T(gh):
    """The top layer of a stack whose loss reads h_T only: its source term is zero except in
    row T, it goes through the step-loss entry point for its dx, and may declare the zero
    guess.  Same bar against the oracle, and agreement to rounding with the undeclared call."""
    from paper_2203_04738_amd.binding import MGRIT_ZERO_ADJOINT_GUESS
    T, B, D, H, cf, levels = 64, 5, 24, 40, 4, 3
    d = random_small(78, T, B, D, H, scale=0.3)
    src = np.zeros((T + 1, B, H), dtype=np.float32)
    src[T] = d["dL_dhT"]
    h = orc.serial_scan(*_P(d), d["x"], d["h0"]).astype(np.float32)
    out = orc.mgrit_backward(*_P(d), d["x"], h, None, np.zeros((T + 1, B, H)), cf, levels, 2,
                             dL_dh=src)
    run = gh.GpuRun(d, cf=cf, levels=levels)
    ia, _, ga = run.backward_steps_iterates(h, src, 2, per_call=2)
    ib, _, gb = run.backward_steps_iterates(h, src, 2, per_call=2,
                                            first_call_flags=MGRIT_ZERO_ADJOINT_GUESS)
    for u, v in zip(ia + list(ga), ib + list(gb)):
        assert gh.rel_err(v, u) <= 2e-6
    for name, g, r in zip(NAMES, [ib[-1]] + list(gb), (out[0],) + tuple(out[2:7])):
        assert gh.rel_err(g, r) <= TOL, name


def _check_mgrit_steps(gh, d, src, cf, levels, iters, fcf=True, prop=orc.IMPLICIT, per_call=1):
    T, B = d["x"].shape[:2]
    H = d["U"].shape[1]
    h, _ = orc.mgrit_forward(*_P(d), d["x"], d["h0"], np.zeros((T + 1, B, H)), cf, levels, 2,
                             fine_relax_fcf=fcf, propagator=prop)
    h = h.astype(np.float32)                     # an inexact forward iterate, as in training
    out = orc.mgrit_backward(*_P(d), d["x"], h, None, np.zeros((T + 1, B, H)), cf, levels, iters,
                             fine_relax_fcf=fcf, propagator=prop, keep_iterates=True, dL_dh=src)
    rits, rres = out[-1], out[1]
    run = gh.GpuRun(d, cf=cf, levels=levels, fine_relax=int(fcf), propagator=prop)
    gits, gres, grads = run.backward_steps_iterates(h, src, iters, per_call=per_call)
    if per_call == 1:
        for i, (g, r) in enumerate(zip(gits, rits)):
            assert gh.rel_err(g, r) <= TOL, ("w", i)
    else:
        assert gh.rel_err(gits[-1], rits[-1]) <= TOL
    assert np.allclose(gres, rres, rtol=1e-4, atol=1e-6 * max(rres))
    for name, g, r in zip(NAMES[1:], grads, out[2:7]):
        assert gh.rel_err(g, r) <= TOL, name


@pytest.mark.parametrize("cf,levels,fcf", [(4, 2, True), (4, 2, False), (2, 3, True), (3, 3, True)])
def test_mgrit_backward_with_source_per_iterate(gh, cf, levels, fcf):
    T = 6 * cf ** (levels - 1)
    d = random_small(600 + cf, T, 3, 20, 36, scale=0.3)
    _check_mgrit_steps(gh, d, _source(cf, T, 3, 36), cf, levels, 3, fcf=fcf)


def test_mgrit_backward_with_source_c1_and_classic(gh):
    wl = WORKLOADS["C1"]
    d = make_inputs(wl)
    src = _source(3, wl.T, wl.B, wl.H, scale=0.1)
    _check_mgrit_steps(gh, d, src, wl.cf, wl.levels, wl.bwd_iters)
    # explicit (Classic) coarse step: cf = 2 keeps gamma inside its stability range
    # (Eq. 13); with gamma = 4 the coarse propagation amplifies fp32 rounding
    _check_mgrit_steps(gh, d, src, 2, 2, 2, prop=orc.CLASSIC)


def test_mgrit_backward_with_source_several_cycles_per_call_and_mfma_rows(gh):
    # 96 intervals x 40 batch rows per launch: the MFMA tile kernels, ragged in rows and K
    T, B, D, H = 384, 40, 72, 100
    d = random_small(91, T, B, D, H, scale=0.2)
    _check_mgrit_steps(gh, d, _source(8, T, B, H, scale=0.1), 4, 3, 2, per_call=2)


@pytest.mark.parametrize("form", ["bf16", "bf16s2"])
def test_bf16_backward_with_source_and_dx(gh, form):
    T, B, D, H = 48, 3, 24, 40
    TIGHT_BF16 = 1e-4 if form == "bf16s2" else TOL_BF16
    d = dict(random_small(43, T, B, D, H, scale=0.3))
    for k in ("x", "W", "U"):
        d[k] = round_to_bf16(d[k])      # the oracle sees exactly the stored bf16 values
    src = _source(5, T, B, H)
    h = orc.serial_scan(*_P(d), d["x"], d["h0"]).astype(np.float32)
    ref = orc.serial_bptt_steps(*_P(d), d["x"], h, src)
    run = gh.GpuRun(d, cf=4, levels=2, dtype=form)
    got = run.serial_backward_steps(h, src)
    for name, g, r in zip(NAMES, got, ref):
        e = gh.rel_err(g, r)
        assert e <= TOL_BF16 and e <= TIGHT_BF16, (name, e)
    out = orc.mgrit_backward(*_P(d), d["x"], h, None, np.zeros_like(h), 4, 2, 2,
                             keep_iterates=True, dL_dh=src)
    gits, _, grads = run.backward_steps_iterates(h, src, 2)
    for i, (g, r) in enumerate(zip(gits, out[-1])):
        e = gh.rel_err(g, r)
        assert e <= TOL_BF16 and e <= TIGHT_BF16, ("w", i, e)
    for name, g, r in zip(NAMES[1:], grads, out[2:7]):
        e = gh.rel_err(g, r)
        assert e <= TOL_BF16 and e <= TIGHT_BF16, (name, e)


def test_two_layer_stack_forward_and_backward(gh):
    """Layer 2 reads the states of layer 1; the loss sits on every state of layer 2;
    dL/dx of layer 2 is the source term of layer 1.  2 forward cycles, 1 backward
    cycle per layer, the iteration counts the paper trains with (Sec. 4)."""
    T, B, D, H, cf, levels = 64, 5, 24, 36, 4, 3
    d1 = random_small(701, T, B, D, H, scale=0.3)
    d2 = random_small(702, T, B, H, H, scale=0.3)
    params = [_P(d1), _P(d2)]
    h0s = [d1["h0"], d2["h0"]]
    src = _source(11, T, B, H)
    src[0] = 0.0
    zeros = np.zeros((T + 1, B, H))

    def fwd(j, W, U, bi, bh, xin, h0):
        return orc.mgrit_forward(W, U, bi, bh, xin, h0, zeros, cf, levels, 2)[0].astype(np.float32)

    def bwd(j, W, U, bi, bh, xin, h, s):
        out = orc.mgrit_backward(W, U, bi, bh, xin, h, None, zeros, cf, levels, 1, dL_dh=s)
        return (out[0],) + tuple(out[2:7])

    rh = orc.stacked_forward(params, d1["x"], h0s, fwd)
    rb = orc.stacked_backward(params, d1["x"], rh, src, bwd)

    # (1) every call on its own, to the bar of a single solve: the HIP path is handed what the
    # oracle's stack hands down (layer 1's states as layer 2's input, layer 2's dL/dx as layer
    # 1's source term, the oracle's iterates as linearisation states), rounded to fp32
    f32 = lambda a: np.ascontiguousarray(a, dtype=np.float32)
    solo = []
    for j, dj in enumerate((d1, d2)):
        dd = dict(dj)
        dd["x"] = f32(d1["x"] if j == 0 else rh[0][1:])
        run = gh.GpuRun(dd, cf=cf, levels=levels)
        its, _ = run.forward_iterates(2, per_call=2)
        solo.append(run)
        assert gh.rel_err(its[-1], rh[j]) <= TOL, ("h", j)
    s_top = src
    for j in (1, 0):
        s_in = s_top
        if j == 0:
            s_in = np.zeros((T + 1, B, H), dtype=np.float32)
            s_in[1:] = rb[1][5]
        its, _, grads = solo[j].backward_steps_iterates(f32(rh[j]), s_in, 1)
        for name, g, r in zip(NAMES, (its[-1],) + grads, rb[j]):
            assert gh.rel_err(g, r) <= TOL, (name, j)

    # (2) the stack end to end on the HIP path's own intermediates: layer 2's states and
    # gradients carry the rounding of layer 1's solve as well, and layer 1's adjoint that of
    # layer 2's dL/dx: two solves' rounding, hence twice the bar of one
    runs, gh_states = [], []
    xin = d1["x"]
    for j, dj in enumerate((d1, d2)):
        dd = dict(dj)
        dd["x"] = np.ascontiguousarray(xin, dtype=np.float32)
        run = gh.GpuRun(dd, cf=cf, levels=levels)
        its, _ = run.forward_iterates(2, per_call=2)
        runs.append(run)
        gh_states.append(its[-1])
        xin = its[-1][1:]
        assert gh.rel_err(its[-1], rh[j]) <= (1 + j) * TOL, ("h", j)
    s = src
    for j in (1, 0):
        its, _, grads = runs[j].backward_steps_iterates(gh_states[j], s, 1)
        got = (its[-1],) + grads
        for name, g, r in zip(NAMES, got, rb[j]):
            assert gh.rel_err(g, r) <= 2 * TOL, (name, j)
        if j > 0:
            s = np.zeros((T + 1, B, H), dtype=np.float32)
            s[1:] = got[5]


@pytest.mark.parametrize("dtype", ["fp32", "bf16", "bf16s2", "fp32x3"])
def test_step_loss_backward_reusing_projection_and_coefficients(gh, dtype):
    """The call sequence of the stacked training step: the forward solve keeps the
    projection and the coefficients of its closing relaxation in the workspace, the
    backward solve with a loss on every state reuses both."""
    import torch
    import paper_2203_04738_amd as mg
    from paper_2203_04738_amd.binding import (MGRIT_KEEP_COEFFS, MGRIT_REUSE_COEFFS,
                                              MGRIT_REUSE_PROJECTION)
    T, B, D, H, cf, levels = 96, 5, 24, 40, 4, 3
    d = dict(random_small(47, T, B, D, H, scale=0.3))
    tol, tight = (TOL_BF16, TIGHT_BF16 if dtype == "bf16s2" else TOL_BF16) if dtype.startswith("bf16") else (TOL, TOL)
    if dtype.startswith("bf16"):
        for k in ("x", "W", "U"):
            d[k] = round_to_bf16(d[k])
    src = _source(13, T, B, H)
    run = gh.GpuRun(d, cf=cf, levels=levels, dtype=dtype)
    dev = gh.DEV
    h = torch.zeros(T + 1, B, H, device=dev)
    mg.mgrit_gru_forward(run.cfg(2, MGRIT_KEEP_COEFFS), *run._p(), run.t["h0"], h, None, run.ws)
    w = torch.zeros(T + 1, B, H, device=dev)
    g = run._grads()
    dx = torch.full((T, B, D), float("nan"), device=dev)
    mg.mgrit_gru_backward_steps(run.cfg(1, MGRIT_REUSE_PROJECTION | MGRIT_REUSE_COEFFS), *run._p(),
                                h, run._dev(src), w, None, *g, dx, run.ws)
    torch.cuda.synchronize()
    hh = h.cpu().numpy()
    rh, _ = orc.mgrit_forward(*_P(d), d["x"], d["h0"], np.zeros((T + 1, B, H)), cf, levels, 2)
    e = gh.rel_err(hh, rh)
    assert e <= tol and e <= tight, e
    out = orc.mgrit_backward(*_P(d), d["x"], hh, None, np.zeros((T + 1, B, H)), cf, levels, 1,
                             dL_dh=src)
    got = (w.cpu().numpy(),) + tuple(a.cpu().numpy() for a in g) + (dx.cpu().numpy(),)
    for name, a, r in zip(NAMES, got, (out[0],) + tuple(out[2:7])):
        e = gh.rel_err(a, r)
        assert e <= tol and e <= tight, (name, e)
