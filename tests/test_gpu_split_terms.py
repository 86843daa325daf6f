"""Parity of the third operand form (MGRIT_F32_BF16X3: fp32 inputs and weights, the tile
kernels contract them as three bf16 terms each on the bf16 matrix pipe) with the CPU oracle,
element by element, through the C ABI.  It is an fp32 path: same inputs, same oracle and
the same bar as the fp32 form, max|gpu - oracle| / max|oracle| <= 1e-5 per tensor.  The
shapes below put more than 64 rows into every launch, so that the tile kernels (and not the
few-row kernels, which are shared with the fp32 form) do the work."""
import numpy as np
import pytest

from oracle import mgrit_gru_oracle as orc
from synthetic_inputs import WORKLOADS, make_inputs, random_small

pytestmark = pytest.mark.gpu

TOL = 1e-5
FORM = "fp32x3"


@pytest.fixture(scope="module")
def gh():
    import gpu_harness
    return gpu_harness


def _P(d):
    return d["W"], d["U"], d["b_i"], d["b_h"]


def _zeros(d):
    T, B = d["x"].shape[:2]
    return np.zeros((T + 1, B, d["U"].shape[1]))


@pytest.mark.parametrize("prop", [orc.IMPLICIT, orc.CLASSIC])
@pytest.mark.parametrize("shape", [(6, 70, 16, 136), (9, 130, 8, 24), (5, 300, 40, 72), (6, 70, 8, 8)])
def test_serial_scan_and_bptt(gh, prop, shape):
    """Few tiles per launch: the K-split tile configuration, ragged rows, columns and K
    (136 = 4 x 32 + 8, 3 x 24 = 72 = 2 x 32 + 8), down to the smallest widths the form takes
    (H = D = 8: a quarter of one K-slice)."""
    T, B, D, H = shape
    d = random_small(900 + H, T, B, D, H, scale=0.3)
    ref = orc.serial_scan(*_P(d), d["x"], d["h0"], prop)
    run = gh.GpuRun(d, propagator=prop, dtype=FORM)
    assert gh.rel_err(run.serial_scan(), ref) <= TOL
    h = ref.astype(np.float32)
    rb = orc.serial_bptt(*_P(d), d["x"], h, d["dL_dhT"], prop)
    for name, g, r in zip(("w", "dW", "dU", "db_i", "db_h"), run.serial_backward(h), rb):
        assert gh.rel_err(g, r) <= TOL, name


def _check_mgrit(gh, d, cf, levels, iters, fcf=True):
    _, _, rits = orc.mgrit_forward(*_P(d), d["x"], d["h0"], _zeros(d), cf, levels, iters,
                                   fine_relax_fcf=fcf, keep_iterates=True)
    run = gh.GpuRun(d, cf=cf, levels=levels, fine_relax=int(fcf), dtype=FORM)
    gits, _ = run.forward_iterates(iters)
    for i, (g, r) in enumerate(zip(gits, rits)):
        assert gh.rel_err(g, r) <= TOL, ("h", i)
    h = rits[-1].astype(np.float32)
    out = orc.mgrit_backward(*_P(d), d["x"], h, d["dL_dhT"], _zeros(d), cf, levels, iters,
                             fine_relax_fcf=fcf, keep_iterates=True)
    wits, gres, grads = run.backward_iterates(h, iters)
    for i, (g, r) in enumerate(zip(wits, out[-1])):
        assert gh.rel_err(g, r) <= TOL, ("w", i)
    for name, g, r in zip(("dW", "dU", "db_i", "db_h"), grads, out[2:6]):
        assert gh.rel_err(g, r) <= TOL, name
    for g, r in zip(gres, out[1]):
        assert abs(g - r) <= 1e-4 * max(r, 1e-30) + 2e-6 * np.sqrt(d["x"].shape[0])


@pytest.mark.parametrize("cf,levels,fcf", [(4, 3, True), (4, 2, False), (2, 4, True)])
def test_mgrit_hierarchies_every_iterate(gh, cf, levels, fcf):
    """96 intervals x 40 rows on level 0 down to 40 rows on the coarsest level: the three
    tile configurations and the few-row kernels in one solve."""
    T = 24 * cf ** (levels - 1) if cf == 4 else 192
    d = random_small(91, T, 40, 72, 104, scale=0.2)
    _check_mgrit(gh, d, cf, levels, 2, fcf)


@pytest.mark.parametrize("name", ["C2", "C3", "C5"])
def test_mgrit_reduced_twins(gh, name):
    wl = WORKLOADS[name].twin()
    _check_mgrit(gh, make_inputs(wl), wl.cf, wl.levels, 2)


def test_terms_of_small_and_large_magnitudes(gh):
    """The three-term split keeps the exponent range of fp32: a tiny loss gradient (1e-20)
    and large inputs change nothing about the relative error."""
    T, B, D, H = 32, 70, 16, 40
    d = dict(random_small(17, T, B, D, H, scale=0.3))
    d["dL_dhT"] = (d["dL_dhT"] * 1e-20).astype(np.float32)
    d["x"] = (d["x"] * 50.0).astype(np.float32)
    _check_mgrit(gh, d, 4, 2, 2)
