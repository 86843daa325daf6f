"""The entry point that allocates nothing (fixed workspace inside the library) against
mgrit_gru_forward with a caller workspace: same kernels, so the same bits."""
import numpy as np
import pytest
import torch

import paper_2203_04738_amd as mg
from paper_2203_04738_amd.binding import MGRIT_ZERO_STATE_GUESS, MgritGruCfg
from synthetic_inputs import random_small

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _both(seed, T, B, D, H, cf, levels, iters, flags):
    d = random_small(seed, T, B, D, H, scale=0.3)
    t = {k: torch.from_numpy(v).to(DEV) for k, v in d.items()}
    cfg = MgritGruCfg(T, B, D, H, cf=cf, levels=levels, iters=iters, flags=flags)
    P = (t["W"], t["U"], t["b_i"], t["b_h"], t["x"])
    ws = torch.empty(mg.mgrit_gru_workspace_bytes(cfg), dtype=torch.uint8, device=DEV)
    h_a = torch.zeros(T + 1, B, H, device=DEV)
    r_a = torch.full((iters,), float("nan"), device=DEV)
    mg.mgrit_gru_forward(cfg, *P, t["h0"], h_a, r_a, ws)
    h_b = torch.zeros(T + 1, B, H, device=DEV)
    r_b = torch.full((iters,), float("nan"), device=DEV)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    mg.mgrit_gru_forward_static(cfg, *P, t["h0"], h_b, r_b)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    return h_a.cpu().numpy(), r_a.cpu().numpy(), h_b.cpu().numpy(), r_b.cpu().numpy()


def test_static_workspace_forward_equals_the_workspace_forward_twice_in_a_row():
    # first call: several row and column tiles with ragged tails (1025 rows on level 0,
    # H = 72), three levels; second call: a smaller problem on the same, now used, array
    for seed, shape, flags in ((5, (1024, 5, 40, 72, 4, 3, 2), MGRIT_ZERO_STATE_GUESS),
                               (6, (64, 2, 16, 32, 4, 2, 3), 0)):
        print("static workspace case", shape, flush=True)
        h_a, r_a, h_b, r_b = _both(seed, *shape, flags)
        assert np.all(np.isfinite(h_a)) and np.any(h_a[-1] != 0)
        assert np.array_equal(h_a, h_b)                  # same kernels, same launch sequence
        assert np.allclose(r_a, r_b, rtol=1e-6, atol=0)  # sums of squares by atomics: ~1e-15


def test_static_workspace_rejects_what_does_not_fit():
    T, B, D, H = 2048, 32, 1024, 512
    cfg = MgritGruCfg(T, B, D, H, cf=4, levels=3, iters=1)
    z = lambda *s: torch.zeros(*s, device=DEV)
    h = z(T + 1, B, H)
    with pytest.raises(mg.MgritGruError) as e:
        mg.mgrit_gru_forward_static(cfg, z(3 * H, D), z(3 * H, H), z(3 * H), z(3 * H), z(T, B, D),
                                    z(B, H), h, None)
    assert e.value.code == -5
    assert not torch.any(h)
