"""Pins of the training-loop oracle (no GPU): its Adam against the library optimiser, its head
gradients against autograd, and one whole serial training step against a library GRU trained by
autograd + the library Adam."""
import numpy as np
import torch

from oracle import mgrit_gru_oracle as orc
from oracle import training_oracle as tro
from synthetic_inputs import ClassificationTask, init_stack


def test_adam_is_the_library_adam():
    rng = np.random.default_rng(0)
    ps = [rng.standard_normal((4, 3)), rng.standard_normal(5)]
    tp = [torch.tensor(p.copy(), dtype=torch.float64) for p in ps]
    opt_t = torch.optim.Adam(tp, lr=1e-3)
    opt_o = tro.Adam(ps, lr=1e-3)
    for k in range(7):
        gs = [rng.standard_normal(p.shape) * 10.0 ** rng.integers(-6, 1) for p in ps]
        for t, g in zip(tp, gs):
            t.grad = torch.from_numpy(g.copy())
        opt_t.step()
        opt_o.step(gs)
        for p, t in zip(ps, tp):
            assert np.allclose(p, t.numpy(), rtol=1e-12, atol=1e-15), k


def test_head_gradients_match_autograd():
    rng = np.random.default_rng(1)
    hT, Wo, bo = rng.standard_normal((5, 7)), rng.standard_normal((4, 7)), rng.standard_normal(4)
    lab = rng.integers(0, 4, size=5)
    loss, g_h, g_W, g_b = tro.head_loss_and_gradients(hT, Wo, bo, lab)
    t = [torch.from_numpy(a).requires_grad_(True) for a in (hT, Wo, bo)]
    lt = torch.nn.functional.cross_entropy(t[0] @ t[1].T + t[2], torch.from_numpy(lab))
    lt.backward()
    assert abs(loss - lt.item()) < 1e-12
    for a, b in zip((g_h, g_W, g_b), t):
        assert np.allclose(a, b.grad.numpy(), atol=1e-13)


def test_serial_training_steps_equal_a_library_gru_trained_by_autograd_and_adam():
    """Alg. 3 with serial propagation and the Implicit step, two layers: the whole loop (stack,
    head, BPTT through both layers, Adam) against the same network written as tensor operations
    and trained by autograd + torch.optim.Adam in float64."""
    task = ClassificationTask(T=12, B=6, D=4, channels=3, classes=3, seed=3)
    H, L = 5, 2
    params, head = init_stack(11, task.D, H, task.classes, L)
    for p in params:                      # non-zero biases so that every term is exercised
        p[2] += 0.1
        p[3] -= 0.2
    o = tro.StackOracle(task.T, task.B, params, head, cf=2, levels=2, parallel=False, lr=1e-2)
    tp = [[torch.tensor(q, dtype=torch.float64, requires_grad=True) for q in p] for p in params]
    th = [torch.tensor(q, dtype=torch.float64, requires_grad=True) for q in head]
    opt = torch.optim.Adam([q for p in tp for q in p] + th, lr=1e-2)

    def net(x):
        inp = x
        for W, U, b_i, b_h in tp:
            h = torch.zeros(task.B, H, dtype=torch.float64)
            out = []
            for t in range(task.T):
                gi, gh = inp[t] @ W.T + b_i, h @ U.T + b_h
                r = torch.sigmoid(gi[:, :H] + gh[:, :H])
                z = torch.sigmoid(gi[:, H:2 * H] + gh[:, H:2 * H])
                n = torch.tanh(gi[:, 2 * H:] + r * gh[:, 2 * H:])
                h = (h + (1 - z) * n) / (1 + (1 - z))            # Eq. 16 with step size 1
                out.append(h)
            inp = torch.stack(out)
        return inp[-1] @ th[0].T + th[1]

    for k in range(4):
        x, y = task.batch(k)
        lo = o.step(x.astype(np.float64), y)
        opt.zero_grad()
        lt = torch.nn.functional.cross_entropy(net(torch.from_numpy(x).double()), torch.from_numpy(y))
        lt.backward()
        opt.step()
        assert abs(lo - lt.item()) < 1e-10, k
        for po, pt in zip([q for p in o.params for q in p] + o.head, [q for p in tp for q in p] + th):
            assert np.allclose(po, pt.detach().numpy(), rtol=0, atol=1e-9), k


def test_mgrit_training_step_with_enough_cycles_equals_the_serial_step():
    """With enough cycles MGRIT reproduces serial propagation and BPTT exactly (finite
    termination), so one training step of the MGRIT loop then equals the serial loop's."""
    task = ClassificationTask(T=16, B=4, D=4, channels=3, classes=3, seed=5)
    H = 4
    params, head = init_stack(13, task.D, H, task.classes, 2)
    kw = dict(cf=2, levels=3, lr=1e-2)
    a = tro.StackOracle(task.T, task.B, params, head, parallel=False, **kw)
    b = tro.StackOracle(task.T, task.B, params, head, parallel=True, fwd_iters=8, bwd_iters=8, **kw)
    x, y = task.batch(0)
    la, lb = a.step(x, y), b.step(x, y)
    assert abs(la - lb) < 1e-12
    for p, q in zip([t for l in a.params for t in l] + a.head, [t for l in b.params for t in l] + b.head):
        assert np.allclose(p, q, rtol=0, atol=1e-9)
