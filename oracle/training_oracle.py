"""CPU oracle of the training loop (Alg. 3 of the paper) for a stack of GRU layers.

TEST INFRASTRUCTURE ONLY (see mgrit_gru_oracle.py): float64 numpy, written from the paper; only
tests, the smoke check and the bench's CPU leg may import it.

Per batch: forward propagation of every layer by `fwd_iters` MGRIT cycles from a zero guess
(Alg. 3 forward block) or by the serial scan, the mean cross-entropy of a linear head on the top
layer's last state, back-propagation by `bwd_iters` MGRIT cycles on the adjoint from a zero guess
(Alg. 3 backward block) or by serial BPTT, the gradient line, and one Adam update (Sec. 4: the
networks are trained with Adam; Kingma & Ba's algorithm with its default constants).
"""
from __future__ import annotations

import numpy as np

from . import mgrit_gru_oracle as orc


class Adam:
    """Kingma & Ba, Algorithm 1: m <- b1 m + (1-b1) g; v <- b2 v + (1-b2) g^2;
    theta <- theta - lr * (m / (1-b1^t)) / (sqrt(v / (1-b2^t)) + eps)."""

    def __init__(self, tensors, lr=1e-3, b1=0.9, b2=0.999, eps=1e-8):
        self.p = tensors
        self.lr, self.b1, self.b2, self.eps = lr, b1, b2, eps
        self.m = [np.zeros_like(p) for p in tensors]
        self.v = [np.zeros_like(p) for p in tensors]
        self.t = 0

    def step(self, grads):
        self.t += 1
        for p, g, m, v in zip(self.p, grads, self.m, self.v):
            m *= self.b1
            m += (1.0 - self.b1) * g
            v *= self.b2
            v += (1.0 - self.b2) * g * g
            m_hat = m / (1.0 - self.b1 ** self.t)
            v_hat = v / (1.0 - self.b2 ** self.t)
            p -= self.lr * m_hat / (np.sqrt(v_hat) + self.eps)


def head_loss_and_gradients(h_T, W_o, b_o, labels):
    """Mean cross-entropy of softmax(h_T W_o^T + b_o); returns (loss, dL/dh_T, dL/dW_o, dL/db_o)."""
    loss, g_h = orc.cross_entropy_head(h_T, W_o, b_o, labels)
    logits = h_T @ W_o.T + b_o
    logits = logits - logits.max(axis=1, keepdims=True)
    p = np.exp(logits)
    p /= p.sum(axis=1, keepdims=True)
    p[np.arange(h_T.shape[0]), labels] -= 1.0
    p /= h_T.shape[0]
    return loss, g_h, p.T @ h_T, p.sum(axis=0)


class StackOracle:
    """params: per layer [W, U, b_i, b_h]; head: [W_o, b_o] (copied to float64 and updated here)."""

    def __init__(self, T, B, params, head, *, cf, levels, fwd_iters=2, bwd_iters=1,
                 fine_relax_fcf=True, lr=1e-3, parallel=True):
        self.T, self.B = T, B
        self.cf, self.levels, self.fcf = cf, levels, fine_relax_fcf
        self.fwd_iters, self.bwd_iters, self.parallel = fwd_iters, bwd_iters, parallel
        self.params = [[np.array(q, dtype=np.float64) for q in p] for p in params]
        self.head = [np.array(q, dtype=np.float64) for q in head]
        self.H = self.params[0][1].shape[1]
        self.opt = Adam([q for p in self.params for q in p] + self.head, lr=lr)

    def forward(self, x, parallel=None):
        parallel = self.parallel if parallel is None else parallel
        z = np.zeros((self.T + 1, self.B, self.H))
        h0s = [np.zeros((self.B, self.H))] * len(self.params)
        if parallel:
            solve = lambda j, W, U, bi, bh, xin, h0: orc.mgrit_forward(
                W, U, bi, bh, xin, h0, z, self.cf, self.levels, self.fwd_iters,
                fine_relax_fcf=self.fcf)[0]
        else:
            solve = lambda j, W, U, bi, bh, xin, h0: orc.serial_scan(W, U, bi, bh, xin, h0)
        return orc.stacked_forward(self.params, x, h0s, solve)

    def step(self, x, labels):
        hs = self.forward(x)
        loss, g_h, g_Wo, g_bo = head_loss_and_gradients(hs[-1][-1], *self.head, labels)
        src = np.zeros((self.T + 1, self.B, self.H))
        src[-1] = g_h
        z = np.zeros_like(src)
        if self.parallel:
            def adj(j, W, U, bi, bh, xin, h, s):
                out = orc.mgrit_backward(W, U, bi, bh, xin, h, None, z, self.cf, self.levels,
                                         self.bwd_iters, fine_relax_fcf=self.fcf, dL_dh=s)
                return (out[0],) + tuple(out[2:7])
        else:
            adj = lambda j, W, U, bi, bh, xin, h, s: orc.serial_bptt_steps(W, U, bi, bh, xin, h, s)
        res = orc.stacked_backward(self.params, x, hs, src, adj)
        grads = [g for r in res for g in r[1:5]] + [g_Wo, g_bo]
        self.opt.step(grads)
        return loss

    def logits(self, x, parallel=None):
        hs = self.forward(x, parallel)
        return hs[-1][-1] @ self.head[0].T + self.head[1]
