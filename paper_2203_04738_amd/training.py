"""Training loop of the paper's Alg. 3 for a stack of GRU layers: per batch, forward
propagation of every layer (MGRIT with a fixed number of cycles, or the serial scan), the loss,
back-propagation of every layer in reverse order (MGRIT on the adjoint, or serial BPTT), and
one optimiser step.

This module only sequences calls of the C-ABI library (through the binding) and torch
operations that are outside the hot path: the linear head with its cross-entropy loss and the
Adam update (the paper trains with Adam, Sec. 4).  Every GRU step, forward and adjoint, runs
in the library's kernels; there is no fallback.

Layers are stacked the usual way (layer j+1 reads the state sequence of layer j); the loss
reads the last state of the top layer.  Remark 3 of the paper (a network trained with MGRIT can
be evaluated with serial propagation) is what `predict(x, parallel=False)` is for.
"""
from __future__ import annotations

from typing import List, Sequence

from . import binding as _b


class GruStackTrainer:
    """params: per layer [W[3H,D_j], U[3H,H], b_i[3H], b_h[3H]] float32 CUDA tensors (updated in
    place); head: [W_o[C,H], b_o[C]].  parallel=True trains with MGRIT (`fwd_iters` forward and
    `bwd_iters` backward cycles per layer), False with the serial scan and serial BPTT."""

    def __init__(self, T: int, B: int, params: Sequence[Sequence], head: Sequence, *, cf: int,
                 levels: int, fwd_iters: int = 2, bwd_iters: int = 1, fine_relax: int = 1,
                 lr: float = 1e-3, parallel: bool = True):
        import torch
        self.T, self.B, self.parallel = T, B, parallel
        self.cf, self.levels, self.fine_relax = cf, levels, fine_relax
        self.fwd_iters, self.bwd_iters = fwd_iters, bwd_iters
        self.params = [list(p) for p in params]
        self.head = list(head)
        self.H = self.params[0][1].shape[1]
        self.dims = [p[0].shape[1] for p in self.params]
        dev = self.params[0][0].device
        L, H = len(self.params), self.H
        self.ws = [torch.empty(_b.mgrit_gru_workspace_bytes(self._cfg(j, max(fwd_iters, bwd_iters, 1))),
                               dtype=torch.uint8, device=dev) for j in range(L)]
        z = lambda: torch.zeros(T + 1, B, H, device=dev)
        self.h = [z() for _ in range(L)]          # states of every layer
        self.w = [z() for _ in range(L)]          # adjoints
        self.src = [z() for _ in range(L)]        # dL/dh of every layer (loss term / dL/dx from above)
        self.h0 = torch.zeros(B, H, device=dev)
        self.grads = [[torch.zeros_like(q) for q in p] for p in self.params]
        flat = [q for p in self.params for q in p] + self.head
        self.opt = torch.optim.Adam(flat, lr=lr)

    def _cfg(self, j: int, iters: int, flags: int = 0):
        return _b.MgritGruCfg(self.T, self.B, self.dims[j], self.H, cf=self.cf, levels=self.levels,
                              iters=iters, fine_relax=self.fine_relax, propagator=0, dtype=0,
                              flags=flags)

    # ---- Alg. 3, forward block
    def forward(self, x, parallel: bool | None = None):
        """States of every layer for the batch x[T,B,D]; returns the top layer's h_T (a view)."""
        parallel = self.parallel if parallel is None else parallel
        for j, p in enumerate(self.params):
            xin = x if j == 0 else self.h[j - 1][1:]
            if parallel:
                self.h[j].zero_()                 # the zero initial guess of Alg. 3
                _b.mgrit_gru_forward(self._cfg(j, self.fwd_iters, _b.MGRIT_ZERO_STATE_GUESS), *p, xin,
                                     self.h0, self.h[j], None, self.ws[j])
            else:
                _b.gru_serial_scan(self._cfg(j, 1), *p, xin, self.h0, self.h[j], self.ws[j])
        return self.h[-1][self.T]

    # ---- Alg. 3, backward block and gradient line
    def backward(self, x, dL_dhT, parallel: bool | None = None) -> None:
        """Fills self.grads from the loss derivative with respect to the top layer's h_T.  Uses
        the states (and the projections in the workspaces) the last forward() left."""
        parallel = self.parallel if parallel is None else parallel
        L, T = len(self.params), self.T
        self.src[-1].zero_()
        self.src[-1][T] = dL_dhT
        for j in range(L - 1, -1, -1):
            xin = x if j == 0 else self.h[j - 1][1:]
            dx = None
            if j > 0:                             # dL/dx of layer j is the loss term of layer j-1
                self.src[j - 1][0].zero_()
                dx = self.src[j - 1][1:]
            if parallel:
                self.w[j].zero_()
                _b.mgrit_gru_backward_steps(self._cfg(j, self.bwd_iters, _b.MGRIT_REUSE_PROJECTION),
                                            *self.params[j], xin, self.h[j], self.src[j], self.w[j],
                                            None, *self.grads[j], dx, self.ws[j])
            else:
                _b.gru_serial_scan_backward_steps(self._cfg(j, 1, _b.MGRIT_REUSE_PROJECTION),
                                                  *self.params[j], xin, self.h[j], self.src[j],
                                                  self.w[j], *self.grads[j], dx, self.ws[j])

    def step(self, x, labels) -> float:
        """One iteration of Alg. 3 on the batch (x, labels); returns the loss before the update."""
        import torch
        hT = self.forward(x).clone().requires_grad_(True)
        Wo, bo = self.head
        Wo.requires_grad_(True)
        bo.requires_grad_(True)
        loss = torch.nn.functional.cross_entropy(hT @ Wo.T + bo, labels)
        gh, gW, gb = torch.autograd.grad(loss, (hT, Wo, bo))
        Wo.requires_grad_(False)
        bo.requires_grad_(False)
        self.backward(x, gh)
        for p, g in zip(self.params, self.grads):
            for q, gq in zip(p, g):
                q.grad = gq
        Wo.grad, bo.grad = gW, gb
        self.opt.step()
        return float(loss.detach())

    def logits(self, x, parallel: bool | None = None):
        hT = self.forward(x, parallel)
        return hT @ self.head[0].T + self.head[1]

    def predict(self, x, parallel: bool | None = None):
        import torch
        return torch.argmax(self.logits(x, parallel), dim=1)
