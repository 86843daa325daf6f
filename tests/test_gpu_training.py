"""The training loop of Alg. 3 on the HIP path (paper_2203_04738_amd.training: library calls +
torch Adam) against the oracle's loop (numpy float64), on the same seeded task."""
import numpy as np
import pytest
import torch

from oracle import training_oracle as tro
from synthetic_inputs import ClassificationTask, init_stack

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

# Parameters after k Adam steps.  Adam divides the gradient's running mean by the root of its
# running second moment, so an element's update is lr * (a ratio of order one) and a relative
# gradient error e changes it by about lr * e.  The HIP path's gradients are within 1e-5 of the
# oracle's relative to the LARGEST element of a tensor; for an element 100 times smaller than
# the largest that is 1e-3 relative, i.e. 1e-3 * lr = 1e-6 absolute per step at lr = 1e-3, against
# parameters of magnitude 0.1-0.5.  The bar below (relative to the tensor's largest element)
# leaves room for such elements over the steps taken and for the drift of the trajectories
# (later gradients are evaluated at slightly different parameters).
PARAM_TOL = 1e-4
LOGIT_TOL = 1e-4


def _rel(a, b):
    return float(np.max(np.abs(a - b)) / max(np.max(np.abs(b)), 1e-300))


@pytest.mark.parametrize("parallel", [True, False])
def test_five_training_steps_follow_the_oracle_loop(parallel):
    from paper_2203_04738_amd.training import GruStackTrainer
    task = ClassificationTask(T=64, B=16, D=12, channels=9, classes=6, seed=0)
    H, L = 40, 2
    params, head = init_stack(7, task.D, H, task.classes, L)
    kw = dict(cf=4, levels=3, fwd_iters=2, bwd_iters=1, lr=1e-3, parallel=parallel)
    o = tro.StackOracle(task.T, task.B, params, head, **kw)
    dp = [[torch.from_numpy(q.copy()).to(DEV) for q in p] for p in params]
    dh = [torch.from_numpy(q.copy()).to(DEV) for q in head]
    g = GruStackTrainer(task.T, task.B, dp, dh, **kw)
    for k in range(5):
        x, y = task.batch(k)
        lo = o.step(x, y)
        lg = g.step(torch.from_numpy(x).to(DEV), torch.from_numpy(y).to(DEV))
        assert abs(lg - lo) <= 1e-5 * max(1.0, abs(lo)), (k, lg, lo)
        errs = [_rel(q.cpu().numpy().astype(np.float64), r)
                for q, r in zip([t for p in g.params for t in p] + g.head,
                                [t for p in o.params for t in p] + o.head)]
        print(f"step {k}: loss {lg:.6f} (oracle {lo:.6f}), max parameter error {max(errs):.2e}",
              flush=True)
        assert max(errs) <= PARAM_TOL, (k, errs)
    # Remark 3: the trained network evaluated with serial and with MGRIT propagation
    x, y = task.batch(100)
    xd = torch.from_numpy(x).to(DEV)
    for inference_parallel in (False, True):
        got = g.logits(xd, inference_parallel).cpu().numpy().astype(np.float64)
        ref = o.logits(x, inference_parallel)
        assert _rel(got, ref) <= LOGIT_TOL, inference_parallel
    ser = g.logits(xd, False).cpu().numpy()
    par = g.logits(xd, True).cpu().numpy()
    # two cycles do not converge the states: the two inference modes differ, by the same amount
    # on both sides
    assert abs(_rel(par, ser) - _rel(o.logits(x, True), o.logits(x, False))) <= 1e-3
