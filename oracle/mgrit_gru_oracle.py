"""CPU oracle for the MGRIT solve over a GRU hidden-state sequence.

TEST INFRASTRUCTURE ONLY.  This file is the plain, slow, float64 statement of
what the method computes, written from the paper (Moon & Cyr, "Parallel
Training of GRU Networks with a Multi-Grid Solver for Long Sequences").  Only
the tests, the smoke check and the bench's ``cpu_baseline`` leg may import it;
the product path (the HIP library) shares no code with it and never calls it.

Conventions
-----------
* ``x[T,B,D]``: row ``t-1`` holds x_t (t = 1..T).  State arrays ``h[(T+1),B,H]``:
  row t holds h_t, row 0 is the initial condition h_0 (Sec. 3.1 notation; the
  paper assumes h_0 = 0, here it is an argument).
* Parameters are the Classic-GRU ones (Eq. 1), gates stacked r, z, n:
  ``W[3H,D]`` (W_ir;W_iz;W_in), ``U[3H,H]`` (W_hr;W_hz;W_hn), ``b_i[3H]``, ``b_h[3H]``.
* Level l of the hierarchy has N_l = T/cf^l steps, points 0..N_l, and step size
  gamma = cf^l (Sec. 3.3: the coarse time step equals cf^l).  Level-l point k is
  fine point k*cf^l and uses the input x_{k*cf^l} (restriction of x is injection,
  Sec. 3.1).
* All arithmetic is float64 on whatever values the caller passes (for the bf16
  workload the caller passes bf16-representable inputs).

Every function cites the passage it follows.  Pins that tie this file to the
paper and to mathematics (closed forms, a library GRU, finite differences,
exactness fronts, the per-level decay factors of a zero-weight problem, and the
cycle of Alg. 2 carried out by dense linear algebra on affine forward problems
and on the linear adjoint problem with autograd Jacobians) are in
tests/test_oracle_pins.py.  Per-iterate values of the NONLINEAR forward cycle
(U != 0) at 2-3 iterations have no published reference: they are pinned through
the same cycle code on the affine and adjoint problems and by the structural
pins, not value by value.
"""
from __future__ import annotations

import numpy as np

IMPLICIT = 0   # Eq. 16 (Implicit GRU), the paper's propagator on every level
CLASSIC = 1    # Eq. 3 (explicit Euler; gamma = 1 is the Classic GRU of Eq. 1)


def _f64(a):
    return np.asarray(a, dtype=np.float64)


def sigmoid(a):
    return 1.0 / (1.0 + np.exp(-a))


def _rows_times(a, M):
    """a[..., K] @ M[K, N] with all leading axes of `a` taken together as the rows of ONE matrix
    product (numpy would otherwise run one small product per leading index)."""
    a = np.asarray(a)
    return (a.reshape(-1, a.shape[-1]) @ M).reshape(a.shape[:-1] + (M.shape[1],))


# --------------------------------------------------------------------------
# Cell: Eq. 1 gates, Eq. 3 / Eq. 16 propagators
# --------------------------------------------------------------------------

def input_projection(W, b_i, x):
    """P[t-1] = W x_t + b_i for every t (the input half of Eq. 1's three
    pre-activations).  Computed once and reused on every level and in the
    adjoint, as the paper reuses its precomputed per-step features
    (Appendix A.3.2)."""
    return _rows_times(_f64(x), _f64(W).T) + _f64(b_i)


def gates(P, h, U, b_h):
    """Eq. 1: r, z, and the candidate n, all evaluated at x_t (through P) and
    the OLD state h = h_{t-1} (Sec. 3.3, text after Eq. 15).  Also returns
    q = W_hn h + b_hn, needed by the adjoint."""
    H = h.shape[-1]
    a = _rows_times(h, U.T) + b_h
    r = sigmoid(P[..., :H] + a[..., :H])
    z = sigmoid(P[..., H:2 * H] + a[..., H:2 * H])
    q = a[..., 2 * H:]
    n = np.tanh(P[..., 2 * H:] + r * q)
    return r, z, q, n


def phi(gamma, P, h, U, b_h, propagator=IMPLICIT):
    """One step h_t = Phi_gamma(x_t, h_{t-1}).
    Implicit (Eq. 16): (1 + gamma(1-z))^{-1} (h + gamma (1-z) n).
    Classic  (Eq. 3):  h + gamma(-(1-z) h + (1-z) n)."""
    r, z, q, n = gates(P, h, U, b_h)
    c = 1.0 - z
    if propagator == IMPLICIT:
        return (h + gamma * c * n) / (1.0 + gamma * c)
    if propagator == CLASSIC:
        return h + gamma * (-c * h + c * n)
    raise ValueError("unknown propagator")


def phi_adjoint_coeffs(gamma, P, h, U, b_h, propagator=IMPLICIT):
    """Coefficient vectors of the transpose Jacobian of one step with respect
    to its input state (discrete adjoint of Eq. 16 / Eq. 3, Appendix A.2), at
    the linearisation point (x_t, h = h_{t-1}).  With h' = Phi_gamma(x_t, h):

        Implicit: d = 1 + gamma(1-z); dh'/dh|direct = 1/d; dh'/dn = gamma(1-z)/d;
                  dh'/dz = -gamma (n - h')/d
        Classic:  dh'/dh|direct = 1 - gamma(1-z); dh'/dn = gamma(1-z);
                  dh'/dz = -gamma (n - h)

    Chain rule through n = tanh(.), r = sigma(.), z = sigma(.) gives
        k_n = dh'/dn (1-n^2),  k_q = k_n r,  k_r = k_n q r(1-r),  k_z = dh'/dz z(1-z).
    Returns (k_d, k_r, k_z, k_q, k_n)."""
    r, z, q, n = gates(P, h, U, b_h)
    c = 1.0 - z
    if propagator == IMPLICIT:
        d = 1.0 + gamma * c
        h_new = (h + gamma * c * n) / d
        k_d = 1.0 / d
        dn = gamma * c / d
        dz = -gamma * (n - h_new) / d
    elif propagator == CLASSIC:
        k_d = 1.0 - gamma * c
        dn = gamma * c
        dz = -gamma * (n - h)
    else:
        raise ValueError("unknown propagator")
    k_n = dn * (1.0 - n * n)
    k_q = k_n * r
    k_r = k_n * q * r * (1.0 - r)
    k_z = dz * z * (1.0 - z)
    return k_d, k_r, k_z, k_q, k_n


def phi_transpose(coeffs, w, U):
    """(dPhi/dh)^T w = k_d*w + U_r^T(k_r*w) + U_z^T(k_z*w) + U_n^T(k_q*w)."""
    k_d, k_r, k_z, k_q, _ = coeffs
    H = w.shape[-1]
    return (k_d * w + _rows_times(k_r * w, U[:H]) + _rows_times(k_z * w, U[H:2 * H])
            + _rows_times(k_q * w, U[2 * H:]))


# --------------------------------------------------------------------------
# Serial forward propagation (Eq. 4 with f(h) = 0) and serial BPTT
# --------------------------------------------------------------------------

def serial_scan(W, U, b_i, b_h, x, h0, propagator=IMPLICIT, gamma=1.0):
    """h_t = Phi_1(x_t, h_{t-1}), t = 1..T: the solution of f(h) = 0 (Eq. 4)."""
    W, U, b_i, b_h, x, h0 = map(_f64, (W, U, b_i, b_h, x, h0))
    P = input_projection(W, b_i, x)
    T = x.shape[0]
    h = np.empty((T + 1,) + h0.shape)
    h[0] = h0
    for t in range(1, T + 1):
        h[t] = phi(gamma, P[t - 1], h[t - 1], U, b_h, propagator)
    return h


def fine_residual(W, U, b_i, b_h, x, h, propagator=IMPLICIT):
    """Eq. 4: f(h)_t = h_t - Phi_1(x_t, h_{t-1}) for all t = 1..T."""
    W, U, b_i, b_h, x, h = map(_f64, (W, U, b_i, b_h, x, h))
    P = input_projection(W, b_i, x)
    return h[1:] - phi(1.0, P, h[:-1], U, b_h, propagator)


def parameter_gradients(W, U, b_i, b_h, x, h, w, propagator=IMPLICIT):
    """Alg. 3, gradient line: g = sum_t w_t * dh_t/dTheta, with the fine-level
    step (gamma = 1) linearised at the given states h.  Returns dW, dU, db_i, db_h."""
    W, U, b_i, b_h, x, h, w = map(_f64, (W, U, b_i, b_h, x, h, w))
    P = input_projection(W, b_i, x)
    dW = np.zeros_like(W)
    dU = np.zeros_like(U)
    db_i = np.zeros_like(b_i)
    db_h = np.zeros_like(b_h)
    T = x.shape[0]
    for t in range(1, T + 1):
        k_d, k_r, k_z, k_q, k_n = phi_adjoint_coeffs(1.0, P[t - 1], h[t - 1], U, b_h, propagator)
        s_h = np.concatenate([k_r * w[t], k_z * w[t], k_q * w[t]], axis=-1)   # [B,3H]
        s_x = np.concatenate([k_r * w[t], k_z * w[t], k_n * w[t]], axis=-1)
        dU += s_h.T @ h[t - 1]
        db_h += s_h.sum(axis=0)
        dW += s_x.T @ x[t - 1]
        db_i += s_x.sum(axis=0)
    return dW, dU, db_i, db_h


def serial_bptt(W, U, b_i, b_h, x, h, dL_dhT, propagator=IMPLICIT):
    """Back-propagation through time for a loss on h_T only: w_T = dL/dh_T,
    w_{t-1} = (dPhi_1/dh)^T(x_t, h_{t-1}) w_t.  Returns (w[(T+1),B,H], dW, dU,
    db_i, db_h); w[0] is dL/dh_0."""
    W, U, b_i, b_h, x, h, dL_dhT = map(_f64, (W, U, b_i, b_h, x, h, dL_dhT))
    P = input_projection(W, b_i, x)
    T = x.shape[0]
    w = np.empty_like(h)
    w[T] = dL_dhT
    for t in range(T, 0, -1):
        co = phi_adjoint_coeffs(1.0, P[t - 1], h[t - 1], U, b_h, propagator)
        w[t - 1] = phi_transpose(co, w[t], U)
    return (w,) + parameter_gradients(W, U, b_i, b_h, x, h, w, propagator)


def input_gradients(W, U, b_i, b_h, x, h, w, propagator=IMPLICIT):
    """dL/dx_t = (dPhi_1/dx)^T(x_t, h_{t-1}) w_t for t = 1..T (row t-1 of the
    result), the input-side counterpart of Alg. 3's gradient line: x_t enters the
    step only through W x_t inside the three gates (Eq. 1), so
    dL/dx_t = W_r^T(k_r w_t) + W_z^T(k_z w_t) + W_n^T(k_n w_t)."""
    W, U, b_i, b_h, x, h, w = map(_f64, (W, U, b_i, b_h, x, h, w))
    P = input_projection(W, b_i, x)
    T = x.shape[0]
    dx = np.empty_like(x)
    for t in range(1, T + 1):
        k_d, k_r, k_z, k_q, k_n = phi_adjoint_coeffs(1.0, P[t - 1], h[t - 1], U, b_h, propagator)
        s_x = np.concatenate([k_r * w[t], k_z * w[t], k_n * w[t]], axis=-1)   # [B,3H]
        dx[t - 1] = s_x @ W
    return dx


def serial_bptt_steps(W, U, b_i, b_h, x, h, dL_dh, propagator=IMPLICIT):
    """Back-propagation through time for a loss that depends on every state:
    dL_dh[(T+1),B,H] holds the direct derivative of the loss with respect to h_t
    in row t.  w_T = dL_dh[T];  w_{t-1} = (dPhi_1/dh)^T(x_t, h_{t-1}) w_t + dL_dh[t-1]
    (the adjoint recurrence of Appendix A.2 with a source term).  Returns
    (w, dW, dU, db_i, db_h, dx)."""
    W, U, b_i, b_h, x, h, dL_dh = map(_f64, (W, U, b_i, b_h, x, h, dL_dh))
    P = input_projection(W, b_i, x)
    T = x.shape[0]
    w = np.empty_like(h)
    w[T] = dL_dh[T]
    for t in range(T, 0, -1):
        co = phi_adjoint_coeffs(1.0, P[t - 1], h[t - 1], U, b_h, propagator)
        w[t - 1] = phi_transpose(co, w[t], U) + dL_dh[t - 1]
    return ((w,) + parameter_gradients(W, U, b_i, b_h, x, h, w, propagator)
            + (input_gradients(W, U, b_i, b_h, x, h, w, propagator),))


# --------------------------------------------------------------------------
# MGRIT: relaxation (Alg. 1, Eq. 8), V-cycle (Alg. 2, Remark 2, Eq. 11)
# --------------------------------------------------------------------------
# The cycle below is written once over an abstract level step
#     step(l, ks, v) -> value at level-l points ks, given the values v at ks-1
# so that forward propagation (step = Phi) and the adjoint (step = transposed
# Jacobian in reversed time, Appendix A.1 last paragraph) run the same code.
# On coarse levels the problem carries a right-hand side g (full approximation
# scheme): level equation  u_k - step(l,k,u_{k-1}) = g_k,  g = 0 on level 0.

def relax(step, l, cf, u, g, include_c):
    """F-relaxation (Alg. 1) when include_c is False, FC-relaxation when True.
    All intervals are independent: interval i starts from the INPUT value at
    its coarse point i*cf (Alg. 1 copies h'_t = h_t first) and propagates over
    the following cf-1 fine points, and for FC also onto the next coarse point
    (Sec. 3.1, text before Eq. 8; Fig. 2).  Point 0 is never written."""
    n_int = (u.shape[0] - 1) // cf
    starts = cf * np.arange(n_int)
    out = u.copy()
    v = u[starts]
    for j in range(1, cf + (1 if include_c else 0)):
        v = step(l, starts + j, v) + g[starts + j]
        out[starts + j] = v
    return out


def v_cycle(step, cf, levels, l, u, g, fine_relax_fcf, resnorms):
    """One MGRIT cycle on level l (Alg. 2; recursive per Remark 2).
    u: current iterate on this level, [N_l+1, ...]; g: right-hand side, same
    shape (row 0 unused).  Returns the new iterate."""
    N = u.shape[0] - 1
    if l == levels - 1:
        # coarsest level: serial propagation solves the level equation exactly
        # (Appendix A.1)
        out = u.copy()
        for k in range(1, N + 1):
            out[k] = step(l, np.array([k]), out[k - 1:k])[0] + g[k]
        return out

    # Alg. 2 line 1: relax.  FCF (Eq. 8) everywhere; on the fine level
    # optionally F only (Sec. 3.2, first paragraph after Alg. 2).
    if l == 0 and not fine_relax_fcf:
        up = relax(step, l, cf, u, g, include_c=False)
    else:
        up = relax(step, l, cf, relax(step, l, cf, u, g, include_c=True), g, include_c=False)

    # line 2: residual of the level equation at the coarse points, restricted
    Nc = N // cf
    cpts = cf * np.arange(1, Nc + 1)
    r_c = up[cpts] - step(l, cpts, up[cpts - 1]) - g[cpts]
    if l == 0:
        resnorms.append(float(np.sqrt(np.sum(r_c * r_c))))

    # line 3: restrict the state (injection, Eq. 5; point 0 carried along)
    Uc = up[cf * np.arange(0, Nc + 1)]

    # line 4 / Eq. 11: coarse equation  A_c(v) = A_c(R u') - R r
    ks = np.arange(1, Nc + 1)
    g_c = np.zeros_like(Uc)
    g_c[ks] = (Uc[ks] - step(l + 1, ks, Uc[ks - 1])) - r_c
    V = v_cycle(step, cf, levels, l + 1, Uc.copy(), g_c, fine_relax_fcf, resnorms)

    # line 5: prolong the coarse correction (Eq. 6: replicate the prior coarse value)
    upp = up.copy()
    t = np.arange(1, N + 1)
    upp[t] = up[t] + (V - Uc)[t // cf]

    # line 6: F-relaxation from the corrected coarse points
    return relax(step, l, cf, upp, g, include_c=False)


def _check_hierarchy(T, cf, levels):
    if cf < 1 or levels < 1 or T < 1:
        raise ValueError("bad hierarchy")
    if T % (cf ** (levels - 1)) != 0:
        raise ValueError("cf^(levels-1) must divide T")


def mgrit_forward(W, U, b_i, b_h, x, h0, h_init, cf, levels, iters,
                  fine_relax_fcf=True, propagator=IMPLICIT, keep_iterates=False):
    """Alg. 3 forward block: `iters` applications of MGProp (Alg. 2) to the
    iterate h_init[(T+1),B,H] (row 0 is overwritten with h0).  Returns
    (h, resnorms) where resnorms[i] is the 2-norm of the level-0 coarse-point
    residual inside iteration i; with keep_iterates also the list of iterates."""
    W, U, b_i, b_h, x, h0 = map(_f64, (W, U, b_i, b_h, x, h0))
    T = x.shape[0]
    _check_hierarchy(T, cf, levels)
    P = input_projection(W, b_i, x)

    def step(l, ks, v):
        gamma = float(cf ** l)
        return phi(gamma, P[ks * cf ** l - 1], v, U, b_h, propagator)

    h = _f64(h_init).copy()
    h[0] = h0
    g0 = np.zeros_like(h)
    resnorms, iterates = [], []
    for _ in range(iters):
        h = v_cycle(step, cf, levels, 0, h, g0, fine_relax_fcf, resnorms)
        if keep_iterates:
            iterates.append(h.copy())
    if keep_iterates:
        return h, resnorms, iterates
    return h, resnorms


def mgrit_backward(W, U, b_i, b_h, x, h, dL_dhT, w_init, cf, levels, iters,
                   fine_relax_fcf=True, propagator=IMPLICIT, keep_iterates=False,
                   dL_dh=None, with_gradients=True):
    """Alg. 3 backward block: `iters` applications of MGBackProp to the adjoint
    iterate w_init[(T+1),B,H] (row T is overwritten with dL/dh_T), then the
    parameter gradients from the final w (Alg. 3 gradient line).

    MGBackProp is the same cycle run on the adjoint recurrence in reversed time
    (Appendix A.1, last paragraph; A.2, last paragraph).  In reversed index
    m = N_l - k the level-l step m-1 -> m is the transposed Jacobian of the
    forward level step k = N_l - m + 1, i.e. of Phi_{cf^l}(x_{k cf^l}, .)
    linearised at h_{(k-1) cf^l}, where h is the given forward iterate.
    Returns (w, resnorms, dW, dU, db_i, db_h).

    With dL_dh[(T+1),B,H] given (a loss on every state; dL_dhT is then ignored)
    the adjoint recurrence carries the source term dL_dh[t] at point t: it is
    the right-hand side of the level-0 equation, which the cycle restricts like
    any other (Eq. 11); the result gains a last element dx = input_gradients.

    with_gradients=False stops after the cycles and returns (w, resnorms[, iterates]): for
    callers that compare the adjoint iterate only (the gradient line is a loop over all T)."""
    if dL_dh is not None:
        dL_dh = _f64(dL_dh)
        dL_dhT = dL_dh[-1]
    W, U, b_i, b_h, x, h, dL_dhT = map(_f64, (W, U, b_i, b_h, x, h, dL_dhT))
    T = x.shape[0]
    _check_hierarchy(T, cf, levels)
    P = input_projection(W, b_i, x)

    def step(l, ms, v):
        s = cf ** l
        k = T // s - ms + 1                       # forward level index of the step
        co = phi_adjoint_coeffs(float(s), P[k * s - 1], h[(k - 1) * s], U, b_h, propagator)
        return phi_transpose(co, v, U)

    w = _f64(w_init).copy()
    w[T] = dL_dhT
    wr = w[::-1].copy()                           # reversed time: wr[m] = w[T-m]
    g0 = np.zeros_like(wr)
    if dL_dh is not None:
        g0[1:] = dL_dh[::-1][1:]                  # source at reversed point m is dL_dh[T-m]
    resnorms, iterates = [], []
    for _ in range(iters):
        wr = v_cycle(step, cf, levels, 0, wr, g0, fine_relax_fcf, resnorms)
        if keep_iterates:
            iterates.append(wr[::-1].copy())
    w = wr[::-1].copy()
    if not with_gradients:
        return (w, resnorms, iterates) if keep_iterates else (w, resnorms)
    grads = parameter_gradients(W, U, b_i, b_h, x, h, w, propagator)
    if dL_dh is not None:
        grads = grads + (input_gradients(W, U, b_i, b_h, x, h, w, propagator),)
    if keep_iterates:
        return (w, resnorms) + grads + (iterates,)
    return (w, resnorms) + grads


# --------------------------------------------------------------------------
# Stacked layers
# --------------------------------------------------------------------------
# The experiments use two GRU layers (Tables of Sec. 4) without saying how layers
# enter the time integration.  Reading taken here: the usual stacked network, layer
# j+1 reading the state sequence of layer j as its input sequence
# (x^{j+1}_t = h^j_t), each layer solved by its own MGRIT solve, layers in order.

def stacked_forward(params, x, h0s, solve):
    """params: list of (W, U, b_i, b_h); h0s: list of h_0 per layer; solve(layer,
    W, U, b_i, b_h, x, h0) -> h[(T+1),B,H].  Returns the list of state arrays."""
    hs = []
    inp = _f64(x)
    for j, (W, U, b_i, b_h) in enumerate(params):
        h = solve(j, W, U, b_i, b_h, inp, h0s[j])
        hs.append(h)
        inp = h[1:]
    return hs


def stacked_backward(params, x, hs, dL_dh_top, solve_adjoint):
    """Reverse pass through the stack: the top layer's source term is the loss
    derivative dL_dh_top[(T+1),B,H]; layer j receives dL/dx^{j+1}_t as the source
    at its point t.  solve_adjoint(layer, W, U, b_i, b_h, x, h, dL_dh) ->
    (w, dW, dU, db_i, db_h, dx).  Returns the per-layer results, bottom layer first."""
    out = [None] * len(params)
    src = _f64(dL_dh_top)
    for j in range(len(params) - 1, -1, -1):
        W, U, b_i, b_h = params[j]
        inp = _f64(x) if j == 0 else hs[j - 1][1:]
        res = solve_adjoint(j, W, U, b_i, b_h, inp, hs[j], src)
        out[j] = res
        dx = res[5]
        src = np.zeros_like(hs[j - 1]) if j > 0 else None
        if j > 0:
            src[1:] = dx                           # x^{j}_t = h^{j-1}_t for t = 1..T
    return out


# --------------------------------------------------------------------------
# Loss head used by the training-step workload (outside the MGRIT path)
# --------------------------------------------------------------------------

def cross_entropy_head(h_T, W_o, b_o, labels):
    """Mean cross-entropy of softmax(h_T W_o^T + b_o) against integer labels;
    returns (loss, dL/dh_T)."""
    h_T, W_o, b_o = map(_f64, (h_T, W_o, b_o))
    logits = h_T @ W_o.T + b_o
    logits = logits - logits.max(axis=1, keepdims=True)
    p = np.exp(logits)
    p /= p.sum(axis=1, keepdims=True)
    B = h_T.shape[0]
    loss = -np.mean(np.log(p[np.arange(B), labels]))
    p[np.arange(B), labels] -= 1.0
    return loss, (p / B) @ W_o


# --------------------------------------------------------------------------
# The library's entry points, by name, on host arrays
# --------------------------------------------------------------------------
# Same argument order and the same configuration fields as the C ABI of the HIP
# library (T, B, D, H are taken from the arrays; cf, levels, iters, fine_relax,
# propagator from cfg, a mapping or an object with those attributes), so that a
# test can call either side with one argument list.  Outputs are returned
# (float64) instead of written through pointers; there is no workspace.

def _cfg(cfg, name, default=None):
    if isinstance(cfg, dict):
        return cfg.get(name, default)
    return getattr(cfg, name, default)


def oracle_gru_serial_scan(cfg, W, U, b_i, b_h, x, h0):
    return serial_scan(W, U, b_i, b_h, x, h0, _cfg(cfg, "propagator", IMPLICIT))


def oracle_mgrit_gru_forward(cfg, W, U, b_i, b_h, x, h0, h_init):
    """Returns (h, resnorms[iters])."""
    return mgrit_forward(W, U, b_i, b_h, x, h0, h_init, _cfg(cfg, "cf"), _cfg(cfg, "levels"),
                         _cfg(cfg, "iters"), bool(_cfg(cfg, "fine_relax", 1)),
                         _cfg(cfg, "propagator", IMPLICIT))


def oracle_gru_serial_scan_backward(cfg, W, U, b_i, b_h, x, h, dL_dhT):
    """Returns (w, dW, dU, db_i, db_h)."""
    return serial_bptt(W, U, b_i, b_h, x, h, dL_dhT, _cfg(cfg, "propagator", IMPLICIT))


def oracle_mgrit_gru_backward(cfg, W, U, b_i, b_h, x, h, dL_dhT, w_init):
    """Returns (w, resnorms[iters], dW, dU, db_i, db_h)."""
    return mgrit_backward(W, U, b_i, b_h, x, h, dL_dhT, w_init, _cfg(cfg, "cf"),
                          _cfg(cfg, "levels"), _cfg(cfg, "iters"),
                          bool(_cfg(cfg, "fine_relax", 1)), _cfg(cfg, "propagator", IMPLICIT))


def oracle_gru_serial_scan_backward_steps(cfg, W, U, b_i, b_h, x, h, dL_dh):
    """Returns (w, dW, dU, db_i, db_h, dx)."""
    return serial_bptt_steps(W, U, b_i, b_h, x, h, dL_dh, _cfg(cfg, "propagator", IMPLICIT))


def oracle_mgrit_gru_backward_steps(cfg, W, U, b_i, b_h, x, h, dL_dh, w_init):
    """Returns (w, resnorms[iters], dW, dU, db_i, db_h, dx)."""
    return mgrit_backward(W, U, b_i, b_h, x, h, None, w_init, _cfg(cfg, "cf"), _cfg(cfg, "levels"),
                          _cfg(cfg, "iters"), bool(_cfg(cfg, "fine_relax", 1)),
                          _cfg(cfg, "propagator", IMPLICIT), dL_dh=dL_dh)
