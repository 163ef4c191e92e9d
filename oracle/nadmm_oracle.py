"""Plain float64 oracle of one ADMM worker's local x-update (Newton-ADMM).

TEST INFRASTRUCTURE ONLY -- see the package docstring.  Every function is the
definition (or the algorithm's steps, in the paper's order) written out with
numpy; no blocking, fusion or reordering.  Inputs may be float32 arrays; they
are up-cast, so that rounding of the inputs is not part of any error.

Objective of the local subproblem (x-update of the ADMM iteration, Section 2.3,
with the l2 regulariser kept local as a run-time parameter; lam = 0 gives the
paper's x-update exactly):

    Fhat(X) = s * sum_i l_i(X) + lam/2 ||X||^2 + rho/2 ||X - z + y/rho||^2

    l_i(X)  = log(1 + sum_c exp<a_i, x_c>) - sum_c 1(b_i = c) <a_i, x_c>
              (cross-entropy with C-1 free weight vectors, Section 2.1)

Conventions
    A   n x p, row i is sample a_i
    b   n labels in 0..C-1; class C-1 is the reference class whose logit is 0
        (the paper numbers classes 1..C with class C as the reference)
    X   p x (C-1); column c is the paper's x_{c+1}.  The paper's stacked vector
        x = [x_1; ...; x_{C-1}] is the column-major flattening of X.  All
        vector operations used here (inner products, norms, axpy) do not
        depend on the flattening order.
        A may also be a scipy.sparse matrix (the paper reports on sparse as well as
        dense data sets, Section 1): it is held as float64 compressed sparse
        rows and every product with it below is scipy's sparse-times-dense
        routine, a library primitive standing for the same matrix product.
        Explicit entries repeated at one position are added up (scipy's rule).
    s   loss scale (1 = the paper's plain sum, 1/n = mean)
    z,y consensus variable and multiplier, same shape as X.  Sign convention of
        y: the penalty is ||X - z + y/rho||^2 (scaled form); the paper writes
        ||z - x + y/rho||^2, which is this one with y replaced by -y.

Parity status: every function below is pinned by tests/test_oracle_pins.py
(closed forms, library routines on the over-parametrised C-class form, finite
differences, explicit brute-force Hessians, Krylov-subspace minimisation,
direct solves and an independent minimiser; sparse storage of A against the
dense results in tests/test_sparse_oracle_pins.py).  The paper prints no worked
numerical example, so no value of the paper's is available as a pin.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np
import scipy.sparse as sp


@dataclass
class Problem:
    """One worker's data share and penalty parameters."""

    A: np.ndarray
    b: np.ndarray
    C: int
    s: float = 1.0
    lam: float = 0.0
    rho: float = 1.0
    z: Optional[np.ndarray] = None
    y: Optional[np.ndarray] = None
    A64: object = field(init=False, repr=False)   # float64 ndarray or scipy.sparse.csr_matrix

    def __post_init__(self):
        if sp.issparse(self.A):
            self.A64 = sp.csr_matrix(self.A, dtype=np.float64)
        else:
            self.A64 = np.asarray(self.A, dtype=np.float64)
        self.b = np.asarray(self.b, dtype=np.int64)
        n, p = self.A64.shape
        shape = (p, self.C - 1)
        self.z = np.zeros(shape) if self.z is None else np.asarray(self.z, dtype=np.float64).reshape(shape)
        self.y = np.zeros(shape) if self.y is None else np.asarray(self.y, dtype=np.float64).reshape(shape)
        self.s = float(self.s)
        self.lam = float(self.lam)
        self.rho = float(self.rho)

    @property
    def n(self):
        return self.A64.shape[0]

    @property
    def p(self):
        return self.A64.shape[1]


def _as_X(prob: Problem, X) -> np.ndarray:
    return np.asarray(X, dtype=np.float64).reshape(prob.p, prob.C - 1)


# --------------------------------------------------------------------------
# Section 2.1 / 2.2: logits, log-sum-exp pieces, probabilities, row losses
# --------------------------------------------------------------------------
def logits(prob: Problem, X) -> np.ndarray:
    """Z[i, c] = <a_i, x_c> for the C-1 free classes (Section 2.1)."""
    return prob.A64 @ _as_X(prob, X)


def lse_parts(Z: np.ndarray):
    """M(a_i) and alpha(a_i) of Section 2.2 (eqs. max_x and log_sum_trick).

    M_i     = max{0, Z_i1, ..., Z_i,C-1}          (0 is the reference logit)
    alpha_i = exp(-M_i) + sum_c exp(Z_ic - M_i)
    Also returns E[i, c] = exp(Z_ic - M_i).
    """
    M = np.maximum(0.0, Z.max(axis=1))
    E = np.exp(Z - M[:, None])
    alpha = np.exp(-M) + E.sum(axis=1)
    return M, alpha, E


def probabilities(prob: Problem, X) -> np.ndarray:
    """P[i, c] = h(a_i, x_c) = exp(Z_ic - M_i) / alpha_i (Section 2.6)."""
    M, alpha, E = lse_parts(logits(prob, X))
    return E / alpha[:, None]


def row_losses(prob: Problem, X) -> np.ndarray:
    """l_i = M_i + log(alpha_i) - Z_{i, b_i} 1(b_i < C-1) (Sections 2.1, 2.2)."""
    Z = logits(prob, X)
    M, alpha, _ = lse_parts(Z)
    ell = M + np.log(alpha)
    free = prob.b < prob.C - 1
    idx = np.nonzero(free)[0]
    ell[idx] -= Z[idx, prob.b[idx]]
    return ell


def penalty(prob: Problem, X) -> float:
    """lam/2 ||X||^2 + rho/2 ||X - z + y/rho||^2 (x-update, Section 2.3)."""
    X = _as_X(prob, X)
    u = X - prob.z + prob.y / prob.rho
    return 0.5 * prob.lam * float(np.sum(X * X)) + 0.5 * prob.rho * float(np.sum(u * u))


def loss(prob: Problem, X) -> float:
    """Fhat(X), the local objective."""
    return prob.s * float(np.sum(row_losses(prob, X))) + penalty(prob, X)


def _onehot_free(prob: Problem) -> np.ndarray:
    Y = np.zeros((prob.n, prob.C - 1))
    idx = np.nonzero(prob.b < prob.C - 1)[0]
    Y[idx, prob.b[idx]] = 1.0
    return Y


def grad(prob: Problem, X) -> np.ndarray:
    """Gradient of Fhat (the paper names it, eq. Newton_G, without a formula).

    d l_i / d x_c = (P_ic - 1(b_i = c)) a_i, hence
    G = s A^T (P - Y) + lam X + rho (X - z) + y.
    """
    X = _as_X(prob, X)
    P = probabilities(prob, X)
    return prob.s * (prob.A64.T @ (P - _onehot_free(prob))) + prob.lam * X + prob.rho * (X - prob.z) + prob.y


def loss_grad(prob: Problem, X):
    return loss(prob, X), grad(prob, X)


# --------------------------------------------------------------------------
# Section 2.6: Hessian-vector product without forming the Hessian
# --------------------------------------------------------------------------
def hessvec(prob: Problem, X, V) -> np.ndarray:
    """H(X) V as in Section 2.6 (eqs. matrix-a, matrix-b, matrix-c, hessianvec).

    W = A V                     (the paper's matrix V of inner products)
    P = h(a_i, x_c)             (the paper's matrix W)
    D = P o W - P o ((P o W) e e^T)   (the paper's U)
    H V = s A^T D + (lam + rho) V     (data term plus the two quadratic terms)
    """
    V = _as_X(prob, V)
    P = probabilities(prob, X)
    W = prob.A64 @ V
    PW = P * W
    t = PW.sum(axis=1)
    D = PW - P * t[:, None]
    return prob.s * (prob.A64.T @ D) + (prob.lam + prob.rho) * V


# --------------------------------------------------------------------------
# Section 2.4: CG with early stopping, Armijo backtracking, Newton iteration
# --------------------------------------------------------------------------
def cg(prob: Problem, X, g, max_iter: int, tol: float):
    """Approximate solution of H(X) p = -g by conjugate gradients.

    Starts from p = 0, plain (unpreconditioned) CG with the recurrence
    residual; stops when ||H p + g|| <= tol ||g|| (eq. inexact) or after
    max_iter iterations, and returns the last iterate.  A direction of
    non-positive or non-finite curvature ends the iteration (it cannot occur
    for H >= (lam + rho) I in exact arithmetic).
    Returns (p, iterations done, ||r|| / ||g||).
    """
    g = _as_X(prob, g)
    p = np.zeros_like(g)
    r = -g.copy()
    d = r.copy()
    rr = float(np.sum(r * r))
    gnorm = np.sqrt(rr)
    iters = 0
    if gnorm == 0.0:
        return p, 0, 0.0
    for _ in range(max_iter):
        q = hessvec(prob, X, d)
        dq = float(np.sum(d * q))
        if not np.isfinite(dq) or dq <= 0.0:
            break
        a = rr / dq
        p = p + a * d
        r = r - a * q
        rr_new = float(np.sum(r * r))
        iters += 1
        if np.sqrt(rr_new) <= tol * gnorm:
            rr = rr_new
            break
        d = r + (rr_new / rr) * d
        rr = rr_new
    return p, iters, np.sqrt(rr) / gnorm


def line_search(prob: Problem, X, p, g, beta: float, gamma: float, max_ls: int, loss_at_X=None):
    """Backtracking Armijo line search, Algorithm 2 taken literally.

    alpha = 1, i = 0; while F(X + alpha p) > F(X) + alpha beta <p, g>:
    leave the loop if i > max_ls, else i += 1 and alpha *= gamma.
    The smallest step that can be returned is gamma^(max_ls + 1); when the
    loop is left by the break the Armijo condition does not hold at the
    returned alpha and armijo_ok is False (the step is still taken by the
    Newton iteration, Algorithm 3 has no reject branch).
    Returns (alpha, F(X + alpha p), armijo_ok, number of evaluations of F).
    """
    X = _as_X(prob, X)
    p = _as_X(prob, p)
    g = _as_X(prob, g)
    f0 = loss(prob, X) if loss_at_X is None else float(loss_at_X)
    slope = float(np.sum(p * g))
    alpha = 1.0
    i = 0
    evals = 1
    f_new = loss(prob, X + alpha * p)
    ok = True
    while f_new > f0 + alpha * beta * slope:
        if i > max_ls:
            ok = False
            break
        i += 1
        alpha *= gamma
        f_new = loss(prob, X + alpha * p)
        evals += 1
    return alpha, f_new, ok, evals


def local_newton(prob: Problem, X0, max_newton: int, max_cg: int, cg_tol: float,
                 grad_tol: float, beta: float, gamma: float, max_ls: int,
                 forced_alphas=None):
    """Algorithm 3: inexact Newton iteration on the local subproblem.

    Per iteration: form g; stop if ||g|| < grad_tol; p from cg(); alpha from
    line_search(); X <- X + alpha p.  `forced_alphas`, if given, replaces the
    line-search result of iteration t by forced_alphas[t] (used by the parity
    harness when a floating-point tie in the Armijo test is decided
    differently by the two sides).
    Returns (X, stats dict with per-iteration records); grad_norm_final is the
    norm of the last gradient that was formed (at the start of the last
    iteration, or at the point where the iteration stopped).
    """
    X = _as_X(prob, X0).copy()
    hist = []
    f = loss(prob, X)
    stats = dict(newton_iters=0, cg_iters_total=0, ls_evals_total=0, armijo_failed=0,
                 loss_initial=f, loss_final=f, grad_norm_final=float("nan"), iters=hist)
    for t in range(max_newton):
        g = grad(prob, X)
        gn = float(np.sqrt(np.sum(g * g)))
        stats["grad_norm_final"] = gn
        if gn < grad_tol:
            break
        p, k, relres = cg(prob, X, g, max_cg, cg_tol)
        alpha, f_new, ok, evals = line_search(prob, X, p, g, beta, gamma, max_ls, loss_at_X=f)
        if forced_alphas is not None and t < len(forced_alphas):
            alpha = float(forced_alphas[t])
            f_new = loss(prob, X + alpha * p)
        hist.append(dict(loss=f, grad_norm=gn, cg_iters=k, relres=relres, alpha=alpha,
                         armijo_ok=ok, ls_evals=evals, X=X.copy(), p=p.copy(), g=g.copy()))
        X = X + alpha * p
        f = f_new
        stats["newton_iters"] += 1
        stats["cg_iters_total"] += k
        stats["ls_evals_total"] += evals
        stats["armijo_failed"] += 0 if ok else 1
        stats["loss_final"] = f
    return X, stats
