"""Plain float64 oracle of the ADMM outer solver (Algorithm 1) with fixed or residual-balanced penalty parameters.

TEST INFRASTRUCTURE ONLY -- see the package docstring.  The steps are taken in
the paper's order and notation (Section 2.3, equations x-update, z-update,
y-update and the closed form of the z-update for g(z) = lam/2 ||z||^2), with
numpy; the local subproblems are handed to nadmm_oracle.local_newton
(Algorithm 3).

Global consensus problem (Section 2.3):

    min  sum_i s * sum_{j in D_i} l_j(x_i) + lam/2 ||z||^2   s.t.  x_i = z

Iteration k (paper's sign convention of the multipliers y_i):

    x_i <- Algorithm 3 on  s sum_{j in D_i} l_j(x) + rho_i/2 ||z - x + y_i/rho_i||^2   (from the previous x_i)
    z   <- sum_i (rho_i x_i - y_i) / (lam + sum_i rho_i)                              (closed form)
    y_i <- y_i + rho_i (z - x_i)
    r_i  = z - x_i,   d_i = -rho_i (z - z_prev)                                         (residuals)

The local objective of nadmm_oracle writes its penalty as ||x - z + u/rho||^2;
the paper's y_i is u = -y_i there, and lam_local = 0 (the regulariser lives in
the z-update).

Stopping (reading of the printed tolerances, which put squared norms next to a
length): the stacked norms ||r|| = sqrt(sum_i ||r_i||^2), ||d|| likewise, are
compared with

    eps_pri  = sqrt(N) eps_abs + eps_rel * max{ sqrt(sum_i ||x_i||^2), sqrt(N) ||z|| }
    eps_dual = sqrt(d) eps_abs + eps_rel * sqrt(sum_i ||y_i||^2)

i.e. the printed expressions with every squared norm replaced by the norm.
The penalty parameters are inputs.  They stay fixed, or follow residual
balancing, which Section 2.3 names as the customary adaptive rule (the spectral
selection that the paper itself uses is defined in a cited work only and is not
part of this oracle).  The paper gives no formula for residual balancing; the
rule below is the published one of the reference it cites for it, applied by
one common factor c to all rho_i: after an iteration whose residuals satisfy
||r|| > mu ||d||, c <- tau c; if ||d|| > mu ||r||, c <- c / tau; else unchanged.
The multipliers y_i are the unscaled ones, so they are not touched by a change.

Parity status: pinned by tests/test_admm_oracle_pins.py (closed-form
z-update against a direct minimisation, the invariant sum_i y_i = -lam z,
convergence of z to the minimiser of the centralised problem, one worker
without regulariser = repeated proximal steps; residual balancing: never
triggered = the fixed-penalty iterates, the invariant and the limit point are
kept, a badly scaled penalty is moved towards balance and fewer iterations are
needed than with the fixed one; the tolerances on numbers worked by hand, and
the balancing update step by step on a two-worker scalar example whose first
iteration has a closed form and whose later x-updates are checked by
substitution into the scalar stationarity condition).  The rule's constants and
its common-factor form are this build's reading, not the paper's text.
"""
from __future__ import annotations

from dataclasses import replace
from typing import List, Sequence

import numpy as np

from . import nadmm_oracle as orc


def z_update(xs: Sequence[np.ndarray], ys: Sequence[np.ndarray], rhos: Sequence[float], lam: float) -> np.ndarray:
    """Closed form of the z-update for g(z) = lam/2 ||z||^2 (Section 2.3)."""
    num = np.zeros_like(np.asarray(xs[0], dtype=np.float64))
    for x, y, rho in zip(xs, ys, rhos):
        num = num + rho * np.asarray(x, dtype=np.float64) - np.asarray(y, dtype=np.float64)
    return num / (lam + float(np.sum(rhos)))


def tolerances(xs, ys, z, eps_abs: float, eps_rel: float):
    N = len(xs)
    d = np.asarray(z).size
    sx = np.sqrt(sum(float(np.sum(np.asarray(x, dtype=np.float64) ** 2)) for x in xs))
    sy = np.sqrt(sum(float(np.sum(np.asarray(y, dtype=np.float64) ** 2)) for y in ys))
    nz = np.sqrt(N) * float(np.sqrt(np.sum(np.asarray(z, dtype=np.float64) ** 2)))
    return np.sqrt(N) * eps_abs + eps_rel * max(sx, nz), np.sqrt(d) * eps_abs + eps_rel * sy


def admm(shards: List[orc.Problem], lam: float, rhos: Sequence[float], X0, max_outer: int,
         max_newton: int, max_cg: int, cg_tol: float, grad_tol: float, beta: float, gamma: float, max_ls: int,
         eps_abs: float = 0.0, eps_rel: float = 0.0, forced_alphas=None,
         penalty_rule: int = 0, rb_mu: float = 10.0, rb_tau: float = 2.0):
    """Algorithm 1.  `shards[i]` carries A_i, b_i, C and the loss scale s; its lam,
    rho, z, y fields are overwritten per iteration.  `forced_alphas[k][i]`, if given, is handed to the
    local solve of worker i in outer iteration k (see nadmm_oracle.local_newton).
    penalty_rule 0: the penalties stay rhos; 1: residual balancing (module docstring).
    Returns (z, xs, ys, history); ys in the paper's sign convention."""
    N = len(shards)
    X0 = np.asarray(X0, dtype=np.float64)
    xs = [X0.copy() for _ in range(N)]
    ys = [np.zeros_like(X0) for _ in range(N)]
    z = np.zeros_like(X0)
    hist = []
    rhos0 = [float(r) for r in rhos]
    c = 1.0
    for k in range(max_outer):
        rhos = [c * r for r in rhos0]
        local = []
        for i in range(N):
            prob = replace(shards[i], lam=0.0, rho=float(rhos[i]), z=z, y=-ys[i])
            fa = None if forced_alphas is None or k >= len(forced_alphas) else forced_alphas[k][i]
            xs[i], st = orc.local_newton(prob, xs[i], max_newton, max_cg, cg_tol, grad_tol, beta, gamma, max_ls,
                                         forced_alphas=fa)
            local.append(st)
        z_prev = z
        z = z_update(xs, ys, rhos, lam)
        ys = [ys[i] + rhos[i] * (z - xs[i]) for i in range(N)]
        r = np.sqrt(sum(float(np.sum((z - xs[i]) ** 2)) for i in range(N)))
        dn = np.sqrt(sum(float(np.sum((rhos[i] * (z - z_prev)) ** 2)) for i in range(N)))
        e_pri, e_dual = tolerances(xs, ys, z, eps_abs, eps_rel)
        hist.append(dict(r_norm=r, d_norm=dn, eps_pri=e_pri, eps_dual=e_dual, z=z.copy(), rho_scale=c,
                         xs=[x.copy() for x in xs], ys=[y.copy() for y in ys], local=local))
        if r <= e_pri and dn <= e_dual:
            break
        if penalty_rule == 1:
            if r > rb_mu * dn:
                c = c * rb_tau
            elif dn > rb_mu * r:
                c = c / rb_tau
    return z, xs, ys, hist
