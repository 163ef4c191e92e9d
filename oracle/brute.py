"""Scalar, per-sample brute-force evaluation for tiny inputs.

TEST INFRASTRUCTURE ONLY.  A second, independent writing of the objective of
Section 2.1 (no log-sum-exp shift, no matrix products, pure Python loops and
math.exp/math.log), of its gradient and of the explicit d x d Hessian
(d = p (C-1)).  Only meant for n <= ~50, p <= ~6, C <= ~4 and moderate logits;
it pins the vectorised oracle.

Flattening used for vectors of length d: index(j, c) = j * (C-1) + c, i.e. the
row-major flattening of the p x (C-1) matrix X.
"""
from __future__ import annotations

import math

import numpy as np


def _row_probs(a, X, p, K):
    z = [sum(a[j] * X[j][c] for j in range(p)) for c in range(K)]
    den = 1.0 + sum(math.exp(zc) for zc in z)
    return z, den, [math.exp(zc) / den for zc in z]


def loss(A, b, C, s, lam, rho, z, y, X):
    """s sum_i [log(1 + sum_c e^{<a_i,x_c>}) - <a_i, x_{b_i}>] + penalties."""
    n, p = len(A), len(A[0])
    K = C - 1
    tot = 0.0
    for i in range(n):
        zi, den, _ = _row_probs(A[i], X, p, K)
        tot += math.log(den)
        if b[i] < K:
            tot -= zi[b[i]]
    pen = 0.0
    for j in range(p):
        for c in range(K):
            pen += 0.5 * lam * X[j][c] ** 2
            pen += 0.5 * rho * (X[j][c] - z[j][c] + y[j][c] / rho) ** 2
    return s * tot + pen


def grad(A, b, C, s, lam, rho, z, y, X):
    n, p = len(A), len(A[0])
    K = C - 1
    G = [[0.0] * K for _ in range(p)]
    for i in range(n):
        _, _, P = _row_probs(A[i], X, p, K)
        for c in range(K):
            coef = P[c] - (1.0 if b[i] == c else 0.0)
            for j in range(p):
                G[j][c] += s * coef * A[i][j]
    for j in range(p):
        for c in range(K):
            G[j][c] += lam * X[j][c] + rho * (X[j][c] - z[j][c]) + y[j][c]
    return np.array(G)


def hessian(A, C, s, lam, rho, X):
    """H = s sum_i (diag(P_i) - P_i P_i^T) (x) a_i a_i^T + (lam + rho) I."""
    n, p = len(A), len(A[0])
    K = C - 1
    d = p * K
    H = np.zeros((d, d))
    for i in range(n):
        _, _, P = _row_probs(A[i], X, p, K)
        for c in range(K):
            for e in range(K):
                w = P[c] * ((1.0 if c == e else 0.0) - P[e])
                for j in range(p):
                    for k in range(p):
                        H[j * K + c, k * K + e] += s * w * A[i][j] * A[i][k]
    for t in range(d):
        H[t, t] += lam + rho
    return H
