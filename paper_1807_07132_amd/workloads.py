"""Seeded synthetic workloads shaped like the paper's data sets (Table 1).

This module only draws inputs.  It holds none of the method's arithmetic and is
imported neither by the HIP binding nor by the CPU oracle; tests, the smoke
check and the benchmark hand the same float32 arrays to both sides.

The real data sets (HIGGS, MNIST, CIFAR-10, E18) are not available; the
workloads below are synthetic stand-ins with their shapes.  `e18_like` is the
sparse one: A is a scipy.sparse CSR matrix of float32 values and `extra["csc"]` holds the same matrix
compressed by columns, the second view the GPU library asks for.  Draws are made in
float64 with numpy's PCG64 and cast to float32; independent sub-streams are
spawned from the seed in the fixed order A, labels, X, z, y, V.

`n` may be overridden (same recipe, fewer rows) for parity tests at sizes the
CPU oracle finishes quickly.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np
import scipy.sparse as sp

_ROW_CHUNK = 8192


@dataclass
class Workload:
    name: str
    A: object               # n x p float32: row-major ndarray, or scipy.sparse.csr_matrix
    b: np.ndarray           # n int32 labels in 0..C-1 (C-1 = reference class)
    C: int
    X0: np.ndarray          # p x (C-1) float32 starting point
    z: np.ndarray           # p x (C-1) float32
    y: np.ndarray           # p x (C-1) float32
    V: np.ndarray           # p x (C-1) float32 direction for Hessian-vector products
    lam: float
    rho: float
    s: float                # loss scale (1/n)
    max_newton: int = 10
    max_cg: int = 10
    max_ls: int = 10
    cg_tol: float = 0.0
    grad_tol: float = 0.0
    beta: float = 1e-4
    gamma: float = 0.5
    extra: dict = field(default_factory=dict)

    @property
    def sparse(self):
        return sp.issparse(self.A)

    @property
    def n(self):
        return self.A.shape[0]

    @property
    def p(self):
        return self.A.shape[1]


def _streams(seed):
    return [np.random.Generator(np.random.PCG64(s)) for s in np.random.SeedSequence(seed).spawn(6)]


def _normal32(rng, shape, std=1.0):
    return (rng.standard_normal(shape) * std).astype(np.float32)


def _balanced_labels(rng, n, C):
    b = (np.arange(n) % C).astype(np.int32)
    return b[rng.permutation(n)]


def _chunked_rows(n, p, fill):
    A = np.empty((n, p), dtype=np.float32)
    for r0 in range(0, n, _ROW_CHUNK):
        r1 = min(n, r0 + _ROW_CHUNK)
        A[r0:r1] = fill(r0, r1)
    return A


def tiny(seed=0, n=1000):
    """1000 x 20, C = 3, i.i.d. N(0,1) features, uniform labels, X0 = 0."""
    p, C = 20, 3
    rA, rb, rX, rz, ry, rV = _streams(seed)
    A = _normal32(rA, (n, p))
    b = rb.integers(0, C, size=n).astype(np.int32)
    X0 = np.zeros((p, C - 1), dtype=np.float32)
    z = _normal32(rz, (p, C - 1), np.sqrt(0.1))
    y = np.zeros((p, C - 1), dtype=np.float32)
    V = _normal32(rV, (p, C - 1))
    return Workload("tiny_1000x20_C3", A, b, C, X0, z, y, V, lam=1e-3, rho=1.0, s=1.0 / n,
                    max_newton=1, max_cg=10, max_ls=10)


def image_like(seed=0, n=60000):
    """60000 x 784, C = 10: uniform[0,1] values with 80 % exact zeros, stored dense."""
    p, C = 784, 10
    rA, rb, rX, rz, ry, rV = _streams(seed)

    def fill(r0, r1):
        u = rA.random((r1 - r0, p))
        keep = rA.random((r1 - r0, p)) < 0.2
        return (u * keep).astype(np.float32)

    A = _chunked_rows(n, p, fill)
    b = _balanced_labels(rb, n, C)
    X0 = _normal32(rX, (p, C - 1), 0.05)
    z = _normal32(rz, (p, C - 1), 0.1)
    y = _normal32(ry, (p, C - 1), 0.1)
    V = _normal32(rV, (p, C - 1))
    return Workload("image_like_60000x784_C10", A, b, C, X0, z, y, V, lam=1e-3, rho=1.0, s=1.0 / n,
                    max_newton=10, max_cg=10, max_ls=10)


def _mixture(rA, b, p, mean_std, unit_rows):
    C = int(b.max()) + 1
    mu = rA.standard_normal((C, p)) * mean_std

    def fill(r0, r1):
        rows = mu[b[r0:r1]] + rA.standard_normal((r1 - r0, p))
        if unit_rows:
            rows /= np.linalg.norm(rows, axis=1, keepdims=True)
        return rows.astype(np.float32)

    return _chunked_rows(len(b), p, fill)


def wide(seed=0, n=50000):
    """50000 x 3072, C = 10: class means N(0, 0.25 I), unit-variance noise, unit-norm rows."""
    p, C = 3072, 10
    rA, rb, rX, rz, ry, rV = _streams(seed)
    b = _balanced_labels(rb, n, C)
    A = _mixture(rA, b, p, 0.5, True)
    X0 = np.zeros((p, C - 1), dtype=np.float32)
    z = _normal32(rz, (p, C - 1), 0.1)
    y = _normal32(ry, (p, C - 1), 0.1)
    V = _normal32(rV, (p, C - 1))
    return Workload("wide_50000x3072_C10", A, b, C, X0, z, y, V, lam=1e-3, rho=1.0, s=1.0 / n,
                    max_newton=10, max_cg=10, max_ls=10)


def tall_binary(seed=0, n=1375000):
    """1375000 x 28, C = 2: correlated standardised Gaussian features, noisy logistic labels."""
    p, C = 28, 2
    rA, rb, rX, rz, ry, rV = _streams(seed)
    Q, _ = np.linalg.qr(rA.standard_normal((p, p)))
    Sigma = (Q * np.logspace(0.0, 1.0, p)) @ Q.T          # condition number 10
    L = np.linalg.cholesky(Sigma)
    A = _chunked_rows(n, p, lambda r0, r1: (rA.standard_normal((r1 - r0, p)) @ L).astype(np.float32))
    A /= A.std(axis=0, dtype=np.float64).astype(np.float32)
    w_true = rb.standard_normal(p) / np.sqrt(p)
    t = A.astype(np.float64) @ w_true
    positive = rb.random(n) < 1.0 / (1.0 + np.exp(-t))
    flip = rb.random(n) < 0.05
    positive ^= flip
    b = np.where(positive, 0, 1).astype(np.int32)          # 0 = class with the free weight column
    X0 = np.zeros((p, 1), dtype=np.float32)
    z = _normal32(rz, (p, 1), 0.1)
    y = _normal32(ry, (p, 1), 0.1)
    V = _normal32(rV, (p, 1))
    return Workload("tall_binary_1375000x28_C2", A, b, C, X0, z, y, V, lam=1e-4, rho=0.5, s=1.0 / n,
                    max_newton=10, max_cg=10, max_ls=10)


def large_multiclass(seed=0, n=250000):
    """250000 x 2000, C = 20: class means N(0, 0.1 I), unit-variance noise."""
    p, C = 2000, 20
    rA, rb, rX, rz, ry, rV = _streams(seed)
    b = _balanced_labels(rb, n, C)
    A = _mixture(rA, b, p, np.sqrt(0.1), False)
    X0 = np.zeros((p, C - 1), dtype=np.float32)
    z = _normal32(rz, (p, C - 1), 0.1)
    y = _normal32(ry, (p, C - 1), 0.1)
    V = _normal32(rV, (p, C - 1))
    return Workload("large_multiclass_250000x2000_C20", A, b, C, X0, z, y, V, lam=1e-5, rho=1.0, s=1.0 / n,
                    max_newton=20, max_cg=20, max_ls=10)


def generic(n, p, C, seed=0, lam=1e-3, rho=1.0, scale=1.0, x_std=0.3, mean=False):
    """Free-shape Gaussian workload for edge-case and sweep tests."""
    rA, rb, rX, rz, ry, rV = _streams(seed)
    A = _normal32(rA, (n, p), scale)
    b = rb.integers(0, C, size=n).astype(np.int32)
    X0 = _normal32(rX, (p, C - 1), x_std)
    z = _normal32(rz, (p, C - 1), 0.3)
    y = _normal32(ry, (p, C - 1), 0.3)
    V = _normal32(rV, (p, C - 1))
    return Workload(f"generic_{n}x{p}_C{C}", A, b, C, X0, z, y, V, lam=lam, rho=rho,
                    s=(1.0 / max(n, 1)) if mean else 1.0, max_newton=3, max_cg=5, max_ls=10)


def _sparse_counts(rA, n, p, nnz_per_row, sigma):
    """CSR/CSC pair with skewed column popularity: column weights are log-normal (a few columns are
    present in most rows, most columns in few or none), positions are drawn with replacement and
    repeated positions are merged, values are log(1 + k) of geometric counts k >= 1."""
    w = np.exp(sigma * rA.standard_normal(p))
    cdf = np.cumsum(w / w.sum())
    cdf[-1] = 1.0
    draws = int(n) * int(nnz_per_row)
    key = np.empty(draws, dtype=np.int64)
    step = 1 << 24
    for k0 in range(0, draws, step):
        k1 = min(draws, k0 + step)
        cols = np.searchsorted(cdf, rA.random(k1 - k0), side="right").astype(np.int64)
        np.minimum(cols, p - 1, out=cols)
        key[k0:k1] = rA.integers(0, n, size=k1 - k0, dtype=np.int64) * p + cols
    key = np.unique(key)                                   # sorted by (row, column), repeats merged
    rows = (key // p).astype(np.int64)
    cols = (key % p).astype(np.int32)
    del key
    val = np.log1p(rA.geometric(0.5, size=cols.size)).astype(np.float32)
    indptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(np.bincount(rows, minlength=n), out=indptr[1:])
    A = sp.csr_matrix((val, cols, indptr), shape=(n, p))
    A.has_sorted_indices = True
    return A


def _with_csc(A):
    At = A.tocsc()
    At.sort_indices()
    return At


def e18_like(seed=0, n=40628, p=279998, nnz_per_row=2000):
    """One of 32 workers' share of a data set shaped like E18 (Table 1: 1,300,128 samples, 279,998
    features, 20 classes), stored sparse: about nnz_per_row entries per row, log-normal column
    popularity (sigma 2), balanced labels."""
    C = 20
    rA, rb, rX, rz, ry, rV = _streams(seed)
    A = _sparse_counts(rA, n, p, nnz_per_row, 2.0)
    b = _balanced_labels(rb, n, C)
    X0 = np.zeros((p, C - 1), dtype=np.float32)
    z = _normal32(rz, (p, C - 1), 0.1)
    y = _normal32(ry, (p, C - 1), 0.1)
    V = _normal32(rV, (p, C - 1))
    return Workload(f"e18_like_{n}x{p}_C{C}_sparse", A, b, C, X0, z, y, V, lam=1e-5, rho=1.0, s=1.0 / n,
                    max_newton=10, max_cg=10, max_ls=10, extra={"csc": _with_csc(A)})


def sparse_generic(n, p, C, nnz_per_row, seed=0, sigma=2.0, lam=1e-3, rho=1.0, x_std=0.3, mean=True):
    """Free-shape sparse workload (same recipe as e18_like) for edge-case tests."""
    rA, rb, rX, rz, ry, rV = _streams(seed)
    A = _sparse_counts(rA, n, p, nnz_per_row, sigma)
    b = rb.integers(0, C, size=n).astype(np.int32)
    X0 = _normal32(rX, (p, C - 1), x_std)
    z = _normal32(rz, (p, C - 1), 0.3)
    y = _normal32(ry, (p, C - 1), 0.3)
    V = _normal32(rV, (p, C - 1))
    return Workload(f"sparse_{n}x{p}_C{C}", A, b, C, X0, z, y, V, lam=lam, rho=rho,
                    s=(1.0 / max(n, 1)) if mean else 1.0, max_newton=3, max_cg=5, max_ls=10,
                    extra={"csc": _with_csc(A)})


CONFIGS = {
    "tiny": tiny,
    "image_like": image_like,
    "wide": wide,
    "tall_binary": tall_binary,
    "large_multiclass": large_multiclass,
    "e18_like": e18_like,
}


def make(name: str, seed: int = 0, n: Optional[int] = None) -> Workload:
    fn = CONFIGS[name]
    return fn(seed) if n is None else fn(seed, n)
