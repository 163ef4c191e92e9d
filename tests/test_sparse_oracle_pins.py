"""Pins of the oracle's sparse storage of A (CPU only).

With a scipy.sparse A the oracle runs the same formulas through scipy's
sparse-times-dense product.  That the result is the one of the (separately
pinned) dense oracle is checked here against a dense matrix that is NOT made by
scipy: it is filled entry by entry from the raw CSR arrays with a Python loop,
repeated positions added up, which is the meaning of the three arrays that the
GPU library's header states.  The workload generator's CSR / CSC pair is checked
to describe one matrix.
"""
import numpy as np
import scipy.sparse as sp

from oracle import nadmm_oracle as orc
from paper_1807_07132_amd import workloads as wl


def _dense_from_csr_arrays(indptr, indices, data, shape):
    D = np.zeros(shape, dtype=np.float64)
    for i in range(shape[0]):
        for k in range(int(indptr[i]), int(indptr[i + 1])):
            D[i, int(indices[k])] += float(data[k])
    return D


def _pair(seed, n=60, p=35, C=4, repeats=False):
    rng = np.random.default_rng(seed)
    lens = rng.integers(0, 9, size=n)
    lens[3] = 0                      # an empty row
    indptr = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    indices = rng.integers(0, p - 2, size=indptr[-1]).astype(np.int32)   # the last two columns stay empty
    if not repeats:
        for i in range(n):           # distinct columns within a row
            k0, k1 = indptr[i], indptr[i + 1]
            indices[k0:k1] = rng.choice(p - 2, size=k1 - k0, replace=False)
    data = rng.standard_normal(indptr[-1]).astype(np.float32)
    A = sp.csr_matrix((data, indices, indptr), shape=(n, p))
    b = rng.integers(0, C, size=n)
    z = rng.standard_normal((p, C - 1)) * 0.3
    y = rng.standard_normal((p, C - 1)) * 0.3
    kw = dict(C=C, s=1.0 / n, lam=0.05, rho=0.7, z=z, y=y)
    dense = _dense_from_csr_arrays(indptr, indices, data, (n, p))
    return orc.Problem(A, b, **kw), orc.Problem(dense, b, **kw), rng


def test_sparse_storage_gives_the_dense_results():
    for seed, repeats in ((0, False), (1, True)):
        ps, pd, rng = _pair(seed, repeats=repeats)
        X = rng.standard_normal((pd.p, pd.C - 1)) * 0.5
        V = rng.standard_normal((pd.p, pd.C - 1))
        assert isinstance(orc.logits(ps, X), np.ndarray)
        np.testing.assert_allclose(orc.logits(ps, X), orc.logits(pd, X), rtol=0, atol=1e-13)
        assert abs(orc.loss(ps, X) - orc.loss(pd, X)) <= 1e-13 * abs(orc.loss(pd, X))
        np.testing.assert_allclose(orc.grad(ps, X), orc.grad(pd, X), rtol=0, atol=1e-13)
        np.testing.assert_allclose(orc.hessvec(ps, X, V), orc.hessvec(pd, X, V), rtol=0, atol=1e-13)


def test_sparse_newton_iterates_follow_the_dense_ones():
    ps, pd, rng = _pair(2)
    X0 = rng.standard_normal((pd.p, pd.C - 1)) * 0.2
    args = (3, 6, 1e-8, 0.0, 1e-4, 0.5, 10)
    Xs, ss = orc.local_newton(ps, X0, *args)
    Xd, sd = orc.local_newton(pd, X0, *args)
    assert [it["alpha"] for it in ss["iters"]] == [it["alpha"] for it in sd["iters"]]
    np.testing.assert_allclose(Xs, Xd, rtol=0, atol=1e-11)
    assert sd["loss_final"] < sd["loss_initial"]


def test_generator_csr_and_csc_describe_one_matrix():
    w = wl.sparse_generic(300, 500, 5, 12, seed=3)
    A, At = w.A, w.extra["csc"]
    assert A.dtype == np.float32 and At.dtype == np.float32
    assert A.indptr[0] == 0 and A.indptr[-1] == A.nnz == At.nnz and np.all(np.diff(A.indptr) >= 0)
    D = _dense_from_csr_arrays(A.indptr, A.indices, A.data, A.shape)
    Dt = _dense_from_csr_arrays(At.indptr, At.indices, At.data, (A.shape[1], A.shape[0]))
    assert np.array_equal(D, Dt.T)
    assert (np.diff(At.indptr) == 0).any() and np.diff(At.indptr).max() > 20 * np.median(np.diff(At.indptr)[np.diff(At.indptr) > 0])
