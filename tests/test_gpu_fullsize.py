"""GPU parity at the full sizes of the benchmark workloads (the five dense ones and the sparse one
shaped like E18), in the launch configuration bench.py times (automatic kernel path, default
stream, library workspace).

The float64 oracle computes every output element (no sampling needed): d = p (C-1) is at most
38000 for the dense workloads, whose oracle cost is one or two dense products per call, and the
sparse workload's products with A are scipy's sparse ones (a few seconds each).  The Newton iteration
runs the workload's configured budget (Algorithm 3 with the CG cap of the appendix: 10 Newton x 10 CG
iterations, 20 x 20 for the large multiclass share) wherever the oracle finishes that within
ORACLE_SECONDS on the host; where it does not (the two largest workloads on a small host), the number of
Newton iterations is cut to what fits, never below 2, with the full CG budget, and the budget used is printed.
"""
import time

import dataclasses
import math

import numpy as np
import pytest
import torch

from oracle import nadmm_oracle as orc
from paper_1807_07132_amd import nadmm, workloads
from parity_utils import TOL_ITERATE, TOL_PRIMITIVE, oracle_newton_following, oracle_problem, rel_abs, rel_l2

pytestmark = pytest.mark.gpu

# name -> (expected kernel path, configured Newton iterations, configured CG iterations per Newton iteration)
FULL = {
    "tiny": (3, 1, 10),
    "image_like": (2, 10, 10),
    "wide": (4, 10, 10),
    "tall_binary": (3, 10, 10),
    "large_multiclass": (4, 20, 20),
    "e18_like": (5, 10, 10),
}
ORACLE_SECONDS = 75.0  # host time allowed for the oracle's Newton run of one workload


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    return t.detach().cpu().numpy()


@pytest.mark.parametrize("name", list(FULL))
def test_full_size_workload(name):
    path, T_cfg, K = FULL[name]
    print(f"full-size parity: {name}", flush=True)
    w = workloads.make(name, 0)
    gp = nadmm.Problem.from_workload(w)
    op = oracle_problem(w)
    nadmm.nadmm_set_kernel_path(0)
    assert nadmm.nadmm_query_kernel_path(gp) == path

    X = w.X0 if w.X0.any() else (np.random.default_rng(5).standard_normal(w.X0.shape) * 0.05).astype(np.float32)
    loss, grad = nadmm.nadmm_loss_grad(gp, dev(X))
    f_ref, g_ref = orc.loss_grad(op, X)
    assert rel_abs(loss.item(), f_ref) <= TOL_PRIMITIVE
    assert rel_l2(host(grad), g_ref) <= TOL_PRIMITIVE

    hv = nadmm.nadmm_hessvec(gp, dev(X), dev(w.V))
    t0 = time.perf_counter()
    hv_ref = orc.hessvec(op, X, w.V)
    t_hv = time.perf_counter() - t0
    err = rel_l2(host(hv), hv_ref)
    print(f"  Hv relative L2 error {err:.2e}", flush=True)
    assert err <= TOL_PRIMITIVE
    # properties that hold at any size: symmetry <w,Hv> = <v,Hw> and the curvature bound
    Wd = (np.random.default_rng(6).standard_normal(w.V.shape)).astype(np.float32)
    hw = nadmm.nadmm_hessvec(gp, dev(X), dev(Wd))
    a, b = float(np.sum(Wd.astype(np.float64) * host(hv))), float(np.sum(w.V.astype(np.float64) * host(hw)))
    assert a == pytest.approx(b, rel=1e-3, abs=1e-6 * np.linalg.norm(Wd) * np.linalg.norm(host(hv)))
    assert float(np.sum(w.V.astype(np.float64) * host(hv))) >= (w.lam + w.rho) * float(np.sum(w.V.astype(np.float64) ** 2)) * (1 - 1e-4)

    # a Newton iteration of the oracle costs about K + 2 passes of the kind just timed
    T = min(T_cfg, max(2, int(ORACLE_SECONDS / (t_hv * (K + 2)))))
    print(f"  Newton budget {T} x {K} (configured {T_cfg} x {K}; oracle Hessian-vector product {t_hv:.3f} s)", flush=True)
    params = nadmm.make_params(T, K, w.max_ls, 0.0, 0.0, w.beta, w.gamma)
    Xd = dev(w.X0.copy())
    st = nadmm.nadmm_local_newton(gp, Xd, params)
    w2 = dataclasses.replace(w, max_cg=K)
    X_ref, st_ref, _ = oracle_newton_following(op, w.X0, w2, st["alpha"], max_newton=T)
    assert st["newton_iters"] == st_ref["newton_iters"] == T
    assert st["alpha"] == pytest.approx([it["alpha"] for it in st_ref["iters"]], rel=1e-6)
    err = rel_l2(host(Xd), X_ref)
    print(f"  Newton iterate relative L2 error after {T} iterations {err:.2e}", flush=True)
    assert err <= TOL_ITERATE
    assert rel_abs(st["loss_final"], st_ref["loss_final"]) <= TOL_PRIMITIVE
    assert math.isfinite(st["grad_norm_final"])
