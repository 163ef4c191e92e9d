"""Helpers of the GPU-vs-oracle parity tests (the oracle side runs on the CPU in float64)."""
import numpy as np

from oracle import nadmm_oracle as orc

# spec tolerances: relative L2 error of loss / gradient / Hv, and of Newton-CG iterates
TOL_PRIMITIVE = 1e-4
TOL_ITERATE = 1e-3


def oracle_problem(w, s=None, with_zy=True):
    return orc.Problem(w.A, w.b, w.C, s=w.s if s is None else s, lam=w.lam, rho=w.rho,
                       z=w.z if with_zy else None, y=w.y if with_zy else None)


def rel_l2(got, ref):
    got = np.asarray(got, dtype=np.float64).reshape(-1)
    ref = np.asarray(ref, dtype=np.float64).reshape(-1)
    den = np.linalg.norm(ref)
    return np.linalg.norm(got - ref) / (den if den > 0 else 1.0)


def rel_abs(got, ref):
    return abs(float(got) - float(ref)) / max(abs(float(ref)), 1e-300)


def armijo_margin(prob, X, p, g, alpha, beta, f0):
    """lhs - rhs of the Armijo test at alpha, in float64."""
    return orc.loss(prob, X + alpha * p) - (f0 + alpha * beta * float(np.sum(p * g)))


def oracle_newton_following(prob, X0, w, gpu_alphas, max_newton=None):
    """Oracle Newton run; where its line search disagrees with the GPU's alpha the
    disagreement must be a floating-point tie of the Armijo test (both sides of
    the comparison within 1e-5 max(1,|F|)), and the oracle is then forced onto
    the GPU's alpha so that the iterates stay comparable."""
    T = w.max_newton if max_newton is None else max_newton
    X, st = orc.local_newton(prob, X0, T, w.max_cg, w.cg_tol, w.grad_tol, w.beta, w.gamma, w.max_ls)
    alphas = [it["alpha"] for it in st["iters"]]
    forced = False
    for _ in range(T):
        m = min(len(alphas), len(gpu_alphas))
        diff = [t for t in range(m) if not np.isclose(alphas[t], gpu_alphas[t], rtol=1e-6)]
        if not diff:
            break
        t = diff[0]
        it = st["iters"][t]
        big = max(alphas[t], float(gpu_alphas[t]))   # the test at the larger step is the one decided differently
        margin = armijo_margin(prob, it["X"], it["p"], it["g"], big, w.beta, it["loss"])
        assert abs(margin) <= 1e-5 * max(1.0, abs(it["loss"])), (
            f"line search disagrees at iteration {t}: oracle alpha {alphas[t]}, GPU alpha {gpu_alphas[t]}, "
            f"Armijo margin {margin:.3e} is not a tie")
        force = [float(a) for a in gpu_alphas[: t + 1]]
        X, st = orc.local_newton(prob, X0, T, w.max_cg, w.cg_tol, w.grad_tol, w.beta, w.gamma, w.max_ls,
                                 forced_alphas=force)
        # forced run: alphas beyond t come from the oracle's own line search again
        alphas = [it2["alpha"] for it2 in st["iters"]]
        forced = True
    return X, st, forced
