"""Pins of the float64 ADMM oracle (Algorithm 1, fixed penalties and residual balancing) against what the mathematics fixes:
the z-update against a direct numerical minimisation of its defining problem, the multiplier invariant
that follows from the z- and y-updates, convergence to the minimiser of the centralised problem found by
an independent optimiser, and the one-worker case against the proximal-point iteration it reduces to."""
import numpy as np
import scipy.optimize

from oracle import admm_oracle as adm
from oracle import nadmm_oracle as orc


def make_shards(N=3, n_each=60, p=4, C=3, seed=0, s=None):
    rng = np.random.default_rng(seed)
    n = N * n_each
    A = rng.standard_normal((n, p))
    Wtrue = rng.standard_normal((p, C))
    b = np.argmax(A @ Wtrue + 0.5 * rng.standard_normal((n, C)), axis=1)
    s = 1.0 / n if s is None else s
    shards = [orc.Problem(A[i * n_each:(i + 1) * n_each], b[i * n_each:(i + 1) * n_each], C, s=s) for i in range(N)]
    return shards, orc.Problem(A, b, C, s=s), rng


def test_admm_z_update_minimises_its_defining_problem():
    rng = np.random.default_rng(1)
    shape, N, lam = (5, 2), 4, 0.37
    xs = [rng.standard_normal(shape) for _ in range(N)]
    ys = [rng.standard_normal(shape) for _ in range(N)]
    rhos = [0.5, 1.0, 2.0, 0.25]

    # g(z) + sum_i rho_i/2 ||z - x_i + y_i/rho_i||^2 (the z-update of Section 2.3) is a linear least-squares
    # problem: rows sqrt(lam) z = 0 and sqrt(rho_i) z = sqrt(rho_i) (x_i - y_i/rho_i); solved by the library
    d = int(np.prod(shape))
    rows = [np.sqrt(lam) * np.eye(d)] + [np.sqrt(r) * np.eye(d) for r in rhos]
    rhs = [np.zeros(d)] + [np.sqrt(r) * (x - y / r).ravel() for x, y, r in zip(xs, ys, rhos)]
    ref = np.linalg.lstsq(np.vstack(rows), np.concatenate(rhs), rcond=None)[0]
    np.testing.assert_allclose(adm.z_update(xs, ys, rhos, lam).ravel(), ref, rtol=0, atol=1e-13)


def test_admm_multipliers_sum_to_minus_lambda_z():
    # z-update optimality: lam z + sum_i rho_i (z - x_i) + sum_i y_i = 0; with the y-update this gives
    # sum_i y_i^{k+1} = -lam z^{k+1} after every iteration, whatever the local solves returned
    shards, _, _ = make_shards(N=4, seed=2)
    lam, rhos = 0.05, [0.3, 0.6, 0.9, 1.2]
    X0 = np.zeros((4, 2))
    z, xs, ys, hist = adm.admm(shards, lam, rhos, X0, 6, 1, 3, 0.0, 0.0, 1e-4, 0.5, 10)
    for h in hist:
        np.testing.assert_allclose(sum(h["ys"]), -lam * h["z"], rtol=0, atol=1e-13)


def test_admm_converges_to_the_centralised_minimiser():
    shards, full, _ = make_shards(N=3, seed=3)
    lam, rho = 0.02, 0.5
    X0 = np.zeros((4, 2))
    z, xs, ys, hist = adm.admm(shards, lam, [rho] * 3, X0, 1500, 20, 50, 1e-12, 1e-12, 1e-4, 0.5, 20)

    central = orc.Problem(full.A, full.b, full.C, s=full.s, lam=0.0, rho=lam)  # lam/2 ||x||^2 written as the prox term

    def fg(xf):
        f, g = orc.loss_grad(central, xf.reshape(X0.shape))
        return f, g.ravel()

    res = scipy.optimize.minimize(fg, np.zeros(X0.size), jac=True, method="L-BFGS-B", options=dict(ftol=1e-15, gtol=1e-11, maxiter=5000))
    np.testing.assert_allclose(z.ravel(), res.x, rtol=0, atol=1e-8)
    for x in xs:
        np.testing.assert_allclose(x, z, rtol=0, atol=1e-10)
    assert hist[-1]["r_norm"] < 1e-10 and hist[-1]["d_norm"] < 1e-10
    # residual norms decrease overall
    assert hist[-1]["r_norm"] < 1e-3 * hist[0]["r_norm"]


def test_admm_stops_on_the_residual_tolerances():
    shards, _, _ = make_shards(N=3, seed=4)
    z, xs, ys, hist = adm.admm(shards, 0.02, [0.5] * 3, np.zeros((4, 2)), 500, 5, 20, 1e-10, 1e-10, 1e-4, 0.5, 20,
                               eps_abs=1e-6, eps_rel=1e-4)
    assert 1 < len(hist) < 500
    last = hist[-1]
    assert last["r_norm"] <= last["eps_pri"] and last["d_norm"] <= last["eps_dual"]
    assert any(h["r_norm"] > h["eps_pri"] or h["d_norm"] > h["eps_dual"] for h in hist[:-1])
    for k in range(1, len(hist)):   # residuals as defined in Section 2.3.1: r_i = z - x_i, d_i = -rho_i (z - z_prev)
        h = hist[k]
        assert np.isclose(h["r_norm"], np.sqrt(sum(np.sum((h["z"] - x) ** 2) for x in h["xs"])))
        assert np.isclose(h["d_norm"], np.sqrt(3 * 0.5 ** 2) * np.linalg.norm(h["z"] - hist[k - 1]["z"]))
    N, d = 3, 8
    sx = np.sqrt(sum(np.sum(x * x) for x in last["xs"]))
    sy = np.sqrt(sum(np.sum(y * y) for y in last["ys"]))
    assert np.isclose(last["eps_pri"], np.sqrt(N) * 1e-6 + 1e-4 * max(sx, np.sqrt(N) * np.linalg.norm(last["z"])))
    assert np.isclose(last["eps_dual"], np.sqrt(d) * 1e-6 + 1e-4 * sy)


def test_admm_one_worker_without_regulariser_is_the_method_of_multipliers():
    # N = 1, lam = 0: z = x - y/rho, hence y <- y + rho (z - x) = 0 ... the iteration reduces to the
    # proximal-point method x <- argmin f(x) + rho/2 ||x - x_prev||^2, written out here independently
    shards, _, _ = make_shards(N=1, n_each=90, seed=5)
    rho = 0.8
    X0 = np.zeros((4, 2))
    z, xs, ys, hist = adm.admm(shards, 0.0, [rho], X0, 5, 30, 60, 1e-13, 1e-13, 1e-4, 0.5, 20)
    x = X0.copy()
    base = shards[0]
    for k in range(5):
        prob = orc.Problem(base.A, base.b, base.C, s=base.s, lam=0.0, rho=rho, z=x if k else np.zeros_like(X0))

        def fg(xf):
            f, g = orc.loss_grad(prob, xf.reshape(X0.shape))
            return f, g.ravel()

        x = scipy.optimize.minimize(fg, x.ravel(), jac=True, method="L-BFGS-B",
                                    options=dict(ftol=1e-16, gtol=1e-12, maxiter=5000)).x.reshape(X0.shape)
        np.testing.assert_allclose(hist[k]["xs"][0], x, rtol=0, atol=5e-7)
        np.testing.assert_allclose(hist[k]["z"], x, rtol=0, atol=5e-7)       # z = x when y = 0 and lam = 0
        np.testing.assert_allclose(hist[k]["ys"][0], 0.0, rtol=0, atol=1e-12)


def _central_minimiser(full, lam, shape):
    central = orc.Problem(full.A, full.b, full.C, s=full.s, lam=0.0, rho=lam)

    def fg(xf):
        f, g = orc.loss_grad(central, xf.reshape(shape))
        return f, g.ravel()

    res = scipy.optimize.minimize(fg, np.zeros(int(np.prod(shape))), jac=True, method="L-BFGS-B",
                                  options=dict(maxiter=5000, ftol=1e-15, gtol=1e-12))
    return res.x.reshape(shape)


def test_residual_balancing_that_never_triggers_is_the_fixed_penalty_iteration():
    shards, _, _ = make_shards(N=3, seed=5)
    lam, rhos = 0.05, [0.3, 0.6, 0.9]
    X0 = np.zeros((4, 2))
    args = (shards, lam, rhos, X0, 8, 2, 5, 0.0, 0.0, 1e-4, 0.5, 10)
    z0, xs0, ys0, h0 = adm.admm(*args)
    z1, xs1, ys1, h1 = adm.admm(*args, penalty_rule=1, rb_mu=1e30, rb_tau=2.0)
    assert np.array_equal(z0, z1) and all(np.array_equal(a, b) for a, b in zip(ys0, ys1))
    assert [h["rho_scale"] for h in h1] == [1.0] * 8


def test_residual_balancing_keeps_the_invariant_and_the_limit_and_repairs_a_bad_penalty():
    shards, full, _ = make_shards(N=3, seed=3)
    lam = 0.02
    X0 = np.zeros((4, 2))
    ref = _central_minimiser(full, lam, X0.shape)
    local = (5, 30, 1e-10, 1e-12, 1e-4, 0.5, 20)
    for rho, up in ((1e-3, True), (50.0, False)):
        z, xs, ys, hist = adm.admm(shards, lam, [rho, 2 * rho, rho], X0, 250, *local, eps_abs=1e-6, eps_rel=1e-5,
                                   penalty_rule=1, rb_mu=10.0, rb_tau=2.0)
        scales = [h["rho_scale"] for h in hist]
        assert len(hist) < 250                                   # stopped by the residual test
        assert np.linalg.norm(z - ref) <= 1e-3 * np.linalg.norm(ref)
        assert scales[0] == 1.0 and (scales[-1] >= 16.0 if up else scales[-1] <= 1.0 / 16.0)
        for h in hist:                                           # the z- and y-updates stay consistent under changing penalties
            np.testing.assert_allclose(sum(h["ys"]), -lam * h["z"], rtol=0, atol=1e-12)
        # the residuals end within the balance that the rule aims at, which the fixed penalty is far from
        ratio = hist[-1]["r_norm"] / hist[-1]["d_norm"]
        assert 1.0 / 20.0 <= ratio <= 20.0
        zf, _, _, hf = adm.admm(shards, lam, [rho, 2 * rho, rho], X0, 250, *local, eps_abs=1e-6, eps_rel=1e-5)
        assert len(hf) == 250                                    # the fixed penalty has not met the same tolerances
        rf = hf[-1]["r_norm"] / max(hf[-1]["d_norm"], 1e-300)
        assert rf > 1e3 if up else rf < 1e-2
