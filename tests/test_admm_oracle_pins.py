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


# ---- a two-worker scalar example worked by hand (tolerances and residual balancing, step by step) ----
#
# Two workers with one sample each, one feature, two classes (one weight, d = 1), loss scale s = 1:
#   worker 1: a = 1, label = the free class:        f_1(x) = log(1 + e^x) - x
#   worker 2: a = 2, label = the reference class:   f_2(x) = log(1 + e^{2x})
# Penalties rho_1 = 1/(4 ln 3), rho_2 = 1/ln 3, regulariser lam = 3/(4 ln 3), start x = y = z = 0.
# Iteration 0 has a closed form.  x-update (paper's sign): f_i'(x) + rho_i (x - z) - y_i = 0 with z = y = 0:
#   worker 1: sigma(x) - 1 + rho_1 x = 0 at x = ln 3:      3/4 - 1 + (1/(4 ln 3)) ln 3 = 0
#   worker 2: 2 sigma(2x) + rho_2 x = 0 at x = -(ln 3)/2:  2/4 - (1/ln 3)(ln 3)/2 = 0
#   z   = (rho_1 x_1 + rho_2 x_2) / (lam + rho_1 + rho_2) = (1/4 - 1/2) / (2/ln 3) = -(ln 3)/8
#   y_1 = rho_1 (z - x_1) = (1/(4 ln 3)) (-(9/8) ln 3) = -9/32,   y_2 = rho_2 (z - x_2) = (1/ln 3)(3/8) ln 3 = 12/32
#   ||r|| = ln 3 sqrt((9/8)^2 + (3/8)^2) = ln 3 sqrt(90)/8,   ||d|| = sqrt(rho_1^2 + rho_2^2) |z| = sqrt(17/16)/8
#   sqrt(sum x_i^2) = ln 3 sqrt(5/4),  sqrt(N) |z| = sqrt(2) ln 3 / 8,  sqrt(sum y_i^2) = 15/32
# so ||r|| / ||d|| = 10.1112: with mu = 10 the factor doubles, with mu = 11 it stays.
# The later x-updates are roots of a strictly increasing scalar function; the values written out below were found by a
# root finder in 30-digit arithmetic and are checked here by substitution into that function.
LN3 = 1.0986122886681098


def _scalar_shards():
    return [orc.Problem(np.array([[1.0]]), np.array([0]), 2, s=1.0), orc.Problem(np.array([[2.0]]), np.array([1]), 2, s=1.0)]


def _stationarity(i, x, z, y, rho):
    a, t = ((1.0, 1.0), (2.0, 0.0))[i]
    return a * (1.0 / (1.0 + np.exp(-a * x)) - t) + rho * (x - z) - y


# Newton iterations, CG iterations (d = 1: one is exact), tolerances, line search.  The local solves stop a few 1e-11 from
# their minimisers (where float64 no longer resolves a decrease of the objective), hence the 1e-9 below.
_LOCAL = (60, 3, 0.0, 1e-15, 1e-4, 0.5, 30)


def test_tolerances_on_hand_numbers():
    # N = 2, d = 4.  sum ||x_i||^2 = 25 + 144 = 13^2, ||z|| = 3, sum ||y_i||^2 = 36 + 64 = 10^2
    xs = [np.array([[3.0, 4.0], [0.0, 0.0]]), np.array([[0.0, 0.0], [12.0, 0.0]])]
    ys = [np.array([[0.0, 6.0], [0.0, 0.0]]), np.array([[0.0, 0.0], [0.0, 8.0]])]
    z = np.array([[1.0, 2.0], [2.0, 0.0]])
    e_pri, e_dual = adm.tolerances(xs, ys, z, 0.5, 0.1)
    assert abs(e_pri - (0.7071067811865476 + 1.3)) < 1e-14        # sqrt(2)/2 + 0.1 max{13, 3 sqrt(2)}
    assert abs(e_dual - 2.0) < 1e-14                               # sqrt(4)/2 + 0.1 * 10
    # ||z|| = 10: sqrt(N) ||z|| = 14.142... now exceeds 13
    e_pri, e_dual = adm.tolerances(xs, ys, np.array([[6.0, 8.0], [0.0, 0.0]]), 0.5, 0.1)
    assert abs(e_pri - (0.7071067811865476 + 1.4142135623730951)) < 1e-14
    assert abs(e_dual - 2.0) < 1e-14


def test_residual_balancing_on_the_scalar_example_growing_penalty():
    rhos, lam = [0.25 / LN3, 1.0 / LN3], 0.75 / LN3
    z, xs, ys, hist = adm.admm(_scalar_shards(), lam, rhos, np.zeros((1, 1)), 3, *_LOCAL, eps_abs=0.01, eps_rel=0.1,
                               penalty_rule=1, rb_mu=10.0, rb_tau=2.0)
    val = lambda a: float(np.asarray(a).ravel()[0])
    h = hist[0]                                                   # closed forms of the comment above
    assert h["rho_scale"] == 1.0
    assert abs(val(h["xs"][0]) - LN3) < 1e-12 and abs(val(h["xs"][1]) + LN3 / 2) < 1e-12
    assert abs(val(h["z"]) + LN3 / 8) < 1e-12
    assert abs(val(h["ys"][0]) + 9.0 / 32) < 1e-12 and abs(val(h["ys"][1]) - 12.0 / 32) < 1e-12
    assert abs(h["r_norm"] - 1.3027939116156068) < 1e-12          # ln 3 sqrt(90) / 8
    assert abs(h["d_norm"] - 0.12884705080055189) < 1e-12         # sqrt(17/16) / 8
    assert abs(h["eps_pri"] - (0.014142135623730951 + 0.12282858791892576)) < 1e-12   # sqrt(2)/100 + ln 3 sqrt(5/4) / 10
    assert abs(h["eps_dual"] - (0.01 + 0.046875)) < 1e-12                              # 1/100 + (15/32)/10
    # ||r|| = 10.11 ||d|| > 10 ||d||: iteration 1 runs with the doubled penalties
    h = hist[1]
    assert h["rho_scale"] == 2.0
    x1, x2 = 0.22191491756765847, -0.31374271578559926
    z0, y0 = -LN3 / 8, (-9.0 / 32, 12.0 / 32)
    assert abs(_stationarity(0, x1, z0, y0[0], 2 * rhos[0])) < 1e-14 and abs(_stationarity(1, x2, z0, y0[1], 2 * rhos[1])) < 1e-14
    assert abs(val(h["xs"][0]) - x1) < 1e-9 and abs(val(h["xs"][1]) - x2) < 1e-9
    # z = (2 rho_1 x_1 - y_1 + 2 rho_2 x_2 - y_2) / (lam + 2 rho_1 + 2 rho_2);  y_i += 2 rho_i (z - x_i)
    assert abs(val(h["z"]) + 0.19062242303077064) < 1e-9
    assert abs(val(h["ys"][0]) + 0.46900383493050316) < 1e-9 and abs(val(h["ys"][1]) - 0.59913784011845003) < 1e-9
    assert abs(h["r_norm"] - 0.43051790192285734) < 1e-9         # sqrt((z - x_1)^2 + (z - x_2)^2)
    assert abs(h["d_norm"] - 0.10001006431528394) < 1e-9         # 2 sqrt(rho_1^2 + rho_2^2) |z - z_prev|
    assert abs(h["eps_pri"] - (0.014142135623730951 + 0.038429249582522942)) < 1e-9   # sqrt(x_1^2 + x_2^2) = 0.38429 > sqrt(2)|z| = 0.26958
    assert abs(h["eps_dual"] - (0.01 + 0.076087498883937567)) < 1e-9
    # ||r|| = 4.30 ||d||: neither ||r|| > 10 ||d|| nor ||d|| > 10 ||r||, the factor stays
    assert hist[2]["rho_scale"] == 2.0
    # the same run with mu = 11 never changes the penalty (10.11 < 11)
    _, _, _, hist11 = adm.admm(_scalar_shards(), lam, rhos, np.zeros((1, 1)), 3, *_LOCAL, penalty_rule=1, rb_mu=11.0, rb_tau=2.0)
    assert [g["rho_scale"] for g in hist11] == [1.0, 1.0, 1.0]


def test_residual_balancing_on_the_scalar_example_shrinking_penalty():
    # the same two workers with penalties 32 times larger, mu = 2, tau = 4: the dual residual dominates twice
    rhos, lam = [8.0 / LN3, 32.0 / LN3], 0.75 / LN3
    z, xs, ys, hist = adm.admm(_scalar_shards(), lam, rhos, np.zeros((1, 1)), 3, *_LOCAL, eps_abs=0.0, eps_rel=0.3,
                               penalty_rule=1, rb_mu=2.0, rb_tau=4.0)
    val = lambda a: float(np.asarray(a).ravel()[0])
    h = hist[0]
    x1, x2 = 0.066384999172433431, -0.033192499586216715
    assert abs(_stationarity(0, x1, 0.0, 0.0, rhos[0])) < 1e-14 and abs(_stationarity(1, x2, 0.0, 0.0, rhos[1])) < 1e-14
    assert abs(val(h["xs"][0]) - x1) < 1e-9 and abs(val(h["xs"][1]) - x2) < 1e-9
    assert abs(val(h["z"]) + 0.013032637874342759) < 1e-9
    assert abs(h["r_norm"] - 0.081936445482674921) < 1e-9 and abs(h["d_norm"] - 0.39129322029692842) < 1e-9
    # ||d|| = 4.78 ||r|| > 2 ||r||: the factor drops to 1/4
    h = hist[1]
    assert h["rho_scale"] == 0.25
    x1, x2 = -0.049283544920872374, -0.061310677975905231
    z0, y0 = -0.013032637874342759, (-0.57831238820790744, 0.58720950187264448)
    assert abs(_stationarity(0, x1, z0, y0[0], rhos[0] / 4)) < 1e-13 and abs(_stationarity(1, x2, z0, y0[1], rhos[1] / 4)) < 1e-13
    assert abs(val(h["xs"][0]) - x1) < 1e-9 and abs(val(h["xs"][1]) - x2) < 1e-9
    assert abs(val(h["z"]) + 0.055704836470208713) < 1e-9
    assert abs(h["r_norm"] - 0.0085239922658674489) < 1e-9 and abs(h["d_norm"] - 0.32029858741410993) < 1e-9
    # here sqrt(N) |z| = 0.078779 exceeds sqrt(x_1^2 + x_2^2) = 0.078663: the maximum of the primal tolerance takes it
    assert abs(h["eps_pri"] - 0.3 * 0.07877853522594457) < 1e-9
    assert abs(h["eps_dual"] - 0.3 * 0.86169904277234104) < 1e-9
    # ||d|| = 0.320 > eps_dual = 0.259: no stop; ||d|| = 37.6 ||r||: down again
    assert hist[2]["rho_scale"] == 0.0625
    # with eps_rel = 0.5 the same iteration meets both tolerances (0.0085 <= 0.039, 0.320 <= 0.431) and is the last one
    _, _, _, short = adm.admm(_scalar_shards(), lam, rhos, np.zeros((1, 1)), 3, *_LOCAL, eps_abs=0.0, eps_rel=0.5,
                              penalty_rule=1, rb_mu=2.0, rb_tau=4.0)
    assert len(short) == 2
