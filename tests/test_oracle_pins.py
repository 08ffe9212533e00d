"""Pins for the CPU oracle (no GPU needed).

The paper prints no worked numeric example, so the oracle is pinned to what the
mathematics fixes: closed forms at w = 0, finite differences, an explicitly built
dense Hessian, a brute-force Newton minimiser written with numpy only, decoupled
special cases with scalar closed forms, ridge normal equations, CG facts on an
explicit SPD system, and layout (CSR vs dense) agreement.
"""
import numpy as np
import pytest

import oracle as orc
from oracle import LOSS_LR, LOSS_L2SVM, Oracle


# ----------------------------------------------------------------------------
# small random problems (dense arrays; CSR built from them when needed)
# ----------------------------------------------------------------------------
def _dense_problem(rng, n, d, density=1.0):
    X = rng.standard_normal((n, d))
    if density < 1.0:
        X *= rng.random((n, d)) < density
    y = np.where(rng.random(n) < 0.5, 1.0, -1.0)
    return X, y


def _to_csr(X):
    n, d = X.shape
    rowptr = np.zeros(n + 1, dtype=np.int64)
    cols, vals = [], []
    for i in range(n):
        nz = np.nonzero(X[i])[0]
        cols.append(nz.astype(np.int32))
        vals.append(X[i, nz])
        rowptr[i + 1] = rowptr[i] + len(nz)
    return rowptr, np.concatenate(cols) if cols else np.zeros(0, np.int32), \
        np.concatenate(vals) if vals else np.zeros(0)


def _f_numpy(X, y, w, loss, C):
    """Objective written with library routines only (logaddexp / maximum)."""
    t = y * (X @ w)
    if loss == LOSS_LR:
        return 0.5 * w @ w + C * np.sum(np.logaddexp(0.0, -t))
    return 0.5 * w @ w + C * np.sum(np.maximum(0.0, 1.0 - t) ** 2)


# ----------------------------------------------------------------------------
# closed forms at w = 0  (Table 1 evaluated at z = 0)
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("layout", ["dense", "csr"])
def test_closed_forms_at_zero(rng, layout):
    n, d, C = 300, 17, 0.7
    X, y = _dense_problem(rng, n, d, density=0.4 if layout == "csr" else 1.0)
    if layout == "csr":
        rp, col, val = _to_csr(X)
        o = Oracle(n=n, d=d, y=y, rowptr=rp, col=col, val=val)
    else:
        o = Oracle(n=n, d=d, y=y, X=X)
    w0 = np.zeros(d)
    v = rng.standard_normal(d)

    f, g, D = o.fun_grad(LOSS_LR, C, w0)
    assert f == pytest.approx(C * n * np.log(2.0), rel=1e-14)
    np.testing.assert_allclose(g, -(C / 2.0) * (X.T @ y), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(D, 0.25, rtol=0, atol=0)
    np.testing.assert_allclose(o.hv(C, D, v), v + (C / 4.0) * (X.T @ (X @ v)), rtol=1e-12, atol=1e-12)

    f, g, D = o.fun_grad(LOSS_L2SVM, C, w0)
    assert f == pytest.approx(C * n, rel=1e-15)
    np.testing.assert_allclose(g, -2.0 * C * (X.T @ y), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(D, 2.0, rtol=0, atol=0)
    np.testing.assert_allclose(o.hv(C, D, v), v + 2.0 * C * (X.T @ (X @ v)), rtol=1e-12, atol=1e-12)


# ----------------------------------------------------------------------------
# objective against the library-routine definition, including huge margins
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("loss", [LOSS_LR, LOSS_L2SVM])
def test_objective_matches_definition(rng, loss):
    n, d, C = 200, 9, 1.3
    X, y = _dense_problem(rng, n, d)
    o = Oracle(n=n, d=d, y=y, X=X)
    for scale in (0.0, 0.1, 1.0, 30.0):
        w = scale * rng.standard_normal(d)
        f, z, zhat, D = o.fun(loss, C, w)
        np.testing.assert_allclose(z, X @ w, rtol=1e-13, atol=1e-13)
        assert f == pytest.approx(_f_numpy(X, y, w, loss, C), rel=1e-13)


def test_lr_terms_extreme_margins():
    # one instance, one feature: z = w, so the margin is set directly
    for t in (-745.0, -700.0, -40.0, -1e-300, 0.0, 1e-300, 40.0, 700.0, 745.0):
        for yi in (1.0, -1.0):
            o = Oracle(n=1, d=1, y=[yi], X=[[1.0]])
            w = np.array([t * yi])
            f, z, zhat, D = o.fun(LOSS_LR, 1.0, w)
            assert np.isfinite([f, zhat[0], D[0]]).all()
            h = 0.5 * (1.0 + np.tanh(0.5 * t))  # h(t) via tanh: a different route to the sigmoid
            assert f - 0.5 * t * t == pytest.approx(np.logaddexp(0.0, -t), rel=1e-12, abs=1e-300) or t * t > 1e3
            assert zhat[0] == pytest.approx((h - 1.0) * yi, rel=1e-9, abs=1e-300) or abs(t) > 30
            assert 0.0 <= D[0] <= 0.25
            if abs(t) <= 30:
                assert D[0] == pytest.approx(h * (1.0 - h), rel=1e-9)
    # symmetric tails: D(t) = D(-t), zhat(-t)*y + zhat(t)*y = -1
    o = Oracle(n=2, d=1, y=[1.0, 1.0], X=[[1.0], [-1.0]])
    _, _, zhat, D = o.fun(LOSS_LR, 1.0, np.array([37.5]))
    assert D[0] == pytest.approx(D[1], rel=1e-14)
    assert zhat[0] + zhat[1] == pytest.approx(-1.0, rel=1e-15)


# ----------------------------------------------------------------------------
# gradient: central finite differences of f
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("loss", [LOSS_LR, LOSS_L2SVM])
def test_gradient_finite_difference(rng, loss):
    n, d, C = 150, 12, 0.9
    X, y = _dense_problem(rng, n, d)
    o = Oracle(n=n, d=d, y=y, X=X)
    w = 0.3 * rng.standard_normal(d)
    _, g, _ = o.fun_grad(loss, C, w)
    for _ in range(5):
        u = rng.standard_normal(d)
        u /= np.linalg.norm(u)
        h = 1e-5
        fp = _f_numpy(X, y, w + h * u, loss, C)
        fm = _f_numpy(X, y, w - h * u, loss, C)
        assert g @ u == pytest.approx((fp - fm) / (2 * h), rel=2e-7, abs=1e-7)


# ----------------------------------------------------------------------------
# Hessian-vector product: finite differences of the gradient, explicit dense H
# ----------------------------------------------------------------------------
def test_hv_lr_finite_difference(rng):
    n, d, C = 120, 10, 1.1
    X, y = _dense_problem(rng, n, d)
    o = Oracle(n=n, d=d, y=y, X=X)
    w = 0.4 * rng.standard_normal(d)
    _, _, D = o.fun_grad(LOSS_LR, C, w)
    v = rng.standard_normal(d)
    h = 1e-5
    gp = o.fun_grad(LOSS_LR, C, w + h * v)[1]
    gm = o.fun_grad(LOSS_LR, C, w - h * v)[1]
    np.testing.assert_allclose(o.hv(C, D, v), (gp - gm) / (2 * h), rtol=1e-6, atol=1e-6)


def test_hv_svm_finite_difference_away_from_kinks(rng):
    n, d, C = 120, 10, 0.6
    X, y = _dense_problem(rng, n, d)
    o = Oracle(n=n, d=d, y=y, X=X)
    w = 0.4 * rng.standard_normal(d)
    v = rng.standard_normal(d)
    h = 1e-6
    slack = np.abs(1.0 - y * (X @ w))
    assert slack.min() > h * np.abs(X @ v).max()  # no instance crosses the hinge
    _, _, D = o.fun_grad(LOSS_L2SVM, C, w)
    gp = o.fun_grad(LOSS_L2SVM, C, w + h * v)[1]
    gm = o.fun_grad(LOSS_L2SVM, C, w - h * v)[1]
    # the objective is piecewise quadratic, so the difference quotient is exact up to rounding
    np.testing.assert_allclose(o.hv(C, D, v), (gp - gm) / (2 * h), rtol=1e-8, atol=1e-8)


@pytest.mark.parametrize("loss", [LOSS_LR, LOSS_L2SVM])
def test_hv_against_explicit_hessian(rng, loss):
    n, d, C = 180, 14, 0.8
    X, y = _dense_problem(rng, n, d)
    o = Oracle(n=n, d=d, y=y, X=X)
    w = 0.5 * rng.standard_normal(d)
    _, _, D = o.fun_grad(loss, C, w)
    t = y * (X @ w)
    if loss == LOSS_LR:
        h = 1.0 / (1.0 + np.exp(-t))
        H = np.eye(d) + C * X.T @ (X * (h * (1 - h))[:, None])
    else:
        act = (1.0 - t) > 0
        assert 0 < act.sum() < n  # both active and inactive rows are present
        H = np.eye(d) + 2.0 * C * X[act].T @ X[act]
    u, v = rng.standard_normal(d), rng.standard_normal(d)
    Hu, Hv = o.hv(C, D, u), o.hv(C, D, v)
    np.testing.assert_allclose(Hv, H @ v, rtol=1e-12, atol=1e-12)
    assert u @ Hv == pytest.approx(v @ Hu, rel=1e-13)       # symmetry
    assert v @ Hv >= v @ v                                    # H >= I


def test_svm_tie_is_inactive():
    # y z = 1 exactly: strict inequality in the active-set definition -> inactive
    o = Oracle(n=3, d=1, y=[1.0, -1.0, 1.0], X=[[1.0], [-1.0], [0.5]])
    f, z, zhat, D = o.fun(LOSS_L2SVM, 1.0, np.array([1.0]))
    np.testing.assert_array_equal(D, [0.0, 0.0, 2.0])
    np.testing.assert_array_equal(zhat, [0.0, 0.0, 2.0 * (0.5 - 1.0)])
    assert f == pytest.approx(0.5 + 0.25)


# ----------------------------------------------------------------------------
# layouts agree
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("loss", [LOSS_LR, LOSS_L2SVM])
def test_csr_and_dense_agree(rng, loss):
    n, d, C = 250, 40, 1.0
    X, y = _dense_problem(rng, n, d, density=0.2)
    X[7] = 0.0  # an empty row
    X[:, 11] = 0.0  # an empty column
    rp, col, val = _to_csr(X)
    od = Oracle(n=n, d=d, y=y, X=X)
    os_ = Oracle(n=n, d=d, y=y, rowptr=rp, col=col, val=val)
    w = 0.5 * rng.standard_normal(d)
    v = rng.standard_normal(d)
    fd, gd, Dd = od.fun_grad(loss, C, w)
    fs, gs, Ds = os_.fun_grad(loss, C, w)
    assert fd == pytest.approx(fs, rel=1e-14)
    np.testing.assert_allclose(gd, gs, rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(Dd, Ds, rtol=1e-13, atol=0)
    np.testing.assert_allclose(od.hv(C, Dd, v), os_.hv(C, Ds, v), rtol=1e-13, atol=1e-14)
    rd = od.tron(loss, C, 1e-6)
    rs = os_.tron(loss, C, 1e-6)
    assert rd.outer_iters == rs.outer_iters and rd.cg_iters_total == rs.cg_iters_total
    assert rd.f == pytest.approx(rs.f, rel=1e-13)


# ----------------------------------------------------------------------------
# CG on an explicit SPD system
# ----------------------------------------------------------------------------
def _explicit_system(rng, n=60, d=8, C=0.9):
    X, y = _dense_problem(rng, n, d)
    o = Oracle(n=n, d=d, y=y, X=X)
    w = 0.3 * rng.standard_normal(d)
    _, g, D = o.fun_grad(LOSS_LR, C, w)
    H = np.eye(d) + C * X.T @ (X * D[:, None])
    return o, C, D, g, H


def test_cg_unconstrained_solves_newton_system(rng):
    o, C, D, g, H = _explicit_system(rng)
    d = len(g)
    s, r, nhv, onb = o.cg(C, D, g, delta=1e30, xi=1e-14, max_cg=d)
    assert not onb and nhv <= d
    np.testing.assert_allclose(s, np.linalg.solve(H, -g), rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(r, -g - H @ s, rtol=0, atol=1e-12)


def test_cg_residuals_are_orthogonal(rng):
    o, C, D, g, H = _explicit_system(rng)
    # residual after k products, for k = 1..4, by capping max_cg
    res = [o.cg(C, D, g, delta=1e30, xi=0.0, max_cg=k)[1] for k in range(1, 5)]
    res = [-g] + res
    for a in range(len(res)):
        for b in range(a):
            cosang = res[a] @ res[b] / (np.linalg.norm(res[a]) * np.linalg.norm(res[b]))
            assert abs(cosang) < 1e-10


def test_cg_boundary_step(rng):
    o, C, D, g, H = _explicit_system(rng)
    newton = np.linalg.solve(H, -g)
    delta = 0.3 * np.linalg.norm(newton)
    s, r, nhv, onb = o.cg(C, D, g, delta=delta, xi=1e-12, max_cg=50)
    assert onb
    assert np.linalg.norm(s) == pytest.approx(delta, rel=1e-14)
    np.testing.assert_allclose(r, -g - H @ s, rtol=0, atol=1e-12)
    q = lambda u: g @ u + 0.5 * u @ H @ u
    # Cauchy point: minimiser of q along -g inside the region
    tc = min((g @ g) / (g @ H @ g), delta / np.linalg.norm(g))
    assert q(s) <= q(-tc * g) + 1e-14
    # first step from s = 0 along -g: a tiny radius must give exactly -delta g/|g|
    s1, _, n1, onb1 = o.cg(C, D, g, delta=1e-3 * np.linalg.norm(g) / np.linalg.norm(H, 2), xi=1e-12, max_cg=50)
    assert onb1 and n1 == 1
    np.testing.assert_allclose(s1 / np.linalg.norm(s1), -g / np.linalg.norm(g), rtol=1e-12, atol=1e-14)


def test_cg_stops_on_relative_residual(rng):
    o, C, D, g, H = _explicit_system(rng)
    s, r, nhv, onb = o.cg(C, D, g, delta=1e30, xi=0.1, max_cg=100)
    assert np.linalg.norm(r) <= 0.1 * np.linalg.norm(g)
    if nhv > 1:  # one fewer product would not have met the test
        r_prev = o.cg(C, D, g, delta=1e30, xi=0.0, max_cg=nhv - 1)[1]
        assert np.linalg.norm(r_prev) > 0.1 * np.linalg.norm(g)


# ----------------------------------------------------------------------------
# full solves
# ----------------------------------------------------------------------------
def _newton_minimise(X, y, loss, C, tol=1e-12, iters=200):
    """Brute force: explicit Hessian, linear solve, backtracking; numpy only."""
    n, d = X.shape
    w = np.zeros(d)

    def grad_hess(w):
        t = y * (X @ w)
        if loss == LOSS_LR:
            h = 0.5 * (1.0 + np.tanh(0.5 * t))
            g = w + C * X.T @ ((h - 1.0) * y)
            H = np.eye(d) + C * X.T @ (X * (h * (1 - h))[:, None])
        else:
            act = (1.0 - t) > 0
            g = w + 2.0 * C * X[act].T @ (X[act] @ w - y[act])
            H = np.eye(d) + 2.0 * C * X[act].T @ X[act]
        return g, H

    for _ in range(iters):
        g, H = grad_hess(w)
        if np.linalg.norm(g) <= tol:
            break
        step = np.linalg.solve(H, -g)
        f0, a = _f_numpy(X, y, w, loss, C), 1.0
        while _f_numpy(X, y, w + a * step, loss, C) > f0 + 1e-4 * a * (g @ step) and a > 1e-12:
            a *= 0.5
        w = w + a * step
    return w, np.linalg.norm(grad_hess(w)[0])


@pytest.mark.parametrize("loss", [LOSS_LR, LOSS_L2SVM])
@pytest.mark.parametrize("shape", [(80, 6), (200, 20)])
def test_tron_matches_brute_force_newton(rng, loss, shape):
    n, d = shape
    C = 1.0
    X, y = _dense_problem(rng, n, d)
    w_star, gn = _newton_minimise(X, y, loss, C)
    assert gn <= 1e-10
    res = Oracle(n=n, d=d, y=y, X=X).tron(loss, C, eps=1e-10)
    assert res.converged
    assert np.linalg.norm(res.w - w_star) <= 1e-8 * np.linalg.norm(w_star)
    assert res.f == pytest.approx(_f_numpy(X, y, w_star, loss, C), rel=1e-12)


def test_tron_identity_features_closed_form(rng):
    # X = I: the problem decouples into n scalar problems
    n, C = 25, 0.8
    y = np.where(rng.random(n) < 0.5, 1.0, -1.0)
    o = Oracle(n=n, d=n, y=y, X=np.eye(n))
    res = o.tron(LOSS_L2SVM, C, eps=1e-12)
    np.testing.assert_allclose(res.w, 2 * C * y / (1 + 2 * C), rtol=1e-10)
    # LR: w_i = y_i a with a solving a = C (1 - h(a)); bisection on [0, C]
    lo, hi = 0.0, C
    for _ in range(200):
        a = 0.5 * (lo + hi)
        if a - C * (1.0 - 1.0 / (1.0 + np.exp(-a))) > 0:
            hi = a
        else:
            lo = a
    res = o.tron(LOSS_LR, C, eps=1e-12)
    np.testing.assert_allclose(res.w, y * a, rtol=1e-9)


def test_tron_all_active_svm_is_ridge(rng):
    # small C keeps |w| small, so every margin stays below 1: ridge normal equations
    n, d, C = 300, 10, 1e-3
    X, y = _dense_problem(rng, n, d)
    res = Oracle(n=n, d=d, y=y, X=X).tron(LOSS_L2SVM, C, eps=1e-12)
    assert np.all(y * (X @ res.w) < 1.0)
    w_ridge = np.linalg.solve(np.eye(d) + 2 * C * X.T @ X, 2 * C * X.T @ y)
    np.testing.assert_allclose(res.w, w_ridge, rtol=1e-9, atol=1e-12)


@pytest.mark.parametrize("loss", [LOSS_LR, LOSS_L2SVM])
def test_tron_invariants(rng, loss):
    n, d, C, eps = 400, 60, 2.0, 1e-2
    X, y = _dense_problem(rng, n, d, density=0.3)
    rp, col, val = _to_csr(X)
    o = Oracle(n=n, d=d, y=y, rowptr=rp, col=col, val=val)
    res = o.tron(loss, C, eps)
    assert res.converged and res.status == 0
    # stationarity, re-evaluated from scratch with numpy
    t = y * (X @ res.w)
    if loss == LOSS_LR:
        g = res.w + C * X.T @ ((0.5 * (1 + np.tanh(0.5 * t)) - 1.0) * y)
        g0 = -(C / 2) * X.T @ y
    else:
        act = (1 - t) > 0
        g = res.w + 2 * C * X[act].T @ (X[act] @ res.w - y[act])
        g0 = -2 * C * X.T @ y
    assert res.gnorm0 == pytest.approx(np.linalg.norm(g0), rel=1e-12)
    assert np.linalg.norm(g) <= eps * np.linalg.norm(g0)
    assert res.gnorm == pytest.approx(np.linalg.norm(g), rel=1e-9)
    assert res.f == pytest.approx(_f_numpy(X, y, res.w, loss, C), rel=1e-13)
    # accepted steps decrease f; rejected ones leave it alone; counts are consistent
    f_prev = _f_numpy(X, y, np.zeros(d), loss, C)
    for rec in res.trace:
        if rec["accepted"]:
            assert rec["f"] < f_prev
        else:
            assert rec["f"] == f_prev
        f_prev = rec["f"]
        assert rec["pred"] > 0 and rec["snorm"] > 0
    assert sum(r["cg_iters"] for r in res.trace) == res.cg_iters_total == res.n_hv
    assert res.n_fun == 1 + res.outer_iters
    assert res.n_grad == 1 + sum(r["accepted"] for r in res.trace)
    # strong convexity (modulus 1): f(w_eps) - f* <= |g|^2 / 2
    tight = o.tron(loss, C, 1e-9)
    assert 0.0 <= res.f - tight.f <= 0.5 * (eps * res.gnorm0) ** 2


def test_tron_warm_start_uses_gradient_at_zero(rng):
    n, d, C = 150, 8, 1.0
    X, y = _dense_problem(rng, n, d)
    o = Oracle(n=n, d=d, y=y, X=X)
    cold = o.tron(LOSS_LR, C, 1e-8)
    warm = o.tron(LOSS_LR, C, 1e-8, w0=cold.w)
    assert warm.gnorm0 == pytest.approx(cold.gnorm0, rel=1e-14)
    assert warm.outer_iters == 0 and warm.converged
    np.testing.assert_array_equal(warm.w, cold.w)


def test_tron_respects_iteration_cap(rng):
    n, d = 200, 15
    X, y = _dense_problem(rng, n, d)
    res = Oracle(n=n, d=d, y=y, X=X).tron(LOSS_LR, 10.0, 1e-12, max_outer=2)
    assert res.status == 1 and not res.converged and res.outer_iters == 2


# ----------------------------------------------------------------------------
# diagonal preconditioner (the paper only names it; pins = what the mathematics fixes)
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("loss", [LOSS_LR, LOSS_L2SVM])
@pytest.mark.parametrize("layout", ["dense", "csr"])
def test_hess_diag_is_the_diagonal_of_the_explicit_hessian(rng, loss, layout):
    n, d, C = 70, 9, 0.7
    X, y = _dense_problem(rng, n, d, density=0.6)
    if layout == "dense":
        o = Oracle(n=n, d=d, y=y, X=X)
    else:
        rowptr, col, val = _to_csr(X)
        o = Oracle(n=n, d=d, y=y, rowptr=rowptr, col=col, val=val)
    _, _, D = o.fun_grad(loss, C, 0.4 * rng.standard_normal(d))
    H = np.eye(d) + C * X.T @ (X * D[:, None])
    np.testing.assert_allclose(o.hess_diag(C, D), np.diag(H), rtol=1e-13)
    # and of the operator itself: e_j . H e_j
    for j in (0, d // 2, d - 1):
        e = np.zeros(d); e[j] = 1.0
        assert o.hess_diag(C, D)[j] == pytest.approx(o.hv(C, D, e)[j], rel=1e-13)


def test_pcg_with_identity_preconditioner_is_cg(rng):
    o, C, D, g, H = _explicit_system(rng)
    ones = np.ones(len(g))
    for delta, xi, cap in ((1e30, 1e-14, 8), (0.3 * np.linalg.norm(np.linalg.solve(H, -g)), 1e-12, 50), (1e30, 0.1, 100)):
        a = o.cg(C, D, g, delta=delta, xi=xi, max_cg=cap)
        b = o.pcg(C, D, g, ones, delta=delta, xi=xi, max_cg=cap)
        np.testing.assert_array_equal(a[0], b[0])
        np.testing.assert_array_equal(a[1], b[1])
        assert a[2:] == b[2:]


def test_pcg_unconstrained_solves_newton_system(rng):
    o, C, D, g, H = _explicit_system(rng)
    d = len(g)
    M = 0.99 + 0.01 * np.diag(H)
    s, r, nhv, onb = o.pcg(C, D, g, M, delta=1e30, xi=1e-14, max_cg=d)
    assert not onb and nhv <= d
    np.testing.assert_allclose(s, np.linalg.solve(H, -g), rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(r, -g - H @ s, rtol=0, atol=1e-12)
    # exact diagonal scaling of a diagonal system: one product solves it (a diagonal X makes H diagonal)
    n = 12
    y = np.where(rng.random(n) < 0.5, 1.0, -1.0)
    oi = Oracle(n=n, d=n, y=y, X=np.diag(rng.uniform(0.5, 3.0, n)))
    _, gi, Di = oi.fun_grad(LOSS_LR, 2.0, rng.standard_normal(n))
    hd = oi.hess_diag(2.0, Di)
    s1, _, n1, _ = oi.pcg(2.0, Di, gi, hd, delta=1e30, xi=1e-13, max_cg=n)
    assert n1 == 1
    np.testing.assert_allclose(s1, -gi / hd, rtol=1e-13)


def test_pcg_residuals_are_conjugate_in_the_inverse_preconditioner(rng):
    o, C, D, g, H = _explicit_system(rng)
    M = rng.uniform(0.5, 4.0, len(g))
    res = [-g] + [o.pcg(C, D, g, M, delta=1e30, xi=0.0, max_cg=k)[1] for k in range(1, 5)]
    for a in range(len(res)):
        for b in range(a):
            cosang = (res[a] / M) @ res[b] / np.sqrt(((res[a] / M) @ res[a]) * ((res[b] / M) @ res[b]))
            assert abs(cosang) < 1e-10


def test_pcg_equals_cg_on_the_scaled_variables(rng):
    # PCG with M on (H, g) is CG on (M^-1/2 H M^-1/2, M^-1/2 g) in the variables M^1/2 s; the scaled system is
    # solved here with a few lines of textbook CG in numpy
    o, C, D, g, H = _explicit_system(rng)
    M = rng.uniform(0.5, 4.0, len(g))
    Hs = H / np.sqrt(M)[:, None] / np.sqrt(M)[None, :]
    gs = g / np.sqrt(M)
    for k in (1, 2, 3, 5):
        u = np.zeros_like(gs); r = -gs.copy(); p = r.copy()
        for _ in range(k):
            Hp = Hs @ p
            al = (r @ r) / (p @ Hp)
            u = u + al * p
            rn = r - al * Hp
            p = rn + (rn @ rn) / (r @ r) * p
            r = rn
        s, rr, nhv, onb = o.pcg(C, D, g, M, delta=1e30, xi=0.0, max_cg=k)
        assert nhv == k and not onb
        np.testing.assert_allclose(s, u / np.sqrt(M), rtol=1e-10, atol=1e-13)
        np.testing.assert_allclose(rr, r * np.sqrt(M), rtol=1e-9, atol=1e-12)


def test_pcg_boundary_step_is_measured_in_the_m_norm(rng):
    o, C, D, g, H = _explicit_system(rng)
    M = rng.uniform(0.5, 4.0, len(g))
    mnorm = lambda u: np.sqrt(u @ (M * u))
    newton = np.linalg.solve(H, -g)
    delta = 0.3 * mnorm(newton)
    s, r, nhv, onb = o.pcg(C, D, g, M, delta=delta, xi=1e-12, max_cg=50)
    assert onb
    assert mnorm(s) == pytest.approx(delta, rel=1e-14)
    np.testing.assert_allclose(r, -g - H @ s, rtol=0, atol=1e-12)
    # a tiny radius: one product, the step is -delta M^-1 g / |M^-1 g|_M
    tiny = 1e-3 * delta / np.linalg.norm(H, 2)
    s1, _, n1, onb1 = o.pcg(C, D, g, M, delta=tiny, xi=1e-12, max_cg=50)
    assert onb1 and n1 == 1
    np.testing.assert_allclose(s1, -tiny * (g / M) / mnorm(g / M), rtol=1e-12, atol=1e-16)
    # the model value is no worse than at the scaled Cauchy point
    q = lambda u: g @ u + 0.5 * u @ H @ u
    dirn = -g / M
    tc = min(-(g @ dirn) / (dirn @ H @ dirn), delta / mnorm(dirn))
    assert q(s) <= q(tc * dirn) + 1e-14


@pytest.mark.parametrize("loss", [LOSS_LR, LOSS_L2SVM])
def test_preconditioned_tron_reaches_the_same_minimiser(rng, loss):
    n, d, C = 200, 20, 1.0
    X, y = _dense_problem(rng, n, d)
    X[:, :3] *= 30.0          # badly scaled features: what the diagonal is for
    w_star, gn = _newton_minimise(X, y, loss, C)
    assert gn <= 1e-9
    o = Oracle(n=n, d=d, y=y, X=X)
    res = o.tron(loss, C, eps=1e-10, precond_blend=0.01)
    assert res.converged
    assert np.linalg.norm(res.w - w_star) <= 1e-7 * np.linalg.norm(w_star)
    assert res.f == pytest.approx(_f_numpy(X, y, w_star, loss, C), rel=1e-12)
    fs = [t["f"] for t in res.trace if t["accepted"]]
    assert all(b <= a for a, b in zip(fs, fs[1:]))
    assert res.n_hv == sum(t["cg_iters"] for t in res.trace)
    # blend = 1 (pure diagonal) also converges there
    res1 = o.tron(loss, C, eps=1e-10, precond_blend=1.0)
    assert res1.converged and np.linalg.norm(res1.w - w_star) <= 1e-7 * np.linalg.norm(w_star)


def test_preconditioned_tron_on_identity_features(rng):
    # X = I: H is diagonal, so with blend = 1 every inner solve is exact after one product
    n, C = 25, 0.8
    y = np.where(rng.random(n) < 0.5, 1.0, -1.0)
    o = Oracle(n=n, d=n, y=y, X=np.eye(n))
    res = o.tron(LOSS_L2SVM, C, eps=1e-12, precond_blend=1.0)
    np.testing.assert_allclose(res.w, 2 * C * y / (1 + 2 * C), rtol=1e-10)
    assert all(t["cg_iters"] <= 1 for t in res.trace)


# ----------------------------------------------------------------------------
# how much of a trajectory does the arithmetic fix?  (oracle vs its plain-fp64 twin)
# ----------------------------------------------------------------------------
def test_rounding_alone_moves_the_eps_0p01_iterate_on_zipf_data():
    """The same source compiled with fp64 instead of long-double accumulators is a second, equally valid
    implementation.  On the url-shaped workload (well separated top Hessian eigenvalue from the Zipf head
    feature) the two agree call by call and for the first outer iterations, then CG amplifies the 1e-16
    differences: the eps = 0.01 iterates differ by ~1e-5 in f.  Both are eps-solutions; with a tight eps both
    reach the same minimiser.  This is why solve-level parity on that workload is stated at eps = 1e-6."""
    import datagen as dg
    p = dg.config3(0.05)
    a = Oracle.from_problem(p)
    b = Oracle.from_problem(p, plain_fp64=True)
    w = 0.5 * np.random.default_rng(3).standard_normal(p.d)
    fa, ga, Da = a.fun_grad(LOSS_LR, 1.0, w)
    fb, gb, Db = b.fun_grad(LOSS_LR, 1.0, w)
    assert abs(fa - fb) <= 1e-12 * abs(fa)
    assert np.linalg.norm(ga - gb) <= 1e-12 * np.linalg.norm(ga)
    ra, rb = a.tron(LOSS_LR, 1.0, 1e-2), b.tron(LOSS_LR, 1.0, 1e-2)
    assert ra.converged and rb.converged and ra.outer_iters == rb.outer_iters
    early = [abs(x["f"] - y["f"]) / abs(x["f"]) for x, y in zip(ra.trace[:3], rb.trace[:3])]
    assert max(early) <= 1e-9
    # both satisfy the stopping rule; their objectives are within the strong-convexity bound of each other
    assert abs(ra.f - rb.f) <= 0.5 * (1e-2 * ra.gnorm0) ** 2
    ta, tb = a.tron(LOSS_LR, 1.0, 1e-6), b.tron(LOSS_LR, 1.0, 1e-6)
    assert abs(ta.f - tb.f) <= 1e-8 * abs(ta.f)


# ----------------------------------------------------------------------------
# Problems over a subset of the instances (the training folds of cross-validation, Section 2.1): the oracle of a
# fold is the oracle over the rows of the fold.  Pinned through the full-data oracle with masked per-instance terms.
# ----------------------------------------------------------------------------
def _folds(rng, n, k=3):
    return rng.integers(0, k, size=n)


@pytest.mark.parametrize("loss", [LOSS_LR, LOSS_L2SVM])
@pytest.mark.parametrize("layout", ["dense", "csr"])
def test_fold_objective_and_gradient_are_masked_sums(rng, loss, layout):
    X, y = _dense_problem(rng, 90, 7, density=0.6 if layout == "csr" else 1.0)
    if layout == "csr":
        rowptr, col, val = _to_csr(X)
        full = Oracle(n=90, d=7, y=y, rowptr=rowptr, col=col, val=val)
    else:
        full = Oracle(n=90, d=7, y=y, X=X)
    fold = _folds(rng, 90)
    w = 0.4 * rng.standard_normal(7)
    C = 0.7
    f_full, z, zhat, D = full.fun(loss, C, w)
    t = y * z
    per_row = np.logaddexp(0.0, -t) if loss == LOSS_LR else np.maximum(0.0, 1.0 - t) ** 2
    total = 0.0
    for k in range(3):
        rows = np.nonzero(fold != k)[0]          # train on the other two folds
        sub = full.restrict(rows)
        f_k, z_k, zhat_k, D_k = sub.fun(loss, C, w)
        assert np.array_equal(z_k, z[rows]) and np.array_equal(zhat_k, zhat[rows]) and np.array_equal(D_k, D[rows])
        assert abs(f_k - (0.5 * w @ w + C * per_row[rows].sum())) <= 1e-13 * abs(f_k)
        g_k = sub.grad(C, w, zhat_k)
        masked = np.where(fold != k, zhat, 0.0)
        np.testing.assert_allclose(g_k, full.grad(C, w, masked), rtol=0, atol=1e-13 * np.abs(g_k).max())
        np.testing.assert_allclose(g_k, w + C * X[rows].T @ zhat[rows], rtol=0, atol=1e-12 * np.abs(g_k).max())
        total += (f_k - 0.5 * w @ w) / C
    # every instance is left out exactly once: the three training sums count each loss twice
    assert abs(total - 2.0 * (f_full - 0.5 * w @ w) / C) <= 1e-12 * abs(total)


@pytest.mark.parametrize("loss", [LOSS_LR, LOSS_L2SVM])
def test_fold_hessian_product_is_the_full_product_with_masked_D(rng, loss):
    X, y = _dense_problem(rng, 120, 9)
    full = Oracle(n=120, d=9, y=y, X=X)
    fold = _folds(rng, 120)
    w = 0.3 * rng.standard_normal(9)
    v = rng.standard_normal(9)
    C = 1.3
    _, _, _, D = full.fun(loss, C, w)
    for k in range(3):
        rows = np.nonzero(fold != k)[0]
        sub = full.restrict(rows)
        _, _, _, D_k = sub.fun(loss, C, w)
        Hv_k = sub.hv(C, D_k, v)
        Hv_masked = full.hv(C, np.where(fold != k, D, 0.0), v)
        np.testing.assert_allclose(Hv_k, Hv_masked, rtol=0, atol=1e-13 * np.abs(Hv_k).max())
        H = np.eye(9) + C * X[rows].T @ (D[rows, None] * X[rows])
        np.testing.assert_allclose(Hv_k, H @ v, rtol=0, atol=1e-12 * np.abs(Hv_k).max())


@pytest.mark.parametrize("loss", [LOSS_LR, LOSS_L2SVM])
def test_fold_solutions_are_stationary_for_the_masked_full_problem(rng, loss):
    X, y = _dense_problem(rng, 150, 6)
    full = Oracle(n=150, d=6, y=y, X=X)
    fold = _folds(rng, 150)
    for k, C in zip(range(3), (0.05, 0.5, 2.0)):
        rows = np.nonzero(fold != k)[0]
        res = full.restrict(rows).tron(loss, C, 1e-9)
        assert res.converged
        _, _, zhat, _ = full.fun(loss, C, res.w)
        g = full.grad(C, res.w, np.where(fold != k, zhat, 0.0))
        assert np.linalg.norm(g) <= 1e-9 * res.gnorm0 * (1 + 1e-6)
        w_ref, _ = _newton_minimise(X[rows], y[rows], loss, C)
        np.testing.assert_allclose(res.w, w_ref, rtol=0, atol=1e-7 * max(1.0, np.abs(w_ref).max()))


# ----------------------------------------------------------------------------
# memory safety: every routine once under the address and undefined-behaviour sanitizers
# ----------------------------------------------------------------------------
def test_oracle_runs_clean_under_sanitizers(tmp_path):
    import os
    import subprocess
    here = os.path.dirname(os.path.abspath(orc.__file__))
    exe = str(tmp_path / "oracle_sanitize")
    subprocess.check_call(["gcc", "-g", "-O1", "-ffp-contract=off", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=all", "-static-libasan", "-o", exe,
                           os.path.join(here, "sanitize_main.c"), "-lm"])
    run = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "oracle sanitize run ok" in run.stdout
