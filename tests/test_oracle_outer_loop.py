"""Pins for the oracle's outer loop (Algorithm 1) on trajectories that reject steps, shrink the radius and end
the inner solver on the trust-region boundary (no GPU needed).

The oracle's solve is replayed iteration by iteration with numpy: the iterate after k iterations comes from a solve
capped at k iterations, the Hessian at that iterate is built explicitly as a dense matrix (Appendix B:
H = I + C X^T D X), and a textbook truncated conjugate-gradient iteration on that matrix gives the step, the model
reduction and the number of products the oracle must report for iteration k + 1.  A Hessian taken at a rejected trial
point, a wrong sign in the model reduction, a wrong radius factor or accept threshold each break the agreement.
The last part plants such mistakes in copies of the oracle's source and checks that the pins notice every one.
"""
import os
import re

import numpy as np
import pytest

import oracle as orc
from oracle import LOSS_LR, LOSS_L2SVM, Oracle


def _far_start_problem():
    # saturated sigmoids far from the optimum: the quadratic model is poor there, so steps get rejected
    rng = np.random.default_rng(5)
    n, d = 2000, 40
    X = 3.0 * rng.standard_normal((n, d)) * (rng.random((n, d)) < 0.3)
    y = np.where(rng.random(n) < 0.5, 1.0, -1.0)
    w0 = 3.0 * rng.standard_normal(d)
    return X, y, w0


def _separable_problem():
    # L2-SVM far out along a separating direction: almost no instance is active there, the model sees H ~ I and steps
    # towards the origin, where every instance is active and the loss is large: rejected, radius halved
    rng = np.random.default_rng(7)
    n, d = 1500, 30
    X = rng.standard_normal((n, d))
    wt = rng.standard_normal(d)
    wt /= np.linalg.norm(wt)
    y = np.where(X @ wt >= 0, 1.0, -1.0)
    return X, y, 20.0 * wt


def _f(X, y, w, loss, C):
    t = y * (X @ w)
    if loss == LOSS_LR:
        return 0.5 * w @ w + C * np.sum(np.logaddexp(0.0, -t))
    return 0.5 * w @ w + C * np.sum(np.maximum(0.0, 1.0 - t) ** 2)


def _grad_hess(X, y, w, loss, C):
    """Gradient and explicit Hessian from the matrix forms of Table 1 / Appendix B."""
    t = y * (X @ w)
    d = X.shape[1]
    if loss == LOSS_LR:
        h = 0.5 * (1.0 + np.tanh(0.5 * t))
        return w + C * X.T @ ((h - 1.0) * y), np.eye(d) + C * X.T @ (X * (h * (1.0 - h))[:, None])
    act = (1.0 - t) > 0
    return w + 2.0 * C * X[act].T @ (X[act] @ w - y[act]), np.eye(d) + 2.0 * C * X[act].T @ X[act]


def _newton(X, y, loss, C, w):
    for _ in range(200):
        g, H = _grad_hess(X, y, w, loss, C)
        if np.linalg.norm(g) <= 1e-11:
            break
        step = np.linalg.solve(H, -g)
        f0, a = _f(X, y, w, loss, C), 1.0
        while _f(X, y, w + a * step, loss, C) > f0 + 1e-4 * a * (g @ step) and a > 1e-12:
            a *= 0.5
        w = w + a * step
    return w


def _truncated_cg(H, g, delta, xi, max_cg):
    """Steihaug-Toint on the explicit matrix: returns s, -q(s), products used, ended on the boundary."""
    s, r = np.zeros_like(g), -g.copy()
    p = r.copy()
    it, onb = 0, False
    while it < max_cg and np.linalg.norm(r) > xi * np.linalg.norm(g):
        Hp = H @ p
        it += 1
        alpha = (r @ r) / (p @ Hp)
        if np.linalg.norm(s + alpha * p) >= delta:
            # the non-negative root of |s + tau p| = delta
            roots = np.roots([p @ p, 2.0 * (s @ p), s @ s - delta * delta])
            tau = max(roots.real)
            s = s + tau * p
            onb = True
            break
        s = s + alpha * p
        r_new = r - alpha * Hp
        p = r_new + ((r_new @ r_new) / (r @ r)) * p
        r = r_new
    return s, -(g @ s + 0.5 * s @ (H @ s)), it, onb


def check_outer_loop(make_oracle, loss=LOSS_LR, C=50.0, eps=1e-4, min_rejected=5, min_boundary=5, problem=_far_start_problem):
    """All pins of one far-start solve; raises AssertionError on the first that fails."""
    X, y, w0 = problem()
    o = make_oracle(X, y)
    xi, max_cg = 0.1, 1000
    full = o.tron(loss, C, eps, w0=w0)
    tr = full.trace
    assert full.converged and full.status == 0
    assert sum(1 - t["accepted"] for t in tr) >= min_rejected
    assert sum(t["on_boundary"] for t in tr) >= min_boundary
    # the minimiser does not depend on the trust-region rules
    w_star = _newton(X, y, loss, C, np.zeros(X.shape[1]))
    tight = o.tron(loss, C, 1e-10, w0=w0)
    assert tight.converged
    assert np.linalg.norm(tight.w - w_star) <= 1e-8 * np.linalg.norm(w_star)
    assert tight.f == pytest.approx(_f(X, y, w_star, loss, C), rel=1e-12)

    g0 = np.linalg.norm(_grad_hess(X, y, np.zeros(X.shape[1]), loss, C)[0])
    assert full.gnorm0 == pytest.approx(g0, rel=1e-12)
    w = w0.copy()
    f = _f(X, y, w, loss, C)
    g, H = _grad_hess(X, y, w, loss, C)
    delta = np.linalg.norm(g)                      # Delta_0 = |g(w0)|
    for k, rec in enumerate(tr, start=1):
        # the inner solve of iteration k, on the Hessian at the *accepted* iterate
        s, pred, ncg, onb = _truncated_cg(H, g, delta, xi, max_cg)
        assert rec["cg_iters"] == ncg and bool(rec["on_boundary"]) == onb, k
        assert rec["snorm"] == pytest.approx(np.linalg.norm(s), rel=1e-9), k
        assert rec["pred"] == pytest.approx(pred, rel=1e-8), k
        if onb:
            assert rec["snorm"] == pytest.approx(delta, rel=1e-12), k
        assert rec["pred"] > 0
        ared = f - _f(X, y, w + s, loss, C)
        assert rec["ared"] == pytest.approx(ared, rel=1e-7, abs=1e-9 * abs(f)), k
        sigma = ared / pred
        # decisions (none of these trajectories comes within 1e-3 of a threshold, checked here)
        assert min(abs(sigma - 1e-4), abs(sigma - 0.25), abs(sigma - 0.75)) > 1e-3 * max(1.0, abs(sigma)), k
        accept = sigma > 1e-4
        assert bool(rec["accepted"]) == accept, k
        snorm = np.linalg.norm(s)
        if sigma < 0.25:
            delta = 0.5 * min(snorm, delta)
        elif sigma >= 0.75:
            delta = min(4.0 * delta, max(delta, 4.0 * snorm))
        assert rec["delta"] == pytest.approx(delta, rel=1e-9), k
        # the iterate after k iterations, from a solve capped at k iterations
        wk = o.tron(loss, C, eps, w0=w0, max_outer=k)
        assert wk.outer_iters == k
        if accept:
            np.testing.assert_allclose(wk.w, w + s, rtol=1e-8, atol=1e-10 * np.linalg.norm(w))
            w = wk.w.copy()
            f = _f(X, y, w, loss, C)
            g, H = _grad_hess(X, y, w, loss, C)
        else:
            np.testing.assert_array_equal(wk.w, w)          # a rejected step leaves w alone ...
            assert rec["f"] == tr[k - 2]["f"] if k > 1 else True   # ... and f
        assert rec["f"] == pytest.approx(f, rel=1e-13), k
        assert rec["gnorm"] == pytest.approx(np.linalg.norm(g), rel=1e-9), k
    assert np.linalg.norm(g) <= eps * g0
    return full


def _dense_oracle(X, y, lib=False):
    return Oracle(n=X.shape[0], d=X.shape[1], y=y, X=X, plain_fp64=lib)


def test_outer_loop_replayed_on_explicit_hessians_lr():
    check_outer_loop(_dense_oracle, LOSS_LR, 50.0)


def test_outer_loop_replayed_on_explicit_hessians_l2svm():
    check_outer_loop(_dense_oracle, LOSS_L2SVM, 1.0, problem=_separable_problem)


def test_rejected_step_shrinks_to_half_the_shorter_length():
    X, y, w0 = _far_start_problem()
    res = _dense_oracle(X, y).tron(LOSS_LR, 50.0, 1e-4, w0=w0)
    prev_delta = None
    seen = 0
    for k, rec in enumerate(res.trace):
        if k > 0 and not rec["accepted"]:
            assert rec["f"] == res.trace[k - 1]["f"] and rec["gnorm"] == res.trace[k - 1]["gnorm"]
            assert rec["ared"] / rec["pred"] <= 1e-4
            assert rec["delta"] == 0.5 * min(rec["snorm"], prev_delta)
            seen += 1
        prev_delta = rec["delta"]
    assert seen >= 5


def check_noise_rule(make_oracle):
    """With an unreachable eps the solve arrives where f(w) - f(w+s) is rounding noise of f: such a step counts as
    a success (sigma := 1), the solve ends (status 1) once one of them no longer reduces |g|, and the iterate is the
    minimiser to machine precision."""
    rng = np.random.default_rng(11)
    n, d, C = 300, 12, 3.0
    X = rng.standard_normal((n, d))
    y = np.where(rng.random(n) < 0.5, 1.0, -1.0)
    res = make_oracle(X, y).tron(LOSS_LR, C, 1e-20, max_outer=200)
    assert res.status == 1 and not res.converged and res.outer_iters < 200     # ended by the stall rule, not the cap
    noisy = [t for t in res.trace if abs(t["ared"]) <= 1e-12 * abs(t["f"]) and t["pred"] <= 1e-12 * abs(t["f"])]
    assert noisy and all(t["accepted"] for t in noisy)
    # at least one of them would have been rejected by the plain ratio test
    assert any(t["ared"] <= 1e-4 * t["pred"] for t in noisy)
    last = res.trace[-1]
    assert last in noisy and last["gnorm"] >= res.trace[-2]["gnorm"]
    for a, b in zip(res.trace[:-2], res.trace[1:-1]):
        assert b["gnorm"] < a["gnorm"]          # every earlier one still made progress
    w_star = _newton(X, y, LOSS_LR, C, np.zeros(d))
    assert np.linalg.norm(res.w - w_star) <= 1e-12 * np.linalg.norm(w_star)
    assert res.gnorm <= 1e-12 * res.gnorm0


def test_noise_level_reductions_are_accepted_and_the_solve_stops():
    check_noise_rule(_dense_oracle)


# ----------------------------------------------------------------------------
# planted mistakes: every one must be noticed by check_outer_loop
# ----------------------------------------------------------------------------
_MUTANTS = {
    "shrink_factor": (r"sig2 = 0\.5", "sig2 = 0.25"),
    "grow_factor": (r"sig3 = 4\.0", "sig3 = 2.0"),
    "accept_threshold": (r"eta0 = 1e-4", "eta0 = 0.3"),
    "shrink_threshold": (r"eta1 = 0\.25", "eta1 = 0.05"),
    "grow_threshold": (r"eta2 = 0\.75", "eta2 = 0.95"),
    "shrink_ignores_step_length": (r"sig2 \* fmin\(snorm, delta\)", "sig2 * delta"),
    "pred_sign": (r"vdot\(d, g, s\) - vdot\(d, s, r\)", "vdot(d, g, s) + vdot(d, s, r)"),
    "initial_radius": (r"double delta = gnorm;", "double delta = 0.001 * gnorm;"),
}


def _mutate(src, name):
    if name == "D_swapped_on_reject":
        # the Hessian diagonal of the trial point replaces the current one whether or not the step is taken
        swap = "{ double *t = Dcur; Dcur = Dnew; Dnew = t; }"
        assert src.count(swap) == 1
        out = src.replace("            " + swap + "\n", "")
        marker = "        int accepted = 0;\n"
        assert out.count(marker) == 1
        return out.replace(marker, "        " + swap + "\n" + marker)
    if name == "boundary_root":
        old = "const double tau = (double)((sp >= (acc_t)0) ? gap / (sp + rad) : (rad - sp) / pp);"
        assert src.count(old) == 2
        return src.replace(old, "const double tau = (double)((sp >= (acc_t)0) ? (rad - sp) / pp * 0.5 : gap / (sp + rad));", 1)
    pat, rep = _MUTANTS[name]
    out, nsub = re.subn(pat, rep, src, count=1)
    assert nsub == 1, name
    return out


@pytest.mark.parametrize("name", [k for k in _MUTANTS] + ["D_swapped_on_reject", "boundary_root"])
def test_planted_mistakes_are_noticed(tmp_path, name):
    src = open(os.path.join(os.path.dirname(orc.__file__), "tron_oracle.c")).read()
    c = tmp_path / f"mutant_{name}.c"
    c.write_text(_mutate(src, name))
    so = orc.build_variant(str(tmp_path / f"mutant_{name}.so"), str(c))
    with pytest.raises(AssertionError):
        check_outer_loop(lambda X, y: _dense_oracle(X, y, lib=so))


@pytest.mark.parametrize("name,pat,rep", [
    ("no_noise_rule", r"noise \? 1\.0 : ared / pred", "ared / pred"),
    ("no_stall_stop", r" \|\| \(noise && gnorm >= gnorm_before\)", ""),
])
def test_planted_mistakes_in_the_noise_rule_are_noticed(tmp_path, name, pat, rep):
    src = open(os.path.join(os.path.dirname(orc.__file__), "tron_oracle.c")).read()
    out, nsub = re.subn(pat, rep, src, count=1)
    assert nsub == 1
    c = tmp_path / f"mutant_{name}.c"
    c.write_text(out)
    so = orc.build_variant(str(tmp_path / f"mutant_{name}.so"), str(c))
    with pytest.raises(AssertionError):
        check_noise_rule(lambda X, y: _dense_oracle(X, y, lib=so))
