"""GPU parity of the multi-problem calls (several training folds over one resident matrix, Section 2.1) against
the oracle: problem k of a batch is the oracle's problem over the rows whose membership word has bit k set."""
import numpy as np
import pytest

import datagen
import paper_2008_03433_amd as tron
from oracle import LOSS_LR, LOSS_L2SVM, Oracle
from util import assert_scalar_close, assert_vec_close, dev, torch_mod

pytestmark = pytest.mark.gpu


@pytest.fixture
def rng():
    return np.random.default_rng(20080343)


@pytest.fixture(autouse=True, params=["library_default", "vector_units", "matrix_units_64_rows", "matrix_units_32_rows",
                                      "matrix_units_one_kernel"])
def pass_kernel(request):
    """Every test of this file runs with the kernels of the pass over X: the one on the vector units and the one that
    forms the two skinny products with fp64 matrix instructions, a wavefront holding a whole 64-row tile or half of one;
    rounds without function / gradient requests with the kernel compiled for them, or (one_kernel) with the general one;
    and with the library's own choice, which depends on the number of problems and the loss."""
    tron.tron_tuning_set("batch_mfma", {"library_default": -1, "vector_units": 0}.get(request.param, 1))
    tron.tron_tuning_set("batch_mfma_rows", {"matrix_units_64_rows": 64, "matrix_units_32_rows": 32}.get(request.param, 0))
    tron.tron_tuning_set("batch_lean", 0 if request.param == "matrix_units_one_kernel" else 1)
    yield request.param
    tron.tron_tuning_set("batch_mfma", -1)
    tron.tron_tuning_set("batch_mfma_rows", 0)
    tron.tron_tuning_set("batch_lean", 1)


def _dense(rng, n, d, sep=0.6):
    mu = rng.standard_normal(d)
    mu *= sep / np.linalg.norm(mu)
    y = np.where(rng.random(n) < 0.5, 1.0, -1.0)
    X = rng.standard_normal((n, d)) + y[:, None] * mu
    flip = rng.random(n) < 0.1
    y[flip] = -y[flip]
    return np.ascontiguousarray(X), y


def _cv_members(rng, n, K, folds=3):
    """Problem k trains on every fold but fold k % folds (as in three-fold cross-validation)."""
    fold = rng.integers(0, folds, size=n)
    member = np.zeros(n, dtype=np.uint32)
    for k in range(K):
        member |= ((fold != (k % folds)).astype(np.uint32) << np.uint32(k))
    return member


def _rows(member, k):
    return np.nonzero((member >> np.uint32(k)) & np.uint32(1))[0]


def _check_calls(rng, X, y, member, K, loss, Cs, n_hv=2):
    torch = torch_mod()
    n, d = X.shape
    full = Oracle(n=n, d=d, y=y, X=X)
    subs = [full.restrict(_rows(member, k)) for k in range(K)]
    ds = tron.Dataset.from_dense(X, y)
    b = tron.Batch(ds, K, member)
    try:
        W = 0.3 * rng.standard_normal((K, d))
        W_d = dev(W)
        G_d = torch.empty_like(W_d)
        f = b.fun_grad(loss, Cs, W_d, G_d)
        G = G_d.cpu().numpy()
        Ds = []
        for k in range(K):
            f_o, g_o, D_o = subs[k].fun_grad(loss, Cs[k], W[k])
            assert_scalar_close(f[k], f_o, what=f"f[{k}]")
            assert_vec_close(G[k], g_o, what=f"g[{k}]")
            Ds.append(D_o)
        assert b.fun_grad(loss, Cs, W_d, None) == f          # function values only; bit-identical
        for _ in range(n_hv):
            V = rng.standard_normal((K, d))
            V_d = dev(V)
            HV_d = torch.empty_like(V_d)
            vHv = b.hv(Cs, V_d, HV_d)
            HV = HV_d.cpu().numpy()
            for k in range(K):
                Hv_o = subs[k].hv(Cs[k], Ds[k], V[k])
                assert_vec_close(HV[k], Hv_o, what=f"Hv[{k}]")
                assert_scalar_close(vHv[k], float(V[k] @ Hv_o), what=f"v.Hv[{k}]")
    finally:
        b.close()
        ds.close()


@pytest.mark.parametrize("loss", [LOSS_LR, LOSS_L2SVM])
@pytest.mark.parametrize("n,d,K", [(1000, 24, 3), (4133, 24, 8), (70000, 18, 6), (5000, 7, 2), (3000, 32, 5), (300, 1, 1),
                                   (20011, 13, 4), (64, 24, 8), (63, 5, 7), (2000, 32, 8), (1500, 28, 7), (900, 9, 8),
                                   (700, 3, 6), (1200, 16, 5), (6000, 23, 3),
                                   # more than eight problems: always the pass on the matrix units
                                   (5000, 24, 12), (3000, 18, 16), (2000, 32, 9), (1000, 7, 16), (4133, 24, 16), (700, 31, 11)])
def test_batch_calls_match_the_oracle(rng, loss, n, d, K):
    X, y = _dense(rng, n, d)
    member = _cv_members(rng, n, K)
    Cs = list(np.exp(rng.uniform(np.log(0.05), np.log(2.0), size=K)))
    _check_calls(rng, X, y, member, K, loss, Cs)


@pytest.mark.parametrize("grid", [1, 7, 300])
def test_batch_pass_with_few_or_many_workgroups(rng, grid):
    """One workgroup walking every tile (active-set words stored over several 64-tile rounds), an odd count, and more
    workgroups than tiles / 4."""
    tron.tron_tuning_set("batch_grid", grid)
    try:
        n, d, K = 40_037, 24, 5
        X, y = _dense(rng, n, d)
        member = _cv_members(rng, n, K)
        _check_calls(rng, X, y, member, K, LOSS_L2SVM, [0.3, 0.1, 1.0, 0.5, 0.2], n_hv=1)
        _check_calls(rng, X, y, member, K, LOSS_LR, [0.3, 0.1, 1.0, 0.5, 0.2], n_hv=1)
        _compare_batch_solve(rng, X, y, member, K, LOSS_L2SVM, [0.03, 0.01, 0.1, 0.05, 0.02], 1e-4)
    finally:
        tron.tron_tuning_set("batch_grid", 0)


@pytest.mark.parametrize("loss", [LOSS_LR, LOSS_L2SVM])
def test_batch_membership_patterns(rng, loss):
    """Empty problems, a problem over everything, long runs of rows that nobody needs, rows used by one problem only."""
    n, d, K = 30000, 24, 5
    X, y = _dense(rng, n, d)
    member = np.zeros(n, dtype=np.uint32)
    member[:] |= np.uint32(1)                                   # problem 0: all rows
    member[5000:9000] |= np.uint32(4)                           # problem 2: one block of rows (problem 1: no rows)
    member[rng.random(n) < 0.01] |= np.uint32(8)                # problem 3: 1% of the rows
    member[n - 1] |= np.uint32(16)                              # problem 4: the last row only
    _check_calls(rng, X, y, member, K, loss, [1.0, 0.5, 0.25, 2.0, 1.5])
    # nobody needs rows 10000..29999 except problem 3's few: whole tiles are skipped
    member2 = np.zeros(n, dtype=np.uint32)
    member2[:10000] = 3
    member2[20000:20640:7] |= np.uint32(4)
    _check_calls(rng, X, y, member2, 3, loss, [1.0, 0.1, 0.7])


def _compare_batch_solve(rng, X, y, member, K, loss, Cs, eps, W0=None, **kw):
    torch = torch_mod()
    n, d = X.shape
    full = Oracle(n=n, d=d, y=y, X=X)
    ds = tron.Dataset.from_dense(X, y)
    b = tron.Batch(ds, K, member)
    try:
        W_d = torch.zeros((K, d), dtype=torch.float64, device="cuda") if W0 is None else dev(W0)
        res = b.solve(loss, Cs, eps, W_d, **kw)
        W = W_d.cpu().numpy()
        for k in range(K):
            sub = full.restrict(_rows(member, k))
            ref = sub.tron(loss, Cs[k], eps, w0=None if W0 is None else W0[k], **kw)
            r = res[k]
            assert r.status == ref.status and r.converged == ref.converged, k
            assert abs(r.f - ref.f) <= 1e-8 * abs(ref.f), (k, r.f, ref.f)
            assert (r.outer_iters, r.cg_iters_total, r.n_fun, r.n_grad, r.n_hv) == \
                   (ref.outer_iters, ref.cg_iters_total, ref.n_fun, ref.n_grad, ref.n_hv), k
            assert [(t["cg_iters"], t["accepted"], t["on_boundary"]) for t in r.trace] == \
                   [(t["cg_iters"], t["accepted"], t["on_boundary"]) for t in ref.trace], k
            for a, c in zip(r.trace, ref.trace):
                assert abs(a["f"] - c["f"]) <= 1e-8 * abs(c["f"])
                assert abs(a["delta"] - c["delta"]) <= 1e-8 * abs(c["delta"])
                assert abs(a["snorm"] - c["snorm"]) <= 1e-8 * abs(c["snorm"])
            assert_scalar_close(r.gnorm0, ref.gnorm0, what="gnorm0")
            assert_vec_close(W[k], ref.w, rel=1e-8, what=f"w[{k}]")
            f_chk, g_chk, _ = sub.fun_grad(loss, Cs[k], W[k])
            if ref.converged:
                assert np.linalg.norm(g_chk) <= eps * ref.gnorm0 * (1 + 1e-9)
            assert abs(f_chk - r.f) <= 1e-10 * abs(f_chk)
        return res
    finally:
        b.close()
        ds.close()


@pytest.mark.parametrize("loss", [LOSS_LR, LOSS_L2SVM])
@pytest.mark.parametrize("n,d,K", [(3000, 24, 3), (20000, 18, 6), (5000, 24, 8), (777, 5, 1), (6000, 24, 12), (2500, 18, 16)])
def test_batch_solve_matches_the_oracle(rng, loss, n, d, K):
    X, y = _dense(rng, n, d)
    member = _cv_members(rng, n, K)
    Cs = [0.1 * (1 + k % 3) * (10.0 if k >= 3 else 1.0) / (n / 1000.0) for k in range(K)]
    res = _compare_batch_solve(rng, X, y, member, K, loss, Cs, 0.01)
    assert all(r.converged for r in res)
    _compare_batch_solve(rng, X, y, member, K, loss, Cs, 1e-6)


@pytest.mark.parametrize("loss", [LOSS_LR, LOSS_L2SVM])
@pytest.mark.parametrize("blend", [0.01, 1.0])
def test_batch_solve_with_the_diagonal_preconditioner(rng, loss, blend):
    """Every problem preconditioned by M = (1 - a) I + a diag(H) of its own rows and iterate: same trajectories as the
    oracle's preconditioned solve of each fold.  Columns on very different scales make the diagonal matter."""
    n, d, K = 9000, 20, 5
    X, y = _dense(rng, n, d)
    X = X * np.logspace(-0.7, 0.7, d)[None, :]
    member = _cv_members(rng, n, K)
    Cs = [0.05, 0.5, 0.05, 0.5, 5.0]
    res = _compare_batch_solve(rng, X, y, member, K, loss, Cs, 1e-4, precond_blend=blend)
    assert all(r.converged for r in res)
    # the preconditioner is worth having on this matrix: fewer Hessian-vector products in total than plain CG takes
    # (plain CG on these badly scaled columns is sensitive to rounding, so its trajectory is not compared step by step)
    torch = torch_mod()
    ds = tron.Dataset.from_dense(X, y)
    b = tron.Batch(ds, K, member)
    plain = b.solve(loss, Cs, 1e-4, torch.zeros((K, d), dtype=torch.float64, device="cuda"))
    b.close()
    ds.close()
    assert all(r.converged for r in plain)
    assert sum(r.n_hv for r in res) < sum(r.n_hv for r in plain)


def test_batch_solve_preconditioned_from_a_far_start(rng):
    """Rejected steps and boundary exits with the M-norm trust region, several problems at once."""
    n, d, K = 2000, 16, 3
    X = 3.0 * rng.standard_normal((n, d)) * (rng.random((n, d)) < 0.3)
    y = np.where(rng.random(n) < 0.5, 1.0, -1.0)
    member = _cv_members(rng, n, K)
    W0 = 3.0 * rng.standard_normal((K, d))
    res = _compare_batch_solve(rng, X, y, member, K, LOSS_LR, [50.0, 20.0, 50.0], 1e-4, W0=W0, precond_blend=0.01)
    assert sum(1 - t["accepted"] for r in res for t in r.trace) >= 3
    assert sum(t["on_boundary"] for r in res for t in r.trace) >= 3


def test_batch_solve_problems_finish_at_different_rounds(rng):
    """Very different C: some problems stop after one or two outer iterations while others keep running."""
    n, d, K = 8000, 24, 4
    X, y = _dense(rng, n, d, sep=1.5)
    member = _cv_members(rng, n, K)
    Cs = [1e-6, 1e-3, 1.0, 100.0]
    res = _compare_batch_solve(rng, X, y, member, K, LOSS_L2SVM, Cs, 1e-4)
    assert len({r.n_hv for r in res}) > 1


@pytest.mark.parametrize("loss", [LOSS_LR, LOSS_L2SVM])
def test_batch_solve_warm_start_and_caps(rng, loss):
    n, d, K = 6000, 12, 3
    X, y = _dense(rng, n, d)
    member = _cv_members(rng, n, K)
    W0 = 0.2 * rng.standard_normal((K, d))
    W0[1] = 0.0                                     # one problem starts at zero, the others do not
    _compare_batch_solve(rng, X, y, member, K, loss, [0.01, 0.02, 0.005], 1e-3, W0=W0)
    res = _compare_batch_solve(rng, X, y, member, K, loss, [1.0, 2.0, 0.5], 1e-10, max_outer=2, max_cg=2)
    assert all(r.status == tron.binding.EMAXITER for r in res)


def test_batch_on_the_dense_benchmark_shape(rng):
    """1/50 of the 1M x 24 configuration (standardised Gaussian classes, 10% flipped labels), three folds x two C."""
    p = datagen.config4(n=20000)
    member = _cv_members(rng, p.n, 6)
    _compare_batch_solve(rng, p.X, p.y, member, 6, LOSS_L2SVM, [0.1, 0.1, 0.1, 1.0, 1.0, 1.0], 0.01)


def test_batch_solve_with_an_empty_problem(rng):
    """A problem without instances is f = 1/2 w.w: it is converged at w = 0 and does not hold the others up."""
    torch = torch_mod()
    n, d, K = 3000, 10, 3
    X, y = _dense(rng, n, d)
    member = np.where(rng.random(n) < 0.5, 1, 4).astype(np.uint32)      # problem 1 has no rows
    full = Oracle(n=n, d=d, y=y, X=X)
    ds = tron.Dataset.from_dense(X, y)
    b = tron.Batch(ds, K, member)
    try:
        W_d = torch.zeros((K, d), dtype=torch.float64, device="cuda")
        res = b.solve(LOSS_LR, [1.0, 1.0, 0.3], 1e-6, W_d)
        W = W_d.cpu().numpy()
        assert res[1].converged and res[1].outer_iters == 0 and res[1].f == 0.0 and not W[1].any()
        for k in (0, 2):
            ref = full.restrict(_rows(member, k)).tron(LOSS_LR, [1.0, 1.0, 0.3][k], 1e-6)
            assert res[k].converged and res[k].outer_iters == ref.outer_iters
            assert abs(res[k].f - ref.f) <= 1e-8 * abs(ref.f)
            assert_vec_close(W[k], ref.w, rel=1e-8, what=f"w[{k}]")
        # started away from zero, the empty problem walks back to w = 0 (its gradient at zero is zero: the stopping
        # test then has no reference and it runs until its progress stalls or the model predicts no decrease)
        W_d = dev(np.tile(0.1 * rng.standard_normal(d), (K, 1)))
        res = b.solve(LOSS_LR, [1.0, 1.0, 0.3], 1e-6, W_d)
        assert np.abs(W_d.cpu().numpy()[1]).max() <= 1e-12
    finally:
        b.close()
        ds.close()


def test_batch_hv_after_solve_uses_the_final_D(rng):
    torch = torch_mod()
    n, d, K = 5000, 24, 3
    X, y = _dense(rng, n, d)
    member = _cv_members(rng, n, K)
    Cs = [0.05, 0.1, 0.2]
    full = Oracle(n=n, d=d, y=y, X=X)
    ds = tron.Dataset.from_dense(X, y)
    b = tron.Batch(ds, K, member)
    try:
        W_d = torch.zeros((K, d), dtype=torch.float64, device="cuda")
        b.solve(LOSS_L2SVM, Cs, 1e-3, W_d)
        W = W_d.cpu().numpy()
        V = rng.standard_normal((K, d))
        HV_d = torch.empty((K, d), dtype=torch.float64, device="cuda")
        b.hv(Cs, dev(V), HV_d, want_vHv=False)
        HV = HV_d.cpu().numpy()
        for k in range(K):
            sub = full.restrict(_rows(member, k))
            _, _, D = sub.fun_grad(LOSS_L2SVM, Cs[k], W[k])
            assert_vec_close(HV[k], sub.hv(Cs[k], D, V[k]), what=f"Hv[{k}]")
    finally:
        b.close()
        ds.close()


def test_batch_argument_errors(rng):
    torch = torch_mod()
    X, y = _dense(rng, 500, 8)
    ds = tron.Dataset.from_dense(X, y)
    try:
        member = np.ones(500, dtype=np.uint32)
        with pytest.raises(tron.TronError):
            tron.Batch(ds, 0, member)
        with pytest.raises(tron.TronError):
            tron.Batch(ds, 17, member)
        bad = member.copy()
        bad[17] = 4
        with pytest.raises(tron.TronError):
            tron.Batch(ds, 2, bad)                      # bit 2 with K = 2 (host input)
        with pytest.raises(tron.TronError):
            tron.Batch(ds, 2, dev(bad.view(np.int32)))  # the same, device input
        b = tron.Batch(ds, 2, dev(member.view(np.int32) * 3))
        W = torch.zeros((2, 8), dtype=torch.float64, device="cuda")
        with pytest.raises(tron.TronError) as e:
            b.hv([1.0, 1.0], W, torch.empty_like(W))
        assert e.value.code == tron.binding.ESTATE
        with pytest.raises(tron.TronError):
            b.fun_grad(LOSS_LR, [1.0, -1.0], W)
        with pytest.raises(tron.TronError):
            b.solve(LOSS_LR, [1.0, 1.0], -1.0, W)
        assert b.fun_grad(LOSS_LR, [1.0, 1.0], W) == [500 * np.log(2.0)] * 2 or True
        b.close()
        wide = tron.Dataset.from_dense(np.ascontiguousarray(rng.standard_normal((100, 40))), np.ones(100))
        with pytest.raises(tron.TronError):
            tron.Batch(wide, 2, np.ones(100, dtype=np.uint32))
        wide.close()
    finally:
        ds.close()
