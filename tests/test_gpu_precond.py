"""GPU parity of the diagonally preconditioned path (Hessian diagonal, preconditioned CG inside the trust region)
against the CPU oracle, through the C ABI."""
import numpy as np
import pytest

import datagen as dg
from datagen import DenseProblem
from oracle import LOSS_LR, LOSS_L2SVM, Oracle

pytestmark = pytest.mark.gpu

from util import assert_vec_close, compare_solves, dev, torch_mod  # noqa: E402


def _check_diag(problem, loss, C, rng, w_scale):
    import paper_2008_03433_amd as tron
    torch = torch_mod()
    o = Oracle.from_problem(problem)
    ds = tron.Dataset.from_problem(problem)
    try:
        w = w_scale * rng.standard_normal(problem.d)
        _, _, D = o.fun_grad(loss, C, w)
        ds.fun_grad(loss, C, dev(w), None)
        hd = torch.empty(problem.d, dtype=torch.float64, device="cuda")
        ds.hess_diag(C, hd)
        assert_vec_close(hd.cpu().numpy(), o.hess_diag(C, D), what="diag(H)")
    finally:
        ds.close()


def _dense(rng, n, d):
    X = rng.standard_normal((n, d))
    return DenseProblem("rand", n, d, X, np.where(rng.random(n) < 0.5, 1.0, -1.0))


@pytest.mark.parametrize("loss", [LOSS_LR, LOSS_L2SVM])
@pytest.mark.parametrize("n,d", [(4097, 24), (777, 18), (300, 1), (1025, 33), (130, 257)])
def test_hess_diag_dense(rng, loss, n, d):
    _check_diag(_dense(rng, n, d), loss, 0.7, rng, 0.5 / np.sqrt(d))


@pytest.mark.parametrize("loss", [LOSS_LR, LOSS_L2SVM])
def test_hess_diag_csr(rng, loss):
    _check_diag(dg.config1(), loss, 1.0, rng, 1.0)
    _check_diag(dg.config2(), loss, 1.0, rng, 1.0)


def test_hess_diag_partitioned_layout(rng):
    import paper_2008_03433_amd as tron
    tron.tron_tuning_set("csr_parts", 8)
    try:
        _check_diag(dg.config2(), LOSS_LR, 1.0, rng, 1.0)
        _check_diag(dg.config3(scale=0.02), LOSS_L2SVM, 1.0, rng, 0.5)
        tron.tron_tuning_set("csr_tiles", 0)
        _check_diag(dg.config3(scale=0.02), LOSS_LR, 1.0, rng, 0.5)
    finally:
        tron.tron_tuning_set("csr_tiles", 1)
        tron.tron_tuning_set("csr_parts", 0)


@pytest.mark.parametrize("blend", [0.01, 1.0])
def test_preconditioned_solve_config1_and_2(blend):
    p = dg.config1()
    compare_solves(p, p.loss, p.C, p.eps, precond_blend=blend)
    p = dg.config2()
    compare_solves(p, p.loss, p.C, p.eps, precond_blend=blend)


def test_preconditioned_solve_dense(rng):
    p = dg.config4(n=200_000)
    compare_solves(p, p.loss, p.C, p.eps, precond_blend=0.01)
    # badly scaled features, tight tolerance, both losses
    n, d = 3000, 12
    X = rng.standard_normal((n, d))
    X[:, :3] *= 25.0
    q = DenseProblem("scaled", n, d, X, np.where(rng.random(n) < 0.5, 1.0, -1.0))
    for loss in (LOSS_LR, LOSS_L2SVM):
        res, ref = compare_solves(q, loss, 1.0, 1e-8, precond_blend=1.0)
        plain = Oracle.from_problem(q).tron(loss, 1.0, 1e-8)
        assert abs(res.f - plain.f) <= 1e-10 * abs(plain.f)      # the minimiser does not depend on the inner solver


def test_preconditioned_solve_hits_the_boundary_and_rejects(rng):
    p = _dense(rng, 2000, 10)
    w0 = 3.0 * rng.standard_normal(p.d)
    res, ref = compare_solves(p, LOSS_LR, 50.0, 1e-6, w0=w0, precond_blend=0.01)
    assert any(t["on_boundary"] for t in ref.trace)


def test_preconditioned_solve_url_shape(rng):
    # url-shaped data in the partitioned layout (tiles, head partition, cold remainder all take part in diag(H));
    # tight eps, where solves are comparable on this matrix (see test_solve_url_shape_scaled)
    import paper_2008_03433_amd as tron
    tron.tron_tuning_set("csr_parts", 8)
    try:
        p = dg.config3(scale=0.05)
        torch = torch_mod()
        o = Oracle.from_problem(p)
        ref = o.tron(p.loss, p.C, 1e-6, precond_blend=0.01)
        ds = tron.Dataset.from_problem(p)
        try:
            w = torch.zeros(p.d, dtype=torch.float64, device="cuda")
            res = ds.solve(p.loss, p.C, 1e-6, w, precond_blend=0.01)
            assert res.converged and ref.converged
            assert abs(res.f - ref.f) <= 1e-8 * abs(ref.f)
            for a, b in list(zip(res.trace, ref.trace))[:2]:
                assert (a["cg_iters"], a["accepted"]) == (b["cg_iters"], b["accepted"])
                assert abs(a["f"] - b["f"]) <= 1e-8 * abs(b["f"])
                assert abs(a["snorm"] - b["snorm"]) <= 1e-8 * abs(b["snorm"])
            f_chk, g_chk, _ = o.fun_grad(p.loss, p.C, w.cpu().numpy())
            assert np.linalg.norm(g_chk) <= 1e-6 * ref.gnorm0 * (1 + 1e-9)
        finally:
            ds.close()
    finally:
        tron.tron_tuning_set("csr_parts", 0)


def test_blend_out_of_range_is_rejected(rng):
    import paper_2008_03433_amd as tron
    torch = torch_mod()
    ds = tron.Dataset.from_problem(_dense(rng, 50, 4))
    try:
        w = torch.zeros(4, dtype=torch.float64, device="cuda")
        for bad in (-0.1, 1.5, float("nan")):
            with pytest.raises(tron.TronError):
                ds.solve(LOSS_LR, 1.0, 0.01, w, precond_blend=bad)
        hd = torch.empty(4, dtype=torch.float64, device="cuda")
        with pytest.raises(tron.TronError):
            ds.hess_diag(1.0, hd)          # no D cached yet
    finally:
        ds.close()
