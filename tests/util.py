"""Helpers shared by the GPU parity tests."""
import os

import numpy as np

import paper_2008_03433_amd as tron
from oracle import Oracle

REL = 1e-10  # per-call parity gate (fp64), norm-wise
PROGRESS_DIR = os.environ.get("TRON_TEST_PROGRESS_DIR", "gpurun_out")   # relative to the repository root


def progress_reporter(capsys, label):
    """Returns a callback for Oracle.tron(progress=...): one line per finished outer iteration of a long oracle solve,
    printed past pytest's capture and appended to a log file in the run's output folder (PROGRESS_DIR), so that whoever
    watches the run sees the solve advance."""
    import os
    import sys
    import time
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    t0 = time.time()

    def report(rec):
        line = (f"[{label}] oracle outer iteration {rec['iter']}: {rec['cg_iters']} CG steps, f = {rec['f']:.10g}, "
                f"|g| = {rec['gnorm']:.3e} ({time.time() - t0:.0f} s)")
        with capsys.disabled():
            print(line, file=sys.stderr, flush=True)
        try:
            os.makedirs(os.path.join(root, PROGRESS_DIR), exist_ok=True)
            with open(os.path.join(root, PROGRESS_DIR, "test_progress.log"), "a") as fh:
                fh.write(line + "\n")
        except OSError:
            pass
    return report


def torch_mod():
    import torch
    return torch


def dev(a):
    torch = torch_mod()
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda")


def assert_vec_close(got, want, rel=REL, what=""):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, what
    assert np.isfinite(got).all(), what
    nrm = np.linalg.norm(want)
    err = np.linalg.norm(got - want)
    assert err <= rel * max(nrm, 1e-300), f"{what}: 2-norm rel err {err / max(nrm, 1e-300):.3e}"
    mx = np.abs(want).max() if want.size else 0.0
    assert np.abs(got - want).max() <= rel * max(mx, 1e-300), f"{what}: max-abs err {np.abs(got - want).max():.3e} vs max {mx:.3e}"


def assert_scalar_close(got, want, rel=REL, what=""):
    assert np.isfinite(got), what
    assert abs(got - want) <= rel * max(abs(want), 1e-300), f"{what}: {got!r} vs {want!r}"


def check_calls(problem, loss, C, rng, w_scale=0.3, n_hv=2):
    """fun_grad + hv through the C ABI against the oracle at a random w and random v's."""
    torch = torch_mod()
    o = Oracle.from_problem(problem)
    ds = tron.Dataset.from_problem(problem)
    try:
        w = w_scale * rng.standard_normal(problem.d)
        f_o, g_o, D_o = o.fun_grad(loss, C, w)
        w_d = dev(w)
        g_d = torch.empty(problem.d, dtype=torch.float64, device="cuda")
        f_g = ds.fun_grad(loss, C, w_d, g_d)
        assert_scalar_close(f_g, f_o, what="f")
        assert_vec_close(g_d.cpu().numpy(), g_o, what="g")
        # function value only (g = NULL) gives the same f
        assert ds.fun_grad(loss, C, w_d, None) == f_g
        for _ in range(n_hv):
            v = rng.standard_normal(problem.d)
            Hv_o = o.hv(C, D_o, v)
            v_d = dev(v)
            Hv_d = torch.empty_like(v_d)
            vHv = ds.hv(C, v_d, Hv_d)
            assert_vec_close(Hv_d.cpu().numpy(), Hv_o, what="Hv")
            assert_scalar_close(vHv, float(v @ Hv_o), what="v.Hv")
    finally:
        ds.close()


def compare_solves(problem, loss, C, eps, obj_rel=1e-8, trace_rel=1e-8, w0=None, **kw):
    torch = torch_mod()
    o = Oracle.from_problem(problem)
    ref = o.tron(loss, C, eps, w0=w0, **kw)
    ds = tron.Dataset.from_problem(problem)
    try:
        w = torch.zeros(problem.d, dtype=torch.float64, device="cuda") if w0 is None else dev(w0)
        res = ds.solve(loss, C, eps, w, **kw)
        assert res.status == ref.status and res.converged == ref.converged
        assert abs(res.f - ref.f) <= obj_rel * abs(ref.f), f"objective {res.f!r} vs {ref.f!r}"
        # same discrete trajectory
        assert res.outer_iters == ref.outer_iters and res.cg_iters_total == ref.cg_iters_total
        assert (res.n_fun, res.n_grad, res.n_hv) == (ref.n_fun, ref.n_grad, ref.n_hv)
        assert [(t["cg_iters"], t["accepted"], t["on_boundary"]) for t in res.trace] == \
               [(t["cg_iters"], t["accepted"], t["on_boundary"]) for t in ref.trace]
        for a, b in zip(res.trace, ref.trace):
            assert abs(a["f"] - b["f"]) <= trace_rel * abs(b["f"])
            assert abs(a["delta"] - b["delta"]) <= max(trace_rel, 1e-8) * abs(b["delta"])
        assert_scalar_close(res.gnorm0, ref.gnorm0, what="gnorm0")
        assert_vec_close(w.cpu().numpy(), ref.w, rel=max(1e-8, 10 * trace_rel), what="w")
        # stationarity re-checked by the oracle at the GPU's iterate
        f_chk, g_chk, _ = o.fun_grad(loss, C, w.cpu().numpy())
        if ref.converged:
            assert np.linalg.norm(g_chk) <= eps * ref.gnorm0 * (1 + 1e-9)
        assert abs(f_chk - res.f) <= 1e-10 * abs(f_chk)
        return res, ref
    finally:
        ds.close()
