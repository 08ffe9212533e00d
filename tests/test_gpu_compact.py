"""The compacted copy of the active rows (X_hat = X_I, Section 5 of the paper) against the oracle and against the
row-skipping pass over X."""
import numpy as np
import pytest

import datagen as dg
from oracle import LOSS_L2SVM, Oracle

pytestmark = pytest.mark.gpu

from util import assert_scalar_close, assert_vec_close, compare_solves, dev, torch_mod  # noqa: E402


@pytest.fixture
def compact_knob():
    import paper_2008_03433_amd as tron

    def set_knob(v):
        tron.tron_tuning_set("dense_compact", v)
    yield set_knob
    tron.tron_tuning_set("dense_compact", -1)
    tron.tron_tuning_set("dense_device_driver", -1)


def _separable(rng, n, d):
    X = rng.standard_normal((n, d))
    wt = rng.standard_normal(d)
    wt /= np.linalg.norm(wt)
    y = np.where(X @ wt >= 0, 1.0, -1.0)
    return X, y, wt


@pytest.mark.parametrize("n,d,scale,lo,hi", [
    (1_000_003, 24, 1.9, 0.3, 0.5),       # about 40% of the rows active, ragged last tile
    (1_000_003, 24, 16.0, 0.02, 0.08),    # about 5%
    (70_001, 7, 2.0, 0.1, 0.6),           # odd d: rows moved 8 bytes at a time
    (50_000, 32, 2.0, 0.1, 0.6),          # the widest supported row
    (333, 18, 2.0, 0.05, 0.9),            # fewer rows than a workgroup's share of the scan
])
def test_hv_over_the_compacted_copy(rng, compact_knob, n, d, scale, lo, hi):
    import paper_2008_03433_amd as tron
    torch = torch_mod()
    X, y, wt = _separable(rng, n, d)
    C = 0.5
    o = Oracle(n=n, d=d, y=y, X=X)
    w = scale * wt + 0.05 * rng.standard_normal(d)
    f_o, g_o, D_o = o.fun_grad(LOSS_L2SVM, C, w)
    frac = float(np.mean(D_o != 0.0))
    assert lo < frac < hi, frac
    ds = tron.Dataset.from_dense(X, y)
    try:
        w_d = dev(w)
        g_d = torch.empty_like(w_d)
        out = {}
        for knob in (0, 1):
            compact_knob(knob)
            f = ds.fun_grad(LOSS_L2SVM, C, w_d, g_d)
            assert_scalar_close(f, f_o, what="f")
            assert_vec_close(g_d.cpu().numpy(), g_o, what="g")
            rows = tron.tron_dataset_stat(ds.handle, "dense_compact_rows")
            assert rows == (int(np.count_nonzero(D_o)) if knob else 0)
            res = []
            for k in range(2):
                v = np.random.default_rng(100 + k).standard_normal(d)
                v_d = dev(v)
                Hv_d = torch.empty_like(v_d)
                vHv = ds.hv(C, v_d, Hv_d)
                Hv_o = o.hv(C, D_o, v)
                assert_vec_close(Hv_d.cpu().numpy(), Hv_o, what=f"Hv (dense_compact = {knob})")
                assert_scalar_close(vHv, float(v @ Hv_o), what="v.Hv")
                res.append(Hv_d.cpu().numpy())
            hd = torch.empty_like(w_d)
            ds.hess_diag(C, hd)
            np.testing.assert_allclose(hd.cpu().numpy(), o.hess_diag(C, D_o), rtol=1e-11)
            out[knob] = res
        for a, b in zip(out[0], out[1]):
            assert_vec_close(a, b, rel=1e-12, what="compacted against row-skipping")
        # a new function/gradient call replaces D: the copy must follow the new active set
        compact_knob(1)
        w2 = 0.5 * w
        f2_o, _, D2_o = o.fun_grad(LOSS_L2SVM, C, w2)
        ds.fun_grad(LOSS_L2SVM, C, dev(w2), None)
        assert tron.tron_dataset_stat(ds.handle, "dense_compact_rows") == int(np.count_nonzero(D2_o))
        v = rng.standard_normal(d)
        Hv_d = torch.empty(d, dtype=torch.float64, device="cuda")
        ds.hv(C, dev(v), Hv_d)
        assert_vec_close(Hv_d.cpu().numpy(), o.hv(C, D2_o, v), what="Hv after the active set changed")
    finally:
        ds.close()


@pytest.mark.parametrize("knob", [1, -1])
@pytest.mark.parametrize("C,scale", [(1.0, 20.0), (10.0, 100.0)])
def test_solves_with_the_compacted_copy_follow_the_oracle(compact_knob, knob, C, scale):
    """Far out along a separating direction few rows are active, steps get rejected (the copy of the accepted iterate
    must survive a rejected trial point) and the active set grows from iterate to iterate (the copy must grow).  A tight
    inner tolerance makes the inner solves long enough for the automatic rule to ask for the copy."""
    import paper_2008_03433_amd as tron
    torch = torch_mod()
    rng = np.random.default_rng(7)
    n, d = 1500, 30
    X, y, wt = _separable(rng, n, d)
    o = Oracle(n=n, d=d, y=y, X=X)
    ref = o.tron(LOSS_L2SVM, C, 1e-6, w0=scale * wt, xi=0.001)
    assert ref.converged and sum(1 - t["accepted"] for t in ref.trace) >= 3
    assert max(t["cg_iters"] for t in ref.trace) >= 10
    tron.tron_tuning_set("dense_device_driver", 0)      # the host-driven path is the one that compacts
    compact_knob(knob)
    ds = tron.Dataset.from_dense(X, y)
    try:
        w = dev(scale * wt)
        tron.tron_profile_enable(ds.handle, True)
        res = ds.solve(LOSS_L2SVM, C, 1e-6, w, cg_xi=0.001)
        prof = tron.tron_profile_read(ds.handle)
        tron.tron_profile_enable(ds.handle, False)
        assert res.converged
        assert [(t["cg_iters"], t["accepted"], t["on_boundary"]) for t in res.trace] == \
               [(t["cg_iters"], t["accepted"], t["on_boundary"]) for t in ref.trace]
        for a, b in zip(res.trace, ref.trace):
            assert abs(a["f"] - b["f"]) <= 1e-8 * abs(b["f"])
            assert abs(a["delta"] - b["delta"]) <= 1e-8 * abs(b["delta"])
        assert abs(res.f - ref.f) <= 1e-8 * abs(ref.f)
        assert_vec_close(w.cpu().numpy(), ref.w, rel=1e-8, what="w")
        # copies were built along the way (one per accepted iterate when forced; after long inner solves otherwise)
        built = prof.get("dense_compact", {"calls": 0})["calls"]
        accepted = sum(t["accepted"] for t in ref.trace)
        assert built >= (accepted if knob == 1 else 2), (built, accepted)
    finally:
        ds.close()
