"""The allocation-free Hessian-vector entry point (tron_hv_static) against tron_hv, through the C ABI."""
import numpy as np
import pytest

import paper_2008_03433_amd as tron
from oracle import LOSS_LR, LOSS_L2SVM, Oracle
from util import assert_vec_close, assert_scalar_close, dev, torch_mod

pytestmark = pytest.mark.gpu


def _handle(rng, n, d):
    X = rng.standard_normal((n, d))
    y = np.where(rng.random(n) < 0.5, 1.0, -1.0)
    return X, y, tron.Dataset.from_dense(X, y)


def _both(ds, C, v):
    torch = torch_mod()
    Hv_a, Hv_b = torch.empty_like(v), torch.full_like(v, float("nan"))
    s_b = torch.full((1,), float("nan"), dtype=torch.float64, device="cuda")
    s_a = ds.hv(C, v, Hv_a)
    ds.hv_static(C, v, Hv_b, s_b)
    torch.cuda.synchronize()
    return Hv_a.cpu().numpy(), s_a, Hv_b.cpu().numpy(), float(s_b.cpu()[0])


@pytest.mark.parametrize("loss", [LOSS_LR, LOSS_L2SVM])
def test_static_hv_equals_hv_on_two_calls_in_a_row(loss):
    """Two handles, the second smaller (fewer workgroups, fewer columns): the second call finds the first call's
    partial sums in the shared static array and must not read them."""
    rng = np.random.default_rng(77 + loss)
    C = 0.7
    big = _handle(rng, 300_001, 24)      # 2048 workgroups would be 600k rows: here about 1172, ragged last tile
    small = _handle(rng, 5_003, 17)      # odd d: the scalar-load variant of the kernels
    try:
        for X, y, ds in (big, small):
            n, d = X.shape
            w = dev(0.4 * rng.standard_normal(d))
            ds.fun_grad(loss, C, w)
            v = dev(rng.standard_normal(d))
            Hv_a, s_a, Hv_b, s_b = _both(ds, C, v)
            # same kernels, same launch shape, same order of every sum: identical bits
            np.testing.assert_array_equal(Hv_b, Hv_a)
            assert s_b == s_a
            # and both equal the oracle's product
            o = Oracle(n=n, d=d, y=y, X=X)
            _, _, D = o.fun_grad(loss, C, w.cpu().numpy())
            Hv_o = o.hv(C, D, v.cpu().numpy())
            assert_vec_close(Hv_b, Hv_o, what="Hv (static work space)")
            assert_scalar_close(s_b, float(v.cpu().numpy() @ Hv_o), what="v.Hv (static work space)")
        # back to the big one: results unchanged after the small call overwrote part of the array
        X, y, ds = big
        v = dev(rng.standard_normal(24))
        Hv_a, s_a, Hv_b, s_b = _both(ds, C, v)
        np.testing.assert_array_equal(Hv_b, Hv_a)
        assert s_b == s_a
        # without the scalar output
        torch = torch_mod()
        Hv_c = torch.empty_like(v)
        ds.hv_static(C, v, Hv_c, None)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(Hv_c.cpu().numpy(), Hv_a)
    finally:
        big[2].close()
        small[2].close()


def test_static_hv_skips_inactive_rows_like_hv():
    # L2-SVM with most rows inactive: the row-skipping variant of the pass
    rng = np.random.default_rng(5)
    n, d, C = 200_000, 24, 1.0
    X = rng.standard_normal((n, d))
    wt = rng.standard_normal(d)
    y = np.where(X @ wt >= 0, 1.0, -1.0)
    ds = tron.Dataset.from_dense(X, y)
    try:
        w = dev(3.0 * wt)
        ds.fun_grad(LOSS_L2SVM, C, w)
        v = dev(rng.standard_normal(d))
        Hv_a, s_a, Hv_b, s_b = _both(ds, C, v)
        np.testing.assert_array_equal(Hv_b, Hv_a)
        assert s_b == s_a
    finally:
        ds.close()


def test_static_hv_rejects_what_does_not_fit_and_wrong_state():
    rng = np.random.default_rng(9)
    torch = torch_mod()
    X, y, ds = _handle(rng, 70_000, 160)          # 160 columns x 2048 workgroups > 262144 doubles
    try:
        assert tron.tron_dataset_stat(ds.handle, "dense_grid") * 160 + 161 > 262144
        v = dev(rng.standard_normal(160)); Hv = torch.empty_like(v)
        with pytest.raises(tron.TronError) as e:
            ds.hv_static(1.0, v, Hv)              # no D cached yet
        assert e.value.code == -4
        ds.fun_grad(LOSS_LR, 1.0, v)
        with pytest.raises(tron.TronError) as e:
            ds.hv_static(1.0, v, Hv)
        assert e.value.code == -1 and "work space" in str(e.value)
        ds.hv(1.0, v, Hv)                         # the allocating entry point still serves it
    finally:
        ds.close()
    # sparse handles are refused
    rp = np.arange(0, 11, dtype=np.int64); col = np.arange(10, dtype=np.int32) % 4; val = np.ones(10)
    sp = tron.Dataset.from_csr(10, 4, rp, col, val, np.ones(10))
    try:
        v = dev(np.ones(4)); Hv = torch.empty_like(v)
        sp.fun_grad(LOSS_LR, 1.0, v)
        with pytest.raises(tron.TronError) as e:
            sp.hv_static(1.0, v, Hv)
        assert e.value.code == -1
    finally:
        sp.close()
