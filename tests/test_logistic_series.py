"""The logistic kernels evaluate log(1 + e), e = exp(-|t|) in [0, 1], by the series 2 atanh(u) = 2 u (1 + u^2/3 + ... +
u^30/31), u = e / (2 + e) (device_util.h: log1p_unit).  This checks the claim made there -- within 2 ulp of the exact
value on that range -- with the same operations in fp64 on the host against numpy's extended-precision log1p.  (The
device path itself is held to the oracle by the GPU parity tests of the objective.)"""
import numpy as np


def series(e):
    u = e / (2.0 + e)
    w = u * u
    p = np.full_like(e, 1.0 / 31.0)
    for k in range(14, -1, -1):
        p = p * w + 1.0 / (2 * k + 1)
    return 2.0 * u * p


def test_series_is_within_two_ulp_on_the_unit_interval():
    rng = np.random.default_rng(2008)
    t = np.concatenate([rng.uniform(0.0, 40.0, 1_000_000), rng.uniform(0.0, 1.0, 300_000), rng.uniform(0.0, 0.01, 100_000),
                        np.array([0.0, 1e-300, 1e-17, 36.0, 37.0, 600.0])])
    e = np.exp(-t)
    assert e.min() > 0.0 and e.max() <= 1.0
    exact = np.log1p(e.astype(np.longdouble))
    rel = np.abs((series(e).astype(np.longdouble) - exact) / exact)
    assert float(rel.max()) <= 2 * np.finfo(np.float64).eps          # 2 ulp = 4.4e-16
    assert float(rel.mean()) <= 1e-16
    # the first term left out, relative to the sum, at the largest u = 1/3
    assert (1.0 / 9.0) ** 16 / 33.0 < 2e-17


def test_series_at_the_ends():
    assert series(np.array([0.0]))[0] == 0.0
    assert abs(series(np.array([1.0]))[0] - np.log(2.0)) <= 2 * np.finfo(np.float64).eps * np.log(2.0)
