"""GPU parity: every call goes through the C ABI and is compared with the CPU oracle
element by element (norm-wise 1e-10 per call; objective 1e-8 and identical trajectory per solve)."""
import numpy as np
import pytest

import datagen as dg
from datagen import DenseProblem, SparseProblem
from oracle import LOSS_LR, LOSS_L2SVM

pytestmark = pytest.mark.gpu

from util import check_calls, compare_solves, dev, torch_mod  # noqa: E402


def _dense(rng, n, d, name="rand"):
    X = rng.standard_normal((n, d))
    y = np.where(rng.random(n) < 0.5, 1.0, -1.0)
    return DenseProblem(name, n, d, X, y)


def _csr_from_dense(X, y, name="rand"):
    n, d = X.shape
    rowptr = np.zeros(n + 1, dtype=np.int64)
    rowptr[1:] = np.cumsum((X != 0).sum(axis=1))
    rr, cc = np.nonzero(X)
    return SparseProblem(name, n, d, rowptr, cc.astype(np.int32), X[rr, cc].copy(), y)


# ------------------------------------------------------------------ dense layout
@pytest.mark.parametrize("loss", [LOSS_LR, LOSS_L2SVM])
@pytest.mark.parametrize("n,d", [(1000, 24), (4097, 24), (777, 18), (513, 7), (300, 1), (64, 8), (1025, 33),
                                 (2050, 28), (999, 32), (515, 100), (130, 257), (70, 512), (1, 24), (63, 5)])
def test_dense_calls(rng, loss, n, d):
    check_calls(_dense(rng, n, d), loss, 0.7, rng, w_scale=0.5 / np.sqrt(d))


@pytest.mark.parametrize("loss", [LOSS_LR, LOSS_L2SVM])
def test_dense_many_tiles_ragged_tail(rng, loss):
    # more wave tiles than resident wavefronts (grid-stride loop taken several times) + ragged tail
    p = dg.config4(n=700_001)
    check_calls(p, loss, p.C, rng, w_scale=0.05, n_hv=1)


def test_dense_svm_mostly_inactive_rows(rng):
    # separable data and a long w along the separating direction: most rows (and many whole 64-row tiles) leave the
    # active set, so the Hessian-vector pass skips them; a second w leaves (almost) no active row (Hv ~ v)
    import paper_2008_03433_amd as tron
    from oracle import Oracle
    torch = torch_mod()
    n, d = 40_000, 24
    y = np.where(rng.random(n) < 0.5, 1.0, -1.0)
    u = rng.standard_normal(d); u /= np.linalg.norm(u)
    X = rng.standard_normal((n, d)) + 4.0 * y[:, None] * u[None, :]
    X[5000:9000] = np.abs(X[5000:9000]) * 0 + 6.0 * y[5000:9000, None] * u[None, :]   # a run of rows far inside their class
    p = DenseProblem("separable", n, d, X, y)
    o = Oracle.from_problem(p)
    ds = tron.Dataset.from_problem(p)
    try:
        for scale in (0.4, 50.0):
            w = scale * u
            f_o, g_o, D_o = o.fun_grad(LOSS_L2SVM, 0.5, w)
            frac = float(np.mean(D_o != 0.0))
            assert (0.0 < frac < 0.5) if scale < 1 else frac < 1e-3
            assert not D_o[5000:9000].any()          # whole tiles without an active row
            g_d = torch.empty(d, dtype=torch.float64, device="cuda")
            f_g = ds.fun_grad(LOSS_L2SVM, 0.5, dev(w), g_d)
            assert abs(f_g - f_o) <= 1e-10 * abs(f_o)
            v = rng.standard_normal(d)
            Hv_d = torch.empty(d, dtype=torch.float64, device="cuda")
            vHv = ds.hv(0.5, dev(v), Hv_d)
            Hv_o = o.hv(0.5, D_o, v)
            assert np.linalg.norm(Hv_d.cpu().numpy() - Hv_o) <= 1e-10 * np.linalg.norm(Hv_o)
            assert abs(vHv - v @ Hv_o) <= 1e-10 * abs(v @ Hv_o)
            hd = torch.empty(d, dtype=torch.float64, device="cuda")
            ds.hess_diag(0.5, hd)
            assert np.linalg.norm(hd.cpu().numpy() - o.hess_diag(0.5, D_o)) <= 1e-10 * np.linalg.norm(o.hess_diag(0.5, D_o))
    finally:
        ds.close()


# ------------------------------------------------------------------ CSR layout
@pytest.mark.parametrize("loss", [LOSS_LR, LOSS_L2SVM])
def test_csr_config1(rng, loss):
    check_calls(dg.config1(), loss, 1.0, rng, w_scale=1.0)


@pytest.mark.parametrize("loss", [LOSS_LR, LOSS_L2SVM])
def test_csr_zipf_skew(rng, loss):
    # Zipf columns: the transposed copy has rows spanning many chunks next to empty ones
    check_calls(dg.config2(), loss, 1.0, rng, w_scale=1.0)


def test_csr_url_shape_small(rng):
    p = dg.config3(scale=0.02)
    check_calls(p, LOSS_LR, 1.0, rng, w_scale=1.0, n_hv=1)
    check_calls(p, LOSS_L2SVM, 1.0, rng, w_scale=0.5, n_hv=1)


@pytest.mark.parametrize("loss", [LOSS_LR, LOSS_L2SVM])
def test_csr_degenerate_shapes(rng, loss):
    # empty rows / columns, one very long row and one very long column, single-entry rows
    n, d = 3000, 5000
    X = rng.standard_normal((n, d)) * (rng.random((n, d)) < 0.002)
    X[5] = rng.standard_normal(d)          # dense row: spans several chunks
    X[:, 17] = rng.standard_normal(n)      # dense column: long row of the transposed copy
    X[100:140] = 0.0                       # run of empty rows
    X[:, 2000:2600] = 0.0                  # run of empty columns
    X[n - 1] = 0.0                         # trailing empty row
    X[:, d - 1] = 0.0                      # trailing empty column
    y = np.where(rng.random(n) < 0.5, 1.0, -1.0)
    check_calls(_csr_from_dense(X, y), loss, 0.5, rng, w_scale=0.2)


@pytest.fixture
def force_partitions():
    import paper_2008_03433_amd as tron
    tron.tron_tuning_set("csr_parts", 8)
    yield
    tron.tron_tuning_set("csr_parts", 0)


@pytest.mark.parametrize("loss", [LOSS_LR, LOSS_L2SVM])
def test_csr_partitioned_layout(rng, loss, force_partitions):
    # the 8-way column-partitioned layout (used for large matrices) forced on small and skewed ones
    check_calls(dg.config2(), loss, 1.0, rng, w_scale=1.0, n_hv=1)
    n, d = 3000, 5000
    X = rng.standard_normal((n, d)) * (rng.random((n, d)) < 0.002)
    X[5] = rng.standard_normal(d)
    X[:, 17] = rng.standard_normal(n)
    X[100:140] = 0.0
    X[:, 2000:2600] = 0.0
    X[n - 1] = 0.0
    X[:, d - 1] = 0.0
    y = np.where(rng.random(n) < 0.5, 1.0, -1.0)
    check_calls(_csr_from_dense(X, y), loss, 0.5, rng, w_scale=0.2, n_hv=1)
    # fewer columns than partitions, and an all-zero matrix
    X = rng.standard_normal((50, 3))
    check_calls(_csr_from_dense(X, np.where(rng.random(50) < 0.5, 1.0, -1.0)), loss, 1.0, rng, n_hv=1)
    p = SparseProblem("empty", 3, 4, np.zeros(4, dtype=np.int64), np.zeros(0, dtype=np.int32), np.zeros(0),
                      np.array([1.0, -1.0, 1.0]))
    check_calls(p, loss, 1.0, rng, n_hv=1)


@pytest.mark.parametrize("segmented", [0, 1, -1])
@pytest.mark.parametrize("loss", [LOSS_LR, LOSS_L2SVM])
def test_csr_unpartitioned_layouts(rng, loss, segmented):
    """Small matrices: plain CSR (one lane group per row) or row segments with flag bits (scans) in a single range; the
    automatic choice takes the second for the Zipf-skewed transposed copy of config 2 and the first for config 1."""
    import paper_2008_03433_amd as tron
    tron.tron_tuning_set("csr_segmented", segmented)
    try:
        for p, expect_bwd in ((dg.config1(), 0), (dg.config2(), 1)):
            if segmented == -1:
                ds = tron.Dataset.from_problem(p)
                got = (tron.tron_dataset_stat(ds.handle, "fwd_segmented"), tron.tron_dataset_stat(ds.handle, "bwd_segmented"))
                ds.close()
                assert got[1] == expect_bwd, (p.name, got)
            check_calls(p, loss, 1.0, rng, w_scale=1.0, n_hv=1)
        n, d = 3000, 5000
        X = rng.standard_normal((n, d)) * (rng.random((n, d)) < 0.002)
        X[5] = rng.standard_normal(d)          # rows and columns longer than a chunk
        X[:, 17] = rng.standard_normal(n)
        X[100:140] = 0.0
        X[:, 2000:2600] = 0.0
        X[n - 1] = 0.0
        X[:, d - 1] = 0.0
        y = np.where(rng.random(n) < 0.5, 1.0, -1.0)
        check_calls(_csr_from_dense(X, y), loss, 0.5, rng, w_scale=0.2, n_hv=1)
        X = rng.standard_normal((50, 3))
        check_calls(_csr_from_dense(X, np.where(rng.random(50) < 0.5, 1.0, -1.0)), loss, 1.0, rng, n_hv=1)
        e = SparseProblem("empty", 3, 4, np.zeros(4, dtype=np.int64), np.zeros(0, dtype=np.int32), np.zeros(0),
                          np.array([1.0, -1.0, 1.0]))
        check_calls(e, loss, 1.0, rng, n_hv=1)
        if segmented == 1:
            p = dg.config2()
            compare_solves(p, p.loss, p.C, p.eps)
            compare_solves(p, p.loss, p.C, p.eps, precond_blend=0.01)
    finally:
        tron.tron_tuning_set("csr_segmented", -1)


@pytest.mark.parametrize("knobs", [{"csr_head": 0}, {"csr_hot": 0}, {"csr_tiles": 0}, {"csr_range_slots": 64}, {"csr_unit": 0}, {"csr_sell": 0},
                                   {"csr_sell_blocks": 1},
                                   {"csr_unit": 0, "csr_head": 0, "csr_tiles": 0},
                                   {"csr_blocks_per_part": 3, "csr_range_blocks_per_part": 2, "csr_hot_blocks_per_part": 1,
                                    "csr_tile_blocks_per_slice": 2}])
def test_csr_layout_variants(rng, force_partitions, knobs):
    # every building block of the partitioned layout switched off or shrunk in turn: the ranges without the head
    # partition, no LDS tables, no hot-row tiles, tiny tables, very few persistent workgroups (many chunks each)
    import paper_2008_03433_amd as tron
    # (config 3 has one value per instance: its layouts keep no value stream unless csr_unit = 0; config 2 has free values)
    defaults = {"csr_head": 1, "csr_hot": 1, "csr_tiles": 1, "csr_range_slots": 4096, "csr_unit": 1, "csr_sell": 1, "csr_sell_blocks": 1024, "csr_blocks_per_part": 128,
                "csr_range_blocks_per_part": 96, "csr_hot_blocks_per_part": 96, "csr_tile_blocks_per_slice": 0}
    try:
        for k, v in knobs.items():
            tron.tron_tuning_set(k, v)
        check_calls(dg.config2(), LOSS_LR, 1.0, rng, w_scale=1.0, n_hv=1)
        p = dg.config3(scale=0.02)
        check_calls(p, LOSS_L2SVM, 1.0, rng, w_scale=0.5, n_hv=1)
    finally:
        for k in knobs:
            tron.tron_tuning_set(k, defaults[k])


@pytest.mark.parametrize("loss", [LOSS_LR, LOSS_L2SVM])
def test_csr_one_value_per_instance(rng, loss, force_partitions):
    """Matrices X = diag(r) B with B binary: the partitioned layouts keep no values ("unit_values" = 1); a single
    differing entry switches back to the layouts with values.  Same results either way (to rounding)."""
    import paper_2008_03433_amd as tron
    n, d = 4000, 6000
    B = (rng.random((n, d)) < 0.004).astype(np.float64)
    B[7] = 1.0                      # a full row
    B[:, 11] = 1.0                  # a full column
    B[200:260] = 0.0                # empty rows
    B[:, 3000:3500] = 0.0           # empty columns
    r = np.exp(rng.standard_normal(n))
    r[::5] = 1.0
    r[3] = -0.75                    # the shared value may be negative
    y = np.where(rng.random(n) < 0.5, 1.0, -1.0)
    p = _csr_from_dense(B * r[:, None], y)
    ds = tron.Dataset.from_problem(p)
    assert tron.tron_dataset_stat(ds.handle, "unit_values") == 1
    ds.close()
    check_calls(p, loss, 0.5, rng, w_scale=0.3, n_hv=2)
    # a solve on binary features normalised to unit length (r_i = 1 / sqrt(number of entries)); the rounding differs
    # from the oracle's (r_i times a sum instead of a sum of products), intermediate iterates agree to 1e-6
    Bn = (rng.random((n, d)) < 0.004).astype(np.float64)
    Bn[:, 11] = 1.0
    pn = _csr_from_dense(Bn / np.sqrt(Bn.sum(axis=1))[:, None], y)
    compare_solves(pn, loss, 1.0, 1e-4, trace_rel=1e-6)
    # many instances, few features: a tile of the transposed product fills up slowly, so the limit on the columns it may
    # span (they are copied into LDS) closes it first
    nt, dt = 20000, 300
    Bt = (rng.random((nt, dt)) < 0.05).astype(np.float64)
    Bt[:, 5] = 1.0
    pt = _csr_from_dense(Bt * np.exp(rng.standard_normal(nt))[:, None], np.where(rng.random(nt) < 0.5, 1.0, -1.0))
    ds = tron.Dataset.from_problem(pt)
    assert tron.tron_dataset_stat(ds.handle, "unit_values") == 1
    tiles, tile_nnz = tron.tron_dataset_stat(ds.handle, "bwd_tiles"), tron.tron_dataset_stat(ds.handle, "bwd_tile_nnz")
    ds.close()
    assert tiles > 0 and tile_nnz / tiles < 0.8 * 2048, (tiles, tile_nnz)   # not filled: closed by the span limit
    check_calls(pt, loss, 0.5, rng, w_scale=0.3, n_hv=2)
    X2 = B * r[:, None]
    X2[7, 5] *= 1.5
    p2 = _csr_from_dense(X2, y)
    ds = tron.Dataset.from_problem(p2)
    assert tron.tron_dataset_stat(ds.handle, "unit_values") == 0
    ds.close()
    check_calls(p2, loss, 0.5, rng, w_scale=0.3, n_hv=1)
    tron.tron_tuning_set("csr_unit", 0)
    try:
        ds = tron.Dataset.from_problem(p)
        assert tron.tron_dataset_stat(ds.handle, "unit_values") == 0
        ds.close()
        check_calls(p, loss, 0.5, rng, w_scale=0.3, n_hv=1)
    finally:
        tron.tron_tuning_set("csr_unit", 1)


def test_hot_row_tiles_are_left_out_when_they_would_stay_nearly_empty(rng, force_partitions):
    """Many instances, every feature equally rare: a tile may span 512 instances only, so the tiles of such a matrix
    would hold a few entries each and cost more than they save; the features stay in the transposed CSR copy."""
    import paper_2008_03433_amd as tron
    n, d, nnz = 300_000, 2000, 90_000
    keys = np.unique(rng.integers(0, n * d, size=nnz))
    rows, cols = keys // d, (keys % d).astype(np.int32)      # sorted by (row, column)
    rowptr = np.zeros(n + 1, dtype=np.int64)
    np.add.at(rowptr, rows + 1, 1)
    rowptr = np.cumsum(rowptr)
    p = SparseProblem("flat", n, d, rowptr, cols, rng.standard_normal(len(keys)),
                      np.where(rng.random(n) < 0.5, 1.0, -1.0))
    ds = tron.Dataset.from_problem(p)
    assert tron.tron_dataset_stat(ds.handle, "bwd_parts") == 8
    assert tron.tron_dataset_stat(ds.handle, "bwd_tiles") == 0
    ds.close()
    check_calls(p, LOSS_LR, 0.5, rng, w_scale=0.3, n_hv=1)


def test_solve_partitioned_layout(force_partitions):
    p = dg.config2()
    compare_solves(p, p.loss, p.C, p.eps)
    p = dg.config1()
    compare_solves(p, p.loss, p.C, p.eps)


def test_solve_url_shape_scaled(force_partitions):
    # url-shaped workload: per-call parity is 1e-10, but CG amplifies rounding on this matrix (the oracle's own
    # plain-fp64 twin departs from it by ~1e-5 in f at eps = 0.01, see tests/test_oracle_pins.py), so solve-level
    # parity is: same history while the histories agree, both end within the strong-convexity bound, and the
    # objectives agree to 1e-8 once eps is tight.
    import paper_2008_03433_amd as tron
    from oracle import Oracle
    torch = torch_mod()
    p = dg.config3(scale=0.1)
    o = Oracle.from_problem(p)
    ds = tron.Dataset.from_problem(p)
    try:
        for eps in (1e-2, 1e-6):
            ref = o.tron(p.loss, p.C, eps)
            w = torch.zeros(p.d, dtype=torch.float64, device="cuda")
            res = ds.solve(p.loss, p.C, eps, w)
            assert res.converged and ref.converged
            assert abs(res.gnorm0 - ref.gnorm0) <= 1e-10 * ref.gnorm0
            for a, b in list(zip(res.trace, ref.trace))[:3]:
                assert (a["cg_iters"], a["accepted"]) == (b["cg_iters"], b["accepted"])
                assert abs(a["f"] - b["f"]) <= 1e-8 * abs(b["f"])
            assert abs(res.f - ref.f) <= 0.5 * (eps * ref.gnorm0) ** 2
            f_chk, g_chk, _ = o.fun_grad(p.loss, p.C, w.cpu().numpy())
            assert abs(f_chk - res.f) <= 1e-10 * abs(f_chk)
            assert np.linalg.norm(g_chk) <= eps * ref.gnorm0 * (1 + 1e-9)
            if eps == 1e-6:
                assert abs(res.f - ref.f) <= 1e-8 * abs(ref.f)
    finally:
        ds.close()


def test_csr_url_shape_partitioned(rng):
    # large enough that the automatic choice partitions both orientations
    import paper_2008_03433_amd as tron
    p = dg.config3(scale=0.1)
    assert p.nnz > (1 << 22) and p.n * 8 > (3 << 19)
    check_calls(p, LOSS_LR, 1.0, rng, w_scale=1.0, n_hv=1)
    # ... and that every building block of the regrouped layout took part
    ds = tron.Dataset.from_problem(p)
    try:
        st = {k: tron.tron_dataset_stat(ds.handle, k) for k in ("fwd_parts", "bwd_parts", "fwd_csr_nnz", "fwd_head_nnz",
                                                                 "fwd_lds_columns", "bwd_csr_nnz", "bwd_tile_nnz", "bwd_tile_rows", "unit_values")}
        assert st["fwd_parts"] == 8 and st["bwd_parts"] == 8
        assert st["unit_values"] == 1                            # one value per instance: no value stream
        assert st["fwd_csr_nnz"] == p.nnz and 0.25 * p.nnz <= st["fwd_head_nnz"] < p.nnz
        assert st["fwd_lds_columns"] > 4096                      # head table + range tables
        assert st["bwd_csr_nnz"] + st["bwd_tile_nnz"] == p.nnz and st["bwd_tile_rows"] > 0 and st["bwd_csr_nnz"] > 0
    finally:
        ds.close()


def test_csr_tiny_and_empty(rng):
    # nnz = 0, and a 1 x 1 matrix
    y = np.array([1.0, -1.0, 1.0])
    p = SparseProblem("empty", 3, 4, np.zeros(4, dtype=np.int64), np.zeros(0, dtype=np.int32), np.zeros(0), y)
    check_calls(p, LOSS_LR, 1.0, rng)
    p = SparseProblem("one", 1, 1, np.array([0, 1], dtype=np.int64), np.array([0], dtype=np.int32), np.array([2.0]),
                      np.array([-1.0]))
    check_calls(p, LOSS_L2SVM, 1.0, rng)


def test_csr_exact_chunk_multiple(rng):
    # nnz an exact multiple of the 2048-nonzero chunk, last rows empty
    n, d, per = 130, 64, 32
    X = np.zeros((n, d))
    for i in range(128):
        X[i, rng.choice(d, per, replace=False)] = rng.standard_normal(per)
    y = np.where(rng.random(n) < 0.5, 1.0, -1.0)
    p = _csr_from_dense(X, y)
    assert p.nnz == 4096
    check_calls(p, LOSS_LR, 1.0, rng)


def test_csr_matches_dense_layout(rng):
    torch = torch_mod()
    import paper_2008_03433_amd as tron
    n, d = 1500, 24
    X = rng.standard_normal((n, d)) * (rng.random((n, d)) < 0.5)
    y = np.where(rng.random(n) < 0.5, 1.0, -1.0)
    a = tron.Dataset.from_problem(DenseProblem("d", n, d, X, y))
    b = tron.Dataset.from_problem(_csr_from_dense(X, y))
    w = dev(0.2 * rng.standard_normal(d)); v = dev(rng.standard_normal(d))
    ga, gb, Ha, Hb = (torch.empty(d, dtype=torch.float64, device="cuda") for _ in range(4))
    for loss in (LOSS_LR, LOSS_L2SVM):
        fa, fb = a.fun_grad(loss, 1.0, w, ga), b.fun_grad(loss, 1.0, w, gb)
        assert abs(fa - fb) <= 1e-13 * abs(fa)
        np.testing.assert_allclose(ga.cpu().numpy(), gb.cpu().numpy(), rtol=1e-12, atol=1e-12)
        a.hv(1.0, v, Ha); b.hv(1.0, v, Hb)
        np.testing.assert_allclose(Ha.cpu().numpy(), Hb.cpu().numpy(), rtol=1e-12, atol=1e-12)
    a.close(); b.close()


# ------------------------------------------------------------------ special values
def test_svm_ties_and_extreme_margins(rng):
    torch = torch_mod()
    import paper_2008_03433_amd as tron
    from oracle import Oracle
    # exactly representable margins: y z == 1 must be inactive on both sides
    X = np.array([[1.0, 0.0], [-1.0, 0.0], [0.5, 0.0], [0.0, 1.0]])
    y = np.array([1.0, -1.0, 1.0, -1.0])
    p = DenseProblem("ties", 4, 2, X, y)
    o = Oracle.from_problem(p)
    ds = tron.Dataset.from_problem(p)
    w = np.array([1.0, 3.0])
    g = torch.empty(2, dtype=torch.float64, device="cuda")
    f = ds.fun_grad(LOSS_L2SVM, 1.0, dev(w), g)
    fo, go, Do = o.fun_grad(LOSS_L2SVM, 1.0, w)
    assert f == fo and np.array_equal(g.cpu().numpy(), go)
    v = np.array([1.0, 1.0]); Hv = torch.empty_like(g)
    ds.hv(1.0, dev(v), Hv)
    assert np.array_equal(Hv.cpu().numpy(), o.hv(1.0, Do, v))
    ds.close()
    # logistic loss at |y z| up to 700: finite, matches the oracle
    X = np.array([[700.0], [-700.0], [40.0], [-40.0], [1e-9], [0.0]])
    y = np.array([1.0, 1.0, -1.0, -1.0, 1.0, -1.0])
    check_calls(DenseProblem("big", 6, 1, X, y), LOSS_LR, 1.0, rng, w_scale=0.0)
    p = DenseProblem("big", 6, 1, X, y)
    ds = tron.Dataset.from_problem(p)
    f = ds.fun_grad(LOSS_LR, 1.0, dev(np.array([1.0])), g[:1])
    fo, go, _ = Oracle.from_problem(p).fun_grad(LOSS_LR, 1.0, np.array([1.0]))
    assert abs(f - fo) <= 1e-12 * abs(fo) and np.isfinite(g[:1].cpu().numpy()).all()
    ds.close()


# ------------------------------------------------------------------ determinism / state
def test_repeated_calls_are_bitwise_identical(rng):
    torch = torch_mod()
    import paper_2008_03433_amd as tron
    for p in (dg.config2(), dg.config4(n=50_000)):
        ds = tron.Dataset.from_problem(p)
        w = dev(0.1 * rng.standard_normal(p.d)); v = dev(rng.standard_normal(p.d))
        g1, g2, H1, H2 = (torch.empty(p.d, dtype=torch.float64, device="cuda") for _ in range(4))
        f1 = ds.fun_grad(p.loss, p.C, w, g1); q1 = ds.hv(p.C, v, H1)
        f2 = ds.fun_grad(p.loss, p.C, w, g2); q2 = ds.hv(p.C, v, H2)
        assert f1 == f2 and q1 == q2
        assert torch.equal(g1, g2) and torch.equal(H1, H2)
        ds.close()


def test_hv_requires_fun_grad(rng):
    torch = torch_mod()
    import paper_2008_03433_amd as tron
    ds = tron.Dataset.from_problem(_dense(rng, 100, 4))
    v = dev(np.ones(4)); Hv = torch.empty_like(v)
    with pytest.raises(tron.TronError) as e:
        ds.hv(1.0, v, Hv)
    assert e.value.code == -4
    with pytest.raises(tron.TronError) as e:
        ds.fun_grad(LOSS_LR, -1.0, v)
    assert e.value.code == -1
    ds.close()


def test_invalid_inputs_are_rejected(rng):
    import paper_2008_03433_amd as tron
    y = np.array([1.0, -1.0])
    bad = [
        (np.array([0, 2, 1], dtype=np.int64), np.array([0, 1], dtype=np.int32), np.ones(2), y),      # rowptr decreases
        (np.array([0, 2, 2], dtype=np.int64), np.array([1, 0], dtype=np.int32), np.ones(2), y),      # unsorted columns
        (np.array([0, 2, 2], dtype=np.int64), np.array([0, 0], dtype=np.int32), np.ones(2), y),      # duplicate column
        (np.array([0, 1, 2], dtype=np.int64), np.array([0, 3], dtype=np.int32), np.ones(2), y),      # column out of range
        (np.array([0, 1, 2], dtype=np.int64), np.array([0, 1], dtype=np.int32), np.array([1.0, np.nan]), y),
        (np.array([0, 1, 2], dtype=np.int64), np.array([0, 1], dtype=np.int32), np.ones(2), np.array([1.0, 0.0])),
    ]
    for rowptr, col, val, yy in bad:
        with pytest.raises(tron.TronError) as e:
            tron.tron_dataset_create_csr(2, 3, rowptr, col, val, yy)
        assert e.value.code == -1
    with pytest.raises(tron.TronError):
        tron.tron_dataset_create_dense(2, 2, np.array([[1.0, np.inf], [0.0, 1.0]]), y)
    with pytest.raises(tron.TronError):
        tron.tron_dataset_create_dense(2, 600, np.zeros((2, 600)), y)


def test_invalid_dense_input_in_device_memory_is_rejected(rng):
    """Rows handed over as device pointers get the checks host input gets: labels exactly +1 / -1, finite entries."""
    import paper_2008_03433_amd as tron
    torch = torch_mod()
    n, d = 5000, 7
    X = rng.standard_normal((n, d))
    y = np.where(rng.random(n) < 0.5, 1.0, -1.0)
    for bad_y in (0.0, 0.5, 2.0, np.nan, -np.inf):
        yy = y.copy(); yy[n - 3] = bad_y
        with pytest.raises(tron.TronError) as e:
            tron.tron_dataset_create_dense(n, d, dev(X), dev(yy))
        assert e.value.code == -1 and "label" in str(e.value)
    for bad_x in (np.nan, np.inf, -np.inf):
        XX = X.copy(); XX[n - 1, d - 1] = bad_x
        with pytest.raises(tron.TronError) as e:
            tron.tron_dataset_create_dense(n, d, dev(XX), dev(y))
        assert e.value.code == -1 and "finite" in str(e.value)
    # a rejected chunk leaves the rows already written alone; a good chunk still goes through afterwards
    h = tron.tron_dataset_create_dense_empty(n, d)
    try:
        tron.tron_dataset_write_rows(h, 0, n, dev(X), dev(y))
        yy = y[:100].copy(); yy[5] = 0.0
        with pytest.raises(tron.TronError):
            tron.tron_dataset_write_rows(h, 0, 100, dev(np.zeros((100, d))), dev(yy))
        w = dev(0.1 * rng.standard_normal(d))
        f = tron.tron_fun_grad(h, LOSS_LR, 1.0, w, None)
        f_o, _, _ = __import__("oracle").Oracle(n=n, d=d, y=y, X=X).fun_grad(LOSS_LR, 1.0, w.cpu().numpy())
        assert abs(f - f_o) <= 1e-10 * abs(f_o)
    finally:
        tron.tron_dataset_destroy(h)


# ------------------------------------------------------------------ full solves
def test_solve_config1():
    p = dg.config1()
    compare_solves(p, p.loss, p.C, p.eps)


def test_solve_config2():
    p = dg.config2()
    res, ref = compare_solves(p, p.loss, p.C, p.eps)
    assert res.cg_iters_total > 10


@pytest.mark.parametrize("fuse", [0, 1])
def test_reductions_finished_in_kernel_or_by_a_launch_agree_bit_for_bit(rng, fuse):
    """The second stage of the reductions -- inside the producing kernel (last workgroup) or as a launch of its own -- adds
    the same partial sums in the same order: identical scalars, identical trajectories."""
    import paper_2008_03433_amd as tron
    torch = torch_mod()
    out = {}
    for knob in (fuse, 1 - fuse):
        tron.tron_tuning_set("fuse_reductions", knob)
        try:
            for p in (dg.config2(), dg.config4(n=50_000)):
                tron.tron_tuning_set("dense_device_driver", 0)
                ds = tron.Dataset.from_problem(p)
                w = torch.zeros(p.d, dtype=torch.float64, device="cuda")
                res = ds.solve(p.loss, p.C, 1e-4, w, precond_blend=0.01 if fuse else 0.0)
                v = torch.ones(p.d, dtype=torch.float64, device="cuda"); Hv = torch.empty_like(v)
                vHv = ds.hv(p.C, v, Hv)
                f = ds.fun_grad(p.loss, p.C, w, Hv)
                ds.close()
                out.setdefault(p.name, []).append((res.f, res.gnorm, res.cg_iters_total, [t["f"] for t in res.trace], vHv, f,
                                                   w.cpu().numpy().tobytes()))
        finally:
            tron.tron_tuning_set("fuse_reductions", -1)
            tron.tron_tuning_set("dense_device_driver", -1)
    for name, (a, b) in out.items():
        assert a == b, name


def test_solve_config2_svm_loss():
    # Off-config stress: H = I + X^T X has a well separated top eigenvalue (~2e3, the Zipf head feature), so CG
    # iterates are sensitive to rounding (plain-fp64 numpy CG departs from the long-double oracle by ~4e-7 in s
    # after 10 iterations, ~2e-5 in f by the second outer iteration, and a CG stopping test can flip).  So at
    # eps = 1e-3 only what the mathematics fixes is compared -- the first outer iteration, convergence, and the
    # objectives to 1e-6 -- and at eps = 1e-8, where both sit on the minimiser, the objectives to 1e-8.
    import paper_2008_03433_amd as tron
    from oracle import Oracle
    torch = torch_mod()
    p = dg.config2()
    o = Oracle.from_problem(p)
    ds = tron.Dataset.from_problem(p)
    try:
        for eps, tol in ((1e-3, 1e-6), (1e-8, 1e-8)):
            ref = o.tron(LOSS_L2SVM, 0.5, eps)
            w = torch.zeros(p.d, dtype=torch.float64, device="cuda")
            res = ds.solve(LOSS_L2SVM, 0.5, eps, w)
            assert res.converged and ref.converged
            a, b = res.trace[0], ref.trace[0]
            assert (a["cg_iters"], a["accepted"]) == (b["cg_iters"], b["accepted"])
            assert abs(a["f"] - b["f"]) <= 1e-5 * abs(b["f"])
            assert abs(res.f - ref.f) <= tol * abs(ref.f)
            f_chk, g_chk, _ = o.fun_grad(LOSS_L2SVM, 0.5, w.cpu().numpy())
            assert abs(f_chk - res.f) <= 1e-10 * abs(f_chk)
            assert np.linalg.norm(g_chk) <= eps * ref.gnorm0 * (1 + 1e-9)
    finally:
        ds.close()


@pytest.fixture(params=[0, 1], ids=["host_driver", "device_driver"])
def dense_driver(request):
    """tron_solve on dense matrices with d <= 32: trust-region / CG steps on the host (scalars read back every iteration)
    or on the device (the multi-problem machinery with one problem over all rows)."""
    import paper_2008_03433_amd as tron
    tron.tron_tuning_set("dense_device_driver", request.param)
    yield request.param
    tron.tron_tuning_set("dense_device_driver", -1)


def test_solve_config4_reduced(dense_driver):
    p = dg.config4(n=200_000)
    compare_solves(p, p.loss, p.C, p.eps)
    compare_solves(p, LOSS_LR, 1e-3, 1e-4)


def test_solve_dense_lr_tight(rng, dense_driver):
    p = _dense(rng, 5000, 18)
    compare_solves(p, LOSS_LR, 2.0, 1e-6)
    compare_solves(p, LOSS_L2SVM, 0.5, 1e-6)


def test_solve_hits_trust_region_boundary(rng):
    # far-away start with saturated sigmoids: the quadratic model is poor, steps get rejected, the
    # radius shrinks and CG ends on the boundary (H >= I means the very first step from Delta_0 = |g|
    # can never be on the boundary)
    rng = np.random.default_rng(5)
    n, d = 2000, 40
    X = 3.0 * rng.standard_normal((n, d)) * (rng.random((n, d)) < 0.3)
    y = np.where(rng.random(n) < 0.5, 1.0, -1.0)
    w0 = 3.0 * rng.standard_normal(d)
    for p in (_csr_from_dense(X, y), DenseProblem("far", n, d, X, y)):
        res, ref = compare_solves(p, LOSS_LR, 50.0, 1e-4, w0=w0)
        assert sum(t["on_boundary"] for t in ref.trace) >= 5
        assert sum(1 - t["accepted"] for t in ref.trace) >= 5


@pytest.mark.parametrize("ahead", [0, 1])
def test_cg_iterations_enqueued_ahead_or_one_by_one_take_the_same_path(rng, ahead):
    """The host-driven CG loop either waits for an iteration's scalars before enqueuing the next iteration, or enqueues
    one iteration ahead and lets the kernels of an iteration that turns out not to exist leave the vectors alone.  Runs
    that end by the residual test, on the trust-region boundary, at the iteration cap, with and without the
    preconditioner, sparse and dense: the oracle's trajectory either way."""
    import paper_2008_03433_amd as tron
    tron.tron_tuning_set("cg_speculate", ahead)
    tron.tron_tuning_set("dense_device_driver", 0)
    try:
        p = dg.config1()
        compare_solves(p, p.loss, p.C, p.eps)
        p = dg.config2()
        compare_solves(p, p.loss, p.C, p.eps)
        compare_solves(p, p.loss, p.C, 1e-4, precond_blend=0.01)
        compare_solves(p, p.loss, p.C, 1e-3, max_cg=3)       # every run cut at three iterations
        compare_solves(p, p.loss, p.C, 1e-3, max_cg=1)
        q = _dense(rng, 5000, 18)
        compare_solves(q, LOSS_LR, 2.0, 1e-6)
        compare_solves(q, LOSS_L2SVM, 0.5, 1e-6, precond_blend=0.5)
        far = np.random.default_rng(5)
        n, d = 2000, 40
        X = 3.0 * far.standard_normal((n, d)) * (far.random((n, d)) < 0.3)
        y = np.where(far.random(n) < 0.5, 1.0, -1.0)
        w0 = 3.0 * far.standard_normal(d)
        for pb in (_csr_from_dense(X, y), DenseProblem("far", n, d, X, y)):
            res, ref = compare_solves(pb, LOSS_LR, 50.0, 1e-4, w0=w0)
            assert sum(t["on_boundary"] for t in ref.trace) >= 5
    finally:
        tron.tron_tuning_set("cg_speculate", -1)
        tron.tron_tuning_set("dense_device_driver", -1)


def test_solve_warm_start_and_iteration_cap(rng, dense_driver):
    torch = torch_mod()
    import paper_2008_03433_amd as tron
    from oracle import Oracle
    p = _dense(rng, 3000, 12)
    o = Oracle.from_problem(p)
    ds = tron.Dataset.from_problem(p)
    w = torch.zeros(p.d, dtype=torch.float64, device="cuda")
    r1 = ds.solve(LOSS_LR, 5.0, 1e-10, w, max_outer=2)
    ref1 = o.tron(LOSS_LR, 5.0, 1e-10, max_outer=2)
    assert r1.status == 1 and ref1.status == 1 and r1.outer_iters == 2
    assert abs(r1.f - ref1.f) <= 1e-8 * abs(ref1.f)
    # continue from the iterate (w0 != 0: the stopping reference is still |grad f(0)|)
    r2 = ds.solve(LOSS_LR, 5.0, 1e-6, w)
    ref2 = o.tron(LOSS_LR, 5.0, 1e-6, w0=ref1.w)
    assert r2.converged and ref2.converged
    assert abs(r2.gnorm0 - ref2.gnorm0) <= 1e-10 * ref2.gnorm0
    assert r2.outer_iters == ref2.outer_iters
    assert abs(r2.f - ref2.f) <= 1e-8 * abs(ref2.f)
    # tron_hv may follow a solve: D at the final iterate is cached
    v = dev(rng.standard_normal(p.d)); Hv = torch.empty_like(v)
    ds.hv(5.0, v, Hv)
    _, _, D = o.fun_grad(LOSS_LR, 5.0, w.cpu().numpy())
    np.testing.assert_allclose(Hv.cpu().numpy(), o.hv(5.0, D, v.cpu().numpy()), rtol=1e-9, atol=1e-9)
    # the same after an L2-SVM solve (the active set of the final iterate), and the Hessian diagonal
    w2 = torch.zeros(p.d, dtype=torch.float64, device="cuda")
    r3 = ds.solve(LOSS_L2SVM, 0.5, 1e-4, w2)
    assert r3.converged
    ds.hv(0.5, v, Hv)
    _, _, D2 = o.fun_grad(LOSS_L2SVM, 0.5, w2.cpu().numpy())
    np.testing.assert_allclose(Hv.cpu().numpy(), o.hv(0.5, D2, v.cpu().numpy()), rtol=1e-9, atol=1e-9)
    hd = torch.empty_like(v)
    ds.hess_diag(0.5, hd)
    np.testing.assert_allclose(hd.cpu().numpy(), o.hess_diag(0.5, D2), rtol=1e-10)
    ds.close()
