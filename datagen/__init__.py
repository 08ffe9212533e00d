"""Seeded synthetic workloads shaped like the paper's datasets (Appendix "Benchmark
Dataset Statistics"): rcv1-/url-shaped sparse matrices for logistic regression and
Kim-/Wilhelm-scale dense matrices for the L2-SVM.

Inputs only: this package holds no loss, gradient, Hessian or trust-region code.
It is the single module shared by the CPU oracle's tests and the GPU path, so both
sides consume the same bytes.  The heavy loops live in ``gen.c`` (counter-based
random numbers, OpenMP); this file is the recipe for each named workload.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, field
from typing import Iterator, Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libdatagen.so")
_SRC = os.path.join(_HERE, "gen.c")

BASE_SEED = 200803433

# stream ids used by the Python-side recipes (gen.c owns 101..203)
_STREAM_WSTAR = 1
_STREAM_NOISE = 2
_STREAM_PERM = 3
_STREAM_MU = 4
_STREAM_WSTAR_MASK = 5


def build(force: bool = False) -> str:
    """Compile gen.c into libdatagen.so (gcc, OpenMP)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-fvisibility=hidden", "-o", _SO, _SRC, "-lm"]
        subprocess.check_call(cmd)
    return _SO


class _Spec(ctypes.Structure):
    _fields_ = [
        ("n", ctypes.c_int64), ("d", ctypes.c_int64),
        ("len_kind", ctypes.c_int), ("len_param", ctypes.c_double), ("len_cap", ctypes.c_int64),
        ("col_kind", ctypes.c_int), ("zipf_s", ctypes.c_double),
        ("val_kind", ctypes.c_int), ("seed", ctypes.c_uint64),
    ]


_lib = None


def _L():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_SO)
        u64, i64, dbl, vp = ctypes.c_uint64, ctypes.c_int64, ctypes.c_double, ctypes.c_void_p
        lib.dg_fill_bits.argtypes = [u64, u64, u64, i64, vp]
        lib.dg_fill_uniform.argtypes = [u64, u64, u64, i64, vp]
        lib.dg_fill_normal.argtypes = [u64, u64, u64, i64, vp]
        lib.dg_dense_rows.argtypes = [u64, i64, i64, i64, vp, dbl, vp, vp, vp, vp]
        lib.dg_sparse_rowptr.argtypes = [ctypes.POINTER(_Spec), vp, vp]
        lib.dg_sparse_rowptr.restype = i64
        lib.dg_sparse_fill.argtypes = [ctypes.POINTER(_Spec), vp, vp, vp, vp]
        lib.dg_csr_scores.argtypes = [i64, vp, vp, vp, vp, vp]
        lib.dg_num_threads.restype = ctypes.c_int
        for f in (lib.dg_fill_bits, lib.dg_fill_uniform, lib.dg_fill_normal, lib.dg_dense_rows,
                  lib.dg_sparse_fill, lib.dg_csr_scores):
            f.restype = None
        _lib = lib
    return _lib


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data


def normals(seed: int, stream: int, count: int, start: int = 0) -> np.ndarray:
    out = np.empty(count, dtype=np.float64)
    _L().dg_fill_normal(seed, stream, start, count, _ptr(out))
    return out


def uniforms(seed: int, stream: int, count: int, start: int = 0) -> np.ndarray:
    out = np.empty(count, dtype=np.float64)
    _L().dg_fill_uniform(seed, stream, start, count, _ptr(out))
    return out


def permutation(seed: int, stream: int, d: int) -> np.ndarray:
    keys = np.empty(d, dtype=np.uint64)
    _L().dg_fill_bits(seed, stream, 0, d, _ptr(keys))
    return np.argsort(keys, kind="stable").astype(np.int32)


# --------------------------------------------------------------------------
# problem containers
# --------------------------------------------------------------------------
LOSS_LR = 0
LOSS_L2SVM = 1


@dataclass
class SparseProblem:
    name: str
    n: int
    d: int
    rowptr: np.ndarray  # int64[n+1]
    col: np.ndarray     # int32[nnz], sorted and distinct inside each row
    val: np.ndarray     # float64[nnz]
    y: np.ndarray       # float64[n], +1/-1
    loss: int = LOSS_LR
    C: float = 1.0
    eps: float = 0.01
    meta: dict = field(default_factory=dict)

    @property
    def nnz(self) -> int:
        return int(self.rowptr[-1])


@dataclass
class DenseProblem:
    name: str
    n: int
    d: int
    X: Optional[np.ndarray]  # float64[n, d] row-major, or None when streamed
    y: Optional[np.ndarray]
    loss: int = LOSS_L2SVM
    C: float = 0.1
    eps: float = 0.01
    meta: dict = field(default_factory=dict)


# --------------------------------------------------------------------------
# sparse recipes
# --------------------------------------------------------------------------
def make_sparse(name: str, n: int, d: int, *, seed: int, len_kind: str, len_param: float, len_cap: int = 0,
                col_kind: str = "zipf", zipf_s: float = 1.1, val_kind: str = "lognormal",
                wstar_density: float = 1.0, noise_std: float = 0.1, noise_relative: bool = False,
                positive_fraction: Optional[float] = None, loss: int = LOSS_LR, C: float = 1.0,
                eps: float = 0.01) -> SparseProblem:
    """Generic sparse recipe.

    Rows: number of column draws from ``len_kind`` in {"const", "poisson", "geometric"}
    (at least 1, capped at ``len_cap``); columns uniform-distinct or Zipf(s) ranks sent
    through a random feature permutation, repeats dropped without top-up; values
    lognormal(0,1) or 1.0; every row scaled to unit 2-norm.
    Labels: sign(x.w* + noise + b), w* ~ N(0,1) on a ``wstar_density`` fraction of the
    features, noise ~ N(0, noise_std^2) (times the sample std of x.w* when
    ``noise_relative``), and b the offset that makes the requested fraction positive
    (b = 0 when ``positive_fraction`` is None).  sign(0) = +1.
    """
    lib = _L()
    spec = _Spec(n=n, d=d,
                 len_kind={"const": 0, "poisson": 1, "geometric": 2}[len_kind],
                 len_param=float(len_param), len_cap=int(len_cap),
                 col_kind={"uniform": 0, "zipf": 1}[col_kind], zipf_s=float(zipf_s),
                 val_kind={"lognormal": 0, "one": 1}[val_kind], seed=seed)
    perm = permutation(seed, _STREAM_PERM, d) if col_kind == "zipf" else None
    rowptr = np.empty(n + 1, dtype=np.int64)
    nnz = lib.dg_sparse_rowptr(ctypes.byref(spec), _ptr(perm), _ptr(rowptr))
    col = np.empty(nnz, dtype=np.int32)
    val = np.empty(nnz, dtype=np.float64)
    lib.dg_sparse_fill(ctypes.byref(spec), _ptr(perm), _ptr(rowptr), _ptr(col), _ptr(val))

    wstar = normals(seed, _STREAM_WSTAR, d)
    if wstar_density < 1.0:
        keep = uniforms(seed, _STREAM_WSTAR_MASK, d) < wstar_density
        wstar = np.where(keep, wstar, 0.0)
    scores = np.empty(n, dtype=np.float64)
    lib.dg_csr_scores(n, _ptr(rowptr), _ptr(col), _ptr(val), _ptr(wstar), _ptr(scores))
    sigma = noise_std * (float(np.std(scores)) if noise_relative else 1.0)
    scores += sigma * normals(seed, _STREAM_NOISE, n)
    b = 0.0
    if positive_fraction is not None:
        # offset = minus the (1 - fraction) quantile, so that `fraction` of rows land >= 0
        k = int(round((1.0 - positive_fraction) * n))
        k = min(max(k, 0), n - 1)
        b = -float(np.partition(scores, k)[k])
    y = np.where(scores + b >= 0.0, 1.0, -1.0)
    meta = {"seed": seed, "nnz": int(nnz), "positive_fraction": float(np.mean(y > 0)), "label_offset": b,
            "noise_sigma": sigma}
    return SparseProblem(name, n, d, rowptr, col, val, y, loss=loss, C=C, eps=eps, meta=meta)


def config1() -> SparseProblem:
    """Small sparse LR case: 2,000 x 5,000, exactly 50 distinct uniform columns per row."""
    return make_sparse("c1_sparse_lr_2k", 2000, 5000, seed=BASE_SEED + 1, len_kind="const", len_param=50,
                       col_kind="uniform", val_kind="lognormal", noise_std=0.1)


def config2() -> SparseProblem:
    """rcv1-shaped sparse LR: 20,242 x 47,236, Poisson(74) draws per row, Zipf(1.1) columns."""
    return make_sparse("c2_sparse_lr_rcv1_shape", 20242, 47236, seed=BASE_SEED + 2, len_kind="poisson",
                       len_param=74, col_kind="zipf", zipf_s=1.1, val_kind="lognormal", noise_std=0.1,
                       noise_relative=True, positive_fraction=0.52)


def config3(scale: float = 1.0) -> SparseProblem:
    """url-shaped sparse LR: 2,000,000 x 3,000,000, geometric(mean 115, cap 2000) draws per
    row, Zipf(1.2) columns, binary values, 1%-dense planted model, about 33% positive.
    ``scale`` < 1 shrinks n and d together (tests only)."""
    n = max(1000, int(round(2_000_000 * scale)))
    d = max(1500, int(round(3_000_000 * scale)))
    return make_sparse("c3_sparse_lr_url_shape" + ("" if scale == 1.0 else f"_x{scale:g}"), n, d,
                       seed=BASE_SEED + 3, len_kind="geometric", len_param=115, len_cap=2000, col_kind="zipf",
                       zipf_s=1.2, val_kind="one", wstar_density=0.01, noise_std=0.1, noise_relative=True,
                       positive_fraction=0.33)


# --------------------------------------------------------------------------
# dense recipes
# --------------------------------------------------------------------------
def dense_mu(seed: int, d: int, norm: float = 0.5) -> np.ndarray:
    u = normals(seed, _STREAM_MU, d)
    return norm * u / np.linalg.norm(u)


def dense_rows(seed: int, row0: int, nrows: int, d: int, mu: np.ndarray, shift: np.ndarray, scale: np.ndarray,
               flip_prob: float = 0.1, X_out: Optional[np.ndarray] = None,
               y_out: Optional[np.ndarray] = None) -> Tuple[np.ndarray, np.ndarray]:
    X = np.empty((nrows, d), dtype=np.float64) if X_out is None else X_out
    y = np.empty(nrows, dtype=np.float64) if y_out is None else y_out
    assert X.flags.c_contiguous and X.dtype == np.float64 and X.shape == (nrows, d)
    _L().dg_dense_rows(seed, row0, nrows, d, _ptr(mu), flip_prob, _ptr(shift), _ptr(scale), _ptr(X), _ptr(y))
    return X, y


def config4(n: int = 1_000_000, d: int = 24) -> DenseProblem:
    """Dense L2-SVM, two Gaussians at +-mu (|mu| = 0.5), alternating classes, 10% label
    flips, columns standardised with the sample mean / population std of the matrix."""
    seed = BASE_SEED + 4
    mu = dense_mu(seed, d)
    zero, one = np.zeros(d), np.ones(d)
    X, y = dense_rows(seed, 0, n, d, mu, zero, one)
    mean = X.mean(axis=0)
    std = X.std(axis=0)
    X -= mean
    X /= std
    return DenseProblem("c4_dense_svm_1m" if n == 1_000_000 else f"c4_dense_svm_{n}", n, d, X, y,
                        meta={"seed": seed, "mu": mu, "active_note": "standardised with sample statistics"})


@dataclass
class DenseStream:
    """Config 5: the same generator streamed in row chunks.  Columns are standardised with
    the population statistics of the mixture (mean 0 for 1:1 classes, var 1 + mu_j^2), so
    chunks are independent of each other."""
    n: int
    d: int
    seed: int
    mu: np.ndarray
    chunk_rows: int = 1_000_000

    def chunks(self) -> Iterator[Tuple[int, np.ndarray, np.ndarray]]:
        shift = np.zeros(self.d)
        scale = 1.0 / np.sqrt(1.0 + self.mu * self.mu)
        for row0 in range(0, self.n, self.chunk_rows):
            m = min(self.chunk_rows, self.n - row0)
            X, y = dense_rows(self.seed, row0, m, self.d, self.mu, shift, scale)
            yield row0, X, y

    def rows(self, row0: int, nrows: int) -> Tuple[np.ndarray, np.ndarray]:
        shift = np.zeros(self.d)
        scale = 1.0 / np.sqrt(1.0 + self.mu * self.mu)
        return dense_rows(self.seed, row0, nrows, self.d, self.mu, shift, scale)


def config5(n: int = 230_000_000, d: int = 24) -> DenseStream:
    seed = BASE_SEED + 5
    return DenseStream(n=n, d=d, seed=seed, mu=dense_mu(seed, d))


def num_threads() -> int:
    return int(_L().dg_num_threads())
