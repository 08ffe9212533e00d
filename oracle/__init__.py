"""ctypes front end of the CPU oracle (``tron_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The product package never imports this module.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import List, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "liboracle.so")
_SRC = os.path.join(_HERE, "tron_oracle.c")

LOSS_LR = 0
LOSS_L2SVM = 1


_SO_F64 = os.path.join(_HERE, "liboracle_f64.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (single-threaded, no fast-math), and its plain-fp64 twin used by the
    rounding-sensitivity tests."""
    for so, extra in ((_SO, []), (_SO_F64, ["-DORC_ACC_DOUBLE"])):
        if force or not os.path.exists(so) or os.path.getmtime(so) < os.path.getmtime(_SRC):
            cmd = ["gcc", "-O2", "-fPIC", "-shared", "-fvisibility=hidden", "-ffp-contract=off", *extra, "-o", so, _SRC, "-lm"]
            subprocess.check_call(cmd)
    return _SO


class _Data(ctypes.Structure):
    _fields_ = [("n", ctypes.c_int64), ("d", ctypes.c_int64), ("rowptr", ctypes.c_void_p),
                ("col", ctypes.c_void_p), ("val", ctypes.c_void_p), ("X", ctypes.c_void_p),
                ("y", ctypes.c_void_p)]


class TraceRec(ctypes.Structure):
    _fields_ = [("iter", ctypes.c_int), ("cg_iters", ctypes.c_int), ("accepted", ctypes.c_int),
                ("on_boundary", ctypes.c_int), ("f", ctypes.c_double), ("gnorm", ctypes.c_double),
                ("delta", ctypes.c_double), ("ared", ctypes.c_double), ("pred", ctypes.c_double),
                ("snorm", ctypes.c_double)]


class _Result(ctypes.Structure):
    _fields_ = [("f", ctypes.c_double), ("gnorm", ctypes.c_double), ("gnorm0", ctypes.c_double),
                ("outer_iters", ctypes.c_int), ("cg_iters_total", ctypes.c_int), ("n_fun", ctypes.c_int),
                ("n_grad", ctypes.c_int), ("n_hv", ctypes.c_int), ("converged", ctypes.c_int)]


_PROGRESS_FN = ctypes.CFUNCTYPE(None, ctypes.POINTER(TraceRec))

_libs = {}


def build_variant(out_so: str, src: str = _SRC, extra_flags=()) -> str:
    """Compile a copy of the oracle source (e.g. one with a planted mistake, for the tests that show the pins
    catch it) into out_so with the flags of build()."""
    cmd = ["gcc", "-O2", "-fPIC", "-shared", "-fvisibility=hidden", "-ffp-contract=off", *extra_flags, "-o", out_so, src, "-lm"]
    subprocess.check_call(cmd)
    return out_so


def _L(plain_fp64=False):
    """plain_fp64: False = the oracle, True = its fp64-accumulator twin, a path = a library made by build_variant."""
    if plain_fp64 not in _libs:
        build()
        lib = ctypes.CDLL(plain_fp64 if isinstance(plain_fp64, str) else (_SO_F64 if plain_fp64 else _SO))
        P, dbl, vp, ci = ctypes.POINTER, ctypes.c_double, ctypes.c_void_p, ctypes.c_int
        lib.orc_fun.argtypes = [P(_Data), ci, dbl, vp, P(dbl), vp, vp, vp]
        lib.orc_grad.argtypes = [P(_Data), dbl, vp, vp, vp]
        lib.orc_hv.argtypes = [P(_Data), dbl, vp, vp, vp]
        lib.orc_cg.argtypes = [P(_Data), dbl, vp, vp, dbl, dbl, ci, vp, vp, P(ci), P(ci)]
        lib.orc_tron.argtypes = [P(_Data), ci, dbl, dbl, ci, ci, dbl, vp, P(_Result), P(TraceRec), ci, P(ci)]
        lib.orc_hess_diag.argtypes = [P(_Data), dbl, vp, vp]
        lib.orc_pcg.argtypes = [P(_Data), dbl, vp, vp, vp, dbl, dbl, ci, vp, vp, P(ci), P(ci)]
        lib.orc_tron_pcg.argtypes = [P(_Data), ci, dbl, dbl, ci, ci, dbl, dbl, vp, P(_Result), P(TraceRec), ci, P(ci)]
        lib.orc_set_progress.argtypes = [_PROGRESS_FN]
        lib.orc_set_progress.restype = None
        for f in (lib.orc_fun, lib.orc_grad, lib.orc_hv, lib.orc_cg, lib.orc_tron, lib.orc_hess_diag, lib.orc_pcg, lib.orc_tron_pcg):
            f.restype = ci
        _libs[plain_fp64] = lib
    return _libs[plain_fp64]


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


@dataclass
class SolveResult:
    w: np.ndarray
    f: float
    gnorm: float
    gnorm0: float
    outer_iters: int
    cg_iters_total: int
    n_fun: int
    n_grad: int
    n_hv: int
    converged: bool
    status: int
    trace: List[dict]


class Oracle:
    """One dataset (CSR or dense row-major) bound to the oracle routines."""

    def __init__(self, *, n: int, d: int, y, rowptr=None, col=None, val=None, X=None, plain_fp64=False):
        self.n, self.d = int(n), int(d)
        # True: sums in fp64 instead of long double (rounding-sensitivity experiments only); a path: a build_variant library
        self._plain = plain_fp64 if isinstance(plain_fp64, str) else bool(plain_fp64)
        self.y = _f64(y)
        assert self.y.shape == (self.n,)
        if X is not None:
            self.X = _f64(X)
            assert self.X.shape == (self.n, self.d)
            self.rowptr = self.col = self.val = None
        else:
            self.X = None
            self.rowptr = np.ascontiguousarray(rowptr, dtype=np.int64)
            self.col = np.ascontiguousarray(col, dtype=np.int32)
            self.val = _f64(val)
            assert self.rowptr.shape == (self.n + 1,)
        self._c = _Data(self.n, self.d,
                        None if self.rowptr is None else self.rowptr.ctypes.data,
                        None if self.col is None else self.col.ctypes.data,
                        None if self.val is None else self.val.ctypes.data,
                        None if self.X is None else self.X.ctypes.data,
                        self.y.ctypes.data)

    @classmethod
    def from_problem(cls, p, plain_fp64: bool = False) -> "Oracle":
        if getattr(p, "X", None) is not None:
            return cls(n=p.n, d=p.d, y=p.y, X=p.X, plain_fp64=plain_fp64)
        return cls(n=p.n, d=p.d, y=p.y, rowptr=p.rowptr, col=p.col, val=p.val, plain_fp64=plain_fp64)

    def restrict(self, rows) -> "Oracle":
        """The problem over the listed instances only (one training fold of the cross-validation of Section 2.1):
        same features, rows X[rows] and labels y[rows], in the order given."""
        rows = np.asarray(rows, dtype=np.int64)
        if self.X is not None:
            return Oracle(n=len(rows), d=self.d, y=self.y[rows], X=self.X[rows], plain_fp64=self._plain)
        lens = self.rowptr[rows + 1] - self.rowptr[rows]
        rowptr = np.zeros(len(rows) + 1, dtype=np.int64)
        np.cumsum(lens, out=rowptr[1:])
        take = np.concatenate([np.arange(self.rowptr[i], self.rowptr[i + 1]) for i in rows]) if len(rows) else np.zeros(0, np.int64)
        return Oracle(n=len(rows), d=self.d, y=self.y[rows], rowptr=rowptr, col=self.col[take], val=self.val[take],
                      plain_fp64=self._plain)

    def fun(self, loss: int, C: float, w):
        """f(w) and the per-instance z, zhat, D at w."""
        w = _f64(w)
        f = ctypes.c_double()
        z = np.empty(self.n); zhat = np.empty(self.n); D = np.empty(self.n)
        rc = _L(self._plain).orc_fun(ctypes.byref(self._c), loss, C, w.ctypes.data, ctypes.byref(f), z.ctypes.data,
                          zhat.ctypes.data, D.ctypes.data)
        assert rc == 0
        return f.value, z, zhat, D

    def grad(self, C: float, w, zhat):
        w, zhat = _f64(w), _f64(zhat)
        g = np.empty(self.d)
        rc = _L(self._plain).orc_grad(ctypes.byref(self._c), C, w.ctypes.data, zhat.ctypes.data, g.ctypes.data)
        assert rc == 0
        return g

    def fun_grad(self, loss: int, C: float, w):
        f, _, zhat, D = self.fun(loss, C, w)
        return f, self.grad(C, w, zhat), D

    def hv(self, C: float, D, v):
        D, v = _f64(D), _f64(v)
        Hv = np.empty(self.d)
        rc = _L(self._plain).orc_hv(ctypes.byref(self._c), C, D.ctypes.data, v.ctypes.data, Hv.ctypes.data)
        assert rc == 0
        return Hv

    def cg(self, C: float, D, g, delta: float, xi: float = 0.1, max_cg: int = 1000):
        D, g = _f64(D), _f64(g)
        s = np.empty(self.d); r = np.empty(self.d)
        nhv, onb = ctypes.c_int(), ctypes.c_int()
        rc = _L(self._plain).orc_cg(ctypes.byref(self._c), C, D.ctypes.data, g.ctypes.data, delta, xi, max_cg,
                         s.ctypes.data, r.ctypes.data, ctypes.byref(nhv), ctypes.byref(onb))
        assert rc == 0
        return s, r, nhv.value, bool(onb.value)

    def hess_diag(self, C: float, D):
        """diag(H) = 1 + C sum_i D_i x_ij^2."""
        D = _f64(D)
        hd = np.empty(self.d)
        rc = _L(self._plain).orc_hess_diag(ctypes.byref(self._c), C, D.ctypes.data, hd.ctypes.data)
        assert rc == 0
        return hd

    def pcg(self, C: float, D, g, M, delta: float, xi: float = 0.1, max_cg: int = 1000):
        """Steihaug-Toint iteration preconditioned by the diagonal M, trust region in the M-norm."""
        D, g, M = _f64(D), _f64(g), _f64(M)
        s = np.empty(self.d); r = np.empty(self.d)
        nhv, onb = ctypes.c_int(), ctypes.c_int()
        rc = _L(self._plain).orc_pcg(ctypes.byref(self._c), C, D.ctypes.data, g.ctypes.data, M.ctypes.data, delta, xi,
                                     max_cg, s.ctypes.data, r.ctypes.data, ctypes.byref(nhv), ctypes.byref(onb))
        assert rc == 0
        return s, r, nhv.value, bool(onb.value)

    def tron(self, loss: int, C: float, eps: float, w0=None, max_outer: int = 1000, max_cg: int = 1000,
             xi: float = 0.1, trace_cap: int = 1024, precond_blend=None, progress=None) -> SolveResult:
        """precond_blend = None: plain CG; a number a in (0, 1]: CG preconditioned by (1-a) I + a diag(H).
        progress: called with the record (a dict) of every finished outer iteration, for long solves."""
        lib = _L(self._plain)
        cb = _PROGRESS_FN(lambda rec: progress({k: getattr(rec.contents, k) for k, _ in TraceRec._fields_})) if progress else None
        lib.orc_set_progress(cb if cb else _PROGRESS_FN())
        try:
            return self._tron(loss, C, eps, w0, max_outer, max_cg, xi, trace_cap, precond_blend)
        finally:
            lib.orc_set_progress(_PROGRESS_FN())

    def _tron(self, loss, C, eps, w0, max_outer, max_cg, xi, trace_cap, precond_blend) -> SolveResult:
        w = np.zeros(self.d) if w0 is None else _f64(w0).copy()
        res = _Result()
        trace = (TraceRec * trace_cap)()
        tl = ctypes.c_int()
        if precond_blend is not None:
            rc = _L(self._plain).orc_tron_pcg(ctypes.byref(self._c), loss, C, eps, max_outer, max_cg, xi,
                                              float(precond_blend), w.ctypes.data, ctypes.byref(res), trace, trace_cap,
                                              ctypes.byref(tl))
        else:
            rc = _L(self._plain).orc_tron(ctypes.byref(self._c), loss, C, eps, max_outer, max_cg, xi, w.ctypes.data,
                           ctypes.byref(res), trace, trace_cap, ctypes.byref(tl))
        assert rc >= 0
        recs = [{k: getattr(trace[i], k) for k, _ in TraceRec._fields_} for i in range(tl.value)]
        return SolveResult(w, res.f, res.gnorm, res.gnorm0, res.outer_iters, res.cg_iters_total, res.n_fun,
                           res.n_grad, res.n_hv, bool(res.converged), rc, recs)
