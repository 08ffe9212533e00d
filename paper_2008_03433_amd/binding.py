"""ctypes binding of include/tron.h: same names, argument marshalling only."""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import List, Optional, Tuple

HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(HERE, "libtron_hip.so")

LOSS_LR = 0
LOSS_L2SVM = 1
MEM_HOST = 0
MEM_DEVICE = 1
OK, EINVAL, ENOMEM, EDEVICE, ESTATE, EMAXITER = 0, -1, -2, -3, -4, 1

_i64, _i32, _dbl, _vp, _int = ctypes.c_int64, ctypes.c_int32, ctypes.c_double, ctypes.c_void_p, ctypes.c_int


class TronError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"tron error {code}: {msg}")
        self.code = code


class _Params(ctypes.Structure):
    _fields_ = [("loss", _int), ("C", _dbl), ("eps", _dbl), ("max_outer", _int), ("max_cg", _int), ("cg_xi", _dbl),
                ("precond_blend", _dbl)]


class TraceRec(ctypes.Structure):
    _fields_ = [("iter", _int), ("cg_iters", _int), ("accepted", _int), ("on_boundary", _int), ("f", _dbl),
                ("gnorm", _dbl), ("delta", _dbl), ("ared", _dbl), ("pred", _dbl), ("snorm", _dbl)]


class _Result(ctypes.Structure):
    _fields_ = [("f", _dbl), ("gnorm", _dbl), ("gnorm0", _dbl), ("outer_iters", _int), ("cg_iters_total", _int),
                ("n_fun", _int), ("n_grad", _int), ("n_hv", _int), ("converged", _int), ("trace_cap", _int),
                ("trace_len", _int), ("trace", ctypes.POINTER(TraceRec))]


# every symbol include/tron.h declares, with its signature
_SIGNATURES = {
    "tron_dataset_create_csr": (_int, [_i64, _i64, _vp, _vp, _vp, _vp, _int, _vp, ctypes.POINTER(_vp)]),
    "tron_dataset_create_dense": (_int, [_i64, _i64, _vp, _vp, _int, _vp, ctypes.POINTER(_vp)]),
    "tron_dataset_create_dense_empty": (_int, [_i64, _i64, _vp, ctypes.POINTER(_vp)]),
    "tron_dataset_write_rows": (_int, [_vp, _i64, _i64, _vp, _vp, _int]),
    "tron_dataset_destroy": (None, [_vp]),
    "tron_dataset_shape": (_int, [_vp, ctypes.POINTER(_i64), ctypes.POINTER(_i64), ctypes.POINTER(_i64), ctypes.POINTER(_int)]),
    "tron_dataset_stat": (_int, [_vp, ctypes.c_char_p, ctypes.POINTER(_i64)]),
    "tron_fun_grad": (_int, [_vp, _int, _dbl, _vp, ctypes.POINTER(_dbl), _vp]),
    "tron_hv": (_int, [_vp, _dbl, _vp, _vp, ctypes.POINTER(_dbl)]),
    "tron_hv_static": (_int, [_vp, _dbl, _vp, _vp, _vp]),
    "tron_solve": (_int, [_vp, ctypes.POINTER(_Params), _vp, ctypes.POINTER(_Result)]),
    "tron_hess_diag": (_int, [_vp, _dbl, _vp]),
    "tron_batch_create": (_int, [_vp, _int, _vp, _int, ctypes.POINTER(_vp)]),
    "tron_batch_destroy": (None, [_vp]),
    "tron_batch_fun_grad": (_int, [_vp, _int, ctypes.POINTER(_dbl), _vp, ctypes.POINTER(_dbl), _vp]),
    "tron_batch_hv": (_int, [_vp, ctypes.POINTER(_dbl), _vp, _vp, ctypes.POINTER(_dbl)]),
    "tron_batch_solve": (_int, [_vp, ctypes.POINTER(_Params), ctypes.POINTER(_dbl), _vp, ctypes.POINTER(_Result), ctypes.POINTER(_int)]),
    "tron_last_error": (ctypes.c_char_p, []),
    "tron_profile_enable": (_int, [_vp, _int]),
    "tron_profile_read": (_int, [_vp, _int, ctypes.POINTER(ctypes.c_char_p), ctypes.POINTER(_dbl), ctypes.POINTER(_i64), ctypes.POINTER(_int)]),
    "tron_probe_read_bandwidth": (_int, [_vp, _i64, _int, _vp, ctypes.POINTER(_dbl), ctypes.POINTER(_dbl)]),
    "tron_tuning_set": (_int, [ctypes.c_char_p, _i64]),
    "tron_probe_copy_bandwidth": (_int, [_vp, _vp, _i64, _int, _vp, ctypes.POINTER(_dbl)]),
}

_lib = None


def lib_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libtron_hip.so.  Fails loudly if it has not been built: there is no fallback."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(f"{_LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                              "(or paper_2008_03433_amd/build.py) first; there is no CPU fallback")
        # torch first: it carries its own copy of the HIP runtime, and the tensors this binding passes are allocated by
        # that copy.  Loaded afterwards, the library resolves its HIP calls against the runtime already in the process
        # instead of bringing in a second one that knows nothing of those allocations.
        import torch  # noqa: F401
        lib = ctypes.CDLL(_LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype = res
            fn.argtypes = args
        _lib = lib
    return _lib


def tron_last_error() -> str:
    return load_library().tron_last_error().decode()


def _check(rc: int) -> int:
    if rc < 0:
        raise TronError(rc, tron_last_error())
    return rc


def _ptr(t) -> Optional[int]:
    """Address of a torch tensor / numpy array / raw int (None passes NULL)."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if hasattr(t, "data_ptr"):
        assert t.is_contiguous()
        return t.data_ptr()
    assert t.flags.c_contiguous
    return t.ctypes.data


def _is_device(t) -> bool:
    return hasattr(t, "is_cuda") and t.is_cuda


def _stream_ptr(stream) -> Optional[int]:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


# --------------------------------------------------------------------------- raw calls
def tron_dataset_create_csr(n, d, rowptr, col, val, y, stream=None) -> int:
    """rowptr int64[n+1], col int32[nnz], val/y float64; all numpy (host) or all torch CUDA tensors."""
    mem = MEM_DEVICE if _is_device(rowptr) else MEM_HOST
    out = _vp()
    _check(load_library().tron_dataset_create_csr(n, d, _ptr(rowptr), _ptr(col), _ptr(val), _ptr(y), mem,
                                                  _stream_ptr(stream), ctypes.byref(out)))
    return out.value


def tron_dataset_create_dense(n, d, X, y, stream=None) -> int:
    mem = MEM_DEVICE if _is_device(X) else MEM_HOST
    out = _vp()
    _check(load_library().tron_dataset_create_dense(n, d, _ptr(X), _ptr(y), mem, _stream_ptr(stream), ctypes.byref(out)))
    return out.value


def tron_dataset_create_dense_empty(n, d, stream=None) -> int:
    out = _vp()
    _check(load_library().tron_dataset_create_dense_empty(n, d, _stream_ptr(stream), ctypes.byref(out)))
    return out.value


def tron_dataset_write_rows(ds, row0, nrows, X_chunk, y_chunk) -> None:
    mem = MEM_DEVICE if _is_device(X_chunk) else MEM_HOST
    _check(load_library().tron_dataset_write_rows(ds, row0, nrows, _ptr(X_chunk), _ptr(y_chunk), mem))


def tron_dataset_destroy(ds) -> None:
    load_library().tron_dataset_destroy(ds)


def tron_dataset_shape(ds) -> Tuple[int, int, int, bool]:
    n, d, nnz, dense = _i64(), _i64(), _i64(), _int()
    _check(load_library().tron_dataset_shape(ds, ctypes.byref(n), ctypes.byref(d), ctypes.byref(nnz), ctypes.byref(dense)))
    return n.value, d.value, nnz.value, bool(dense.value)


def tron_dataset_stat(ds, name: str) -> int:
    v = _i64()
    _check(load_library().tron_dataset_stat(ds, name.encode(), ctypes.byref(v)))
    return v.value


def tron_fun_grad(ds, loss, C, w, g=None) -> float:
    """Returns f(w); writes the gradient into the CUDA tensor g when given."""
    f = _dbl()
    _check(load_library().tron_fun_grad(ds, loss, C, _ptr(w), ctypes.byref(f), _ptr(g)))
    return f.value


def tron_hv(ds, C, v, Hv, want_vHv=True) -> Optional[float]:
    """Hv = H(w) v for the w of the last tron_fun_grad; returns v.Hv (or None, without synchronising)."""
    if want_vHv:
        s = _dbl()
        _check(load_library().tron_hv(ds, C, _ptr(v), _ptr(Hv), ctypes.byref(s)))
        return s.value
    _check(load_library().tron_hv(ds, C, _ptr(v), _ptr(Hv), None))
    return None


def tron_hv_static(ds, C, v, Hv, vHv=None) -> None:
    """tron_hv without any allocation (dense handles): enqueues only; vHv is a CUDA tensor of one double, or None."""
    _check(load_library().tron_hv_static(ds, C, _ptr(v), _ptr(Hv), _ptr(vHv)))


def tron_hess_diag(ds, C, hd) -> None:
    """hd (CUDA tensor, d doubles) = diagonal of the Hessian at the w of the last tron_fun_grad."""
    _check(load_library().tron_hess_diag(ds, C, _ptr(hd)))


@dataclass
class SolveResult:
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


def tron_solve(ds, loss, C, eps, w, max_outer=1000, max_cg=1000, cg_xi=0.1, trace_cap=1024, precond_blend=0.0) -> SolveResult:
    """Runs the solve in place on the CUDA tensor w (in: w0, out: final iterate)."""
    params = _Params(loss, C, eps, max_outer, max_cg, cg_xi, precond_blend)
    trace = (TraceRec * max(trace_cap, 1))()
    res = _Result()
    res.trace_cap = trace_cap
    res.trace = ctypes.cast(trace, ctypes.POINTER(TraceRec)) if trace_cap > 0 else None
    rc = _check(load_library().tron_solve(ds, ctypes.byref(params), _ptr(w), ctypes.byref(res)))
    recs = [{k: getattr(trace[i], k) for k, _ in TraceRec._fields_} for i in range(res.trace_len)]
    return SolveResult(res.f, res.gnorm, res.gnorm0, res.outer_iters, res.cg_iters_total, res.n_fun, res.n_grad,
                       res.n_hv, bool(res.converged), rc, recs)


BATCH_MAX = 16
BATCH_MAX_D = 32


def tron_batch_create(ds, K, member) -> int:
    """member: n uint32 words (numpy or torch CUDA tensor of dtype int32/uint32); bit k = instance belongs to problem k."""
    mem = MEM_DEVICE if _is_device(member) else MEM_HOST
    out = _vp()
    _check(load_library().tron_batch_create(ds, K, _ptr(member), mem, ctypes.byref(out)))
    return out.value


def tron_batch_destroy(b) -> None:
    load_library().tron_batch_destroy(b)


def _dbl_array(values):
    return (_dbl * len(values))(*[float(v) for v in values])


def tron_batch_fun_grad(b, loss, C, W, G=None) -> List[float]:
    """C: K values; W, G: CUDA tensors of K*d doubles.  Returns the K function values."""
    K = len(C)
    f = (_dbl * K)()
    _check(load_library().tron_batch_fun_grad(b, loss, _dbl_array(C), _ptr(W), f, _ptr(G)))
    return list(f)


def tron_batch_hv(b, C, V, HV, want_vHv=True) -> Optional[List[float]]:
    K = len(C)
    s = (_dbl * K)() if want_vHv else None
    _check(load_library().tron_batch_hv(b, _dbl_array(C), _ptr(V), _ptr(HV), s))
    return list(s) if want_vHv else None


def tron_batch_solve(b, loss, C, eps, W, max_outer=1000, max_cg=1000, cg_xi=0.1, trace_cap=1024, precond_blend=0.0) -> List[SolveResult]:
    """Solves the K problems in place on the CUDA tensor W (K*d doubles); one SolveResult per problem."""
    K = len(C)
    params = _Params(loss, 0.0, eps, max_outer, max_cg, cg_xi, precond_blend)
    traces = [(TraceRec * max(trace_cap, 1))() for _ in range(K)]
    res = (_Result * K)()
    for k in range(K):
        res[k].trace_cap = trace_cap
        res[k].trace = ctypes.cast(traces[k], ctypes.POINTER(TraceRec)) if trace_cap > 0 else None
    status = (_int * K)()
    _check(load_library().tron_batch_solve(b, ctypes.byref(params), _dbl_array(C), _ptr(W), res, status))
    out = []
    for k in range(K):
        r = res[k]
        recs = [{f: getattr(traces[k][i], f) for f, _ in TraceRec._fields_} for i in range(r.trace_len)]
        out.append(SolveResult(r.f, r.gnorm, r.gnorm0, r.outer_iters, r.cg_iters_total, r.n_fun, r.n_grad, r.n_hv,
                               bool(r.converged), status[k], recs))
    return out


def tron_profile_enable(ds, on: bool) -> None:
    _check(load_library().tron_profile_enable(ds, 1 if on else 0))


def tron_profile_read(ds) -> dict:
    cap = 64
    names = (ctypes.c_char_p * cap)()
    ms = (_dbl * cap)()
    calls = (_i64 * cap)()
    count = _int()
    _check(load_library().tron_profile_read(ds, cap, names, ms, calls, ctypes.byref(count)))
    return {names[i].decode(): {"ms": ms[i], "calls": calls[i]} for i in range(min(count.value, cap)) if calls[i] > 0}


def tron_probe_read_bandwidth(src, count, reps=10, stream=None) -> Tuple[float, float]:
    ms, cs = _dbl(), _dbl()
    _check(load_library().tron_probe_read_bandwidth(_ptr(src), count, reps, _stream_ptr(stream), ctypes.byref(ms), ctypes.byref(cs)))
    return ms.value, cs.value


def tron_tuning_set(name: str, value: int) -> None:
    _check(load_library().tron_tuning_set(name.encode(), value))


def tron_probe_copy_bandwidth(dst, src, count, reps=10, stream=None) -> float:
    ms = _dbl()
    _check(load_library().tron_probe_copy_bandwidth(_ptr(dst), _ptr(src), count, reps, _stream_ptr(stream), ctypes.byref(ms)))
    return ms.value


# --------------------------------------------------------------------------- convenience wrapper
class Dataset:
    """Owns a handle; thin sugar over the raw calls above."""

    def __init__(self, handle: int):
        self.handle = handle
        self.n, self.d, self.nnz, self.dense = tron_dataset_shape(handle)

    @classmethod
    def from_csr(cls, n, d, rowptr, col, val, y, stream=None) -> "Dataset":
        return cls(tron_dataset_create_csr(n, d, rowptr, col, val, y, stream))

    @classmethod
    def from_dense(cls, X, y, stream=None) -> "Dataset":
        n, d = X.shape
        return cls(tron_dataset_create_dense(n, d, X, y, stream))

    @classmethod
    def from_problem(cls, p, stream=None) -> "Dataset":
        if getattr(p, "X", None) is not None:
            return cls.from_dense(p.X, p.y, stream)
        return cls.from_csr(p.n, p.d, p.rowptr, p.col, p.val, p.y, stream)

    def fun_grad(self, loss, C, w, g=None):
        return tron_fun_grad(self.handle, loss, C, w, g)

    def hv(self, C, v, Hv, want_vHv=True):
        return tron_hv(self.handle, C, v, Hv, want_vHv)

    def hv_static(self, C, v, Hv, vHv=None):
        return tron_hv_static(self.handle, C, v, Hv, vHv)

    def hess_diag(self, C, hd):
        return tron_hess_diag(self.handle, C, hd)

    def solve(self, loss, C, eps, w, **kw):
        return tron_solve(self.handle, loss, C, eps, w, **kw)

    def close(self):
        if self.handle:
            tron_dataset_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Batch:
    """Up to BATCH_MAX problems over the rows of one dense Dataset (which must outlive the batch)."""

    def __init__(self, dataset: Dataset, K: int, member):
        self.dataset = dataset
        self.K = K
        self.handle = tron_batch_create(dataset.handle, K, member)

    def fun_grad(self, loss, C, W, G=None):
        return tron_batch_fun_grad(self.handle, loss, C, W, G)

    def hv(self, C, V, HV, want_vHv=True):
        return tron_batch_hv(self.handle, C, V, HV, want_vHv)

    def solve(self, loss, C, eps, W, **kw):
        return tron_batch_solve(self.handle, loss, C, eps, W, **kw)

    def close(self):
        if self.handle:
            tron_batch_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
