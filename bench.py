#!/usr/bin/env python3
"""Benchmark of the TRON hot path on one MI355X.

A "step" is one full trust-region Newton solve from w = 0 on a resident synthetic workload: it
exercises every stage of the path (z = Xw, loss terms, f reduction, gradient, the Hessian-vector
products of the CG loop, the CG vector updates and the host driver).  `value` is the number of
Hessian-vector products completed per second of solve wall-clock (all stages included); the
stand-alone tron_hv and tron_fun_grad rates, the solve seconds and the HBM roofline of the dominant
kernel are reported next to it.  One JSON line is printed on stdout; progress goes to stderr.

    python bench.py [--workload c3|c5|c4|c2|c1] [--steps K] [--warmup W] [--gpus 1]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, published peak


def log(msg: str) -> None:
    print(f"[bench {time.strftime('%H:%M:%S')}] {msg}", file=sys.stderr, flush=True)


def make_workload(name: str, scale: float):
    """Returns (problem-or-stream, description).  Data are generated on the host, seeded."""
    import datagen as dg
    if name == "c1":
        return dg.config1()
    if name == "c2":
        return dg.config2()
    if name == "c3":
        return dg.config3(scale)
    if name == "c4":
        return dg.config4(n=max(1000, int(round(1_000_000 * scale))))
    if name == "c5":
        return dg.config5(n=max(1000, int(round(230_000_000 * scale))))
    raise SystemExit(f"unknown workload {name!r}")


def upload(tron, workload):
    """Creates the device dataset; config 5 is streamed in 1M-row chunks."""
    import datagen as dg
    if isinstance(workload, dg.DenseStream):
        ds = tron.Dataset(tron.tron_dataset_create_dense_empty(workload.n, workload.d))
        t0 = time.time()
        for row0, X, y in workload.chunks():
            tron.tron_dataset_write_rows(ds.handle, row0, X.shape[0], X, y)
            if (row0 // workload.chunk_rows) % 20 == 0:
                log(f"  uploaded rows {row0 + X.shape[0]:,} / {workload.n:,} ({time.time() - t0:.0f} s)")
        return ds
    return tron.Dataset.from_problem(workload)


def algorithmic_bytes(ds, kernel: str) -> float:
    """Bytes the method has to move per launch of the named kernel (fp64 values, int32 columns, int64 row
    pointers): one SpMV pass = 12 nnz + 24 rows + 8 cols; the fused dense pass = 8 n d + 8 n."""
    n, d, nnz = ds.n, ds.d, ds.nnz
    if kernel in ("dense_hv",):
        return 8.0 * n * d + 8.0 * n                       # X once + D
    if kernel == "dense_fun_grad":
        return 8.0 * n * d + 16.0 * n                      # X once + y read + D written
    if kernel in ("spmv_fwd_a1",):
        return 12.0 * nnz + 24.0 * n + 8.0 * d             # col+val, rowptr + D + a1 written, v gathered
    if kernel in ("spmv_bwd_hv", "spmv_bwd_g"):
        return 12.0 * nnz + 24.0 * d + 8.0 * n             # col+val, rowptr + v/w + out written, a1/zhat gathered
    if kernel == "spmv_fwd_z":
        return 12.0 * nnz + 16.0 * n + 8.0 * d
    raise KeyError(kernel)


def hv_call_bytes(ds) -> float:
    if ds.dense:
        return 8.0 * ds.n * ds.d + 8.0 * ds.n
    return 24.0 * ds.nnz + 32.0 * ds.n + 32.0 * ds.d


def cpu_baseline(workload, loss, C, budget_s: float = 20.0):
    """The CPU oracle timed on this host, one thread, on a bounded sample of the same workload."""
    import numpy as np
    import datagen as dg
    from oracle import Oracle

    if isinstance(workload, dg.DenseStream):
        rows = min(workload.n, 4_000_000)
        X, y = workload.rows(0, rows)
        o = Oracle(n=rows, d=workload.d, y=y, X=X)
        scale = rows / workload.n
        sample = f"first {rows:,} of {workload.n:,} rows; rate scaled by {scale:.5f}"
    elif getattr(workload, "X", None) is not None:
        o = Oracle.from_problem(workload)
        scale = 1.0
        sample = "full matrix"
    else:
        o = Oracle.from_problem(workload)
        scale = 1.0
        sample = "full matrix"
    w = np.zeros(o.d)
    t0 = time.perf_counter()
    _, g, D = o.fun_grad(loss, C, w)
    t_fg = time.perf_counter() - t0
    v = -g
    times = []
    t_start = time.perf_counter()
    while len(times) < 3 or (time.perf_counter() - t_start < budget_s and len(times) < 20):
        t0 = time.perf_counter()
        o.hv(C, D, v)
        times.append(time.perf_counter() - t0)
    med = float(np.median(times))
    return {
        "value": scale / med, "unit": "Hv/s", "cores": 1, "kind": "oracle",
        "sample": f"{len(times)} oracle Hv calls, {sample}; median {med:.3f} s per sampled call; "
                  f"one fun+grad took {t_fg:.3f} s",
        "fun_grad_per_s": scale / t_fg,
    }


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="c3", choices=["c1", "c2", "c3", "c4", "c5"])
    ap.add_argument("--scale", type=float, default=1.0, help="shrink the workload (debugging only; reported)")
    ap.add_argument("--hv-reps", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--tune", action="append", default=[], metavar="KNOB=VALUE", help="library tuning knob (see tron_tuning_set)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch
    import datagen as dg
    import paper_2008_03433_amd as tron

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the library has no CPU fallback", file=sys.stderr)
        return 3
    torch.cuda.set_device(0)
    tron.load_library()
    for kv in args.tune:
        k, v_ = kv.split("=")
        tron.tron_tuning_set(k, int(v_))

    t0 = time.time()
    log(f"generating workload {args.workload} (scale {args.scale:g}) with {dg.num_threads()} host threads")
    workload = make_workload(args.workload, args.scale)
    loss, C, eps = (dg.LOSS_L2SVM, 0.1, 0.01) if args.workload in ("c4", "c5") else (dg.LOSS_LR, 1.0, 0.01)
    log(f"generated in {time.time() - t0:.1f} s; uploading")
    t0 = time.time()
    ds = upload(tron, workload)
    log(f"dataset resident: n={ds.n:,} d={ds.d:,} nnz={ds.nnz:,} dense={ds.dense} ({time.time() - t0:.1f} s)")
    name = workload.name if hasattr(workload, "name") else f"c5_dense_svm_{ds.n}"

    w = torch.zeros(ds.d, dtype=torch.float64, device="cuda")

    # ---- timed region: K full solves from w = 0
    def one_solve():
        w.zero_()
        return ds.solve(loss, C, eps, w)

    for _ in range(args.warmup):
        res = one_solve()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    n_hv = 0
    for _ in range(args.steps):
        res = one_solve()
        n_hv += res.n_hv
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    solve_s = elapsed / args.steps
    log(f"solve: {solve_s * 1e3:.2f} ms, outer={res.outer_iters} cg={res.cg_iters_total} f={res.f:.10g} converged={res.converged}")

    # ---- stand-alone call rates (HIP events on the handle's stream via the library's profiler)
    g = torch.empty_like(w)
    v = torch.randn(ds.d, dtype=torch.float64, device="cuda")
    Hv = torch.empty_like(v)
    w.zero_()
    ds.fun_grad(loss, C, w, g)
    for _ in range(3):
        ds.hv(C, v, Hv, want_vHv=False)
    torch.cuda.synchronize()
    tron.tron_profile_enable(ds.handle, True)
    t0 = time.perf_counter()
    for _ in range(args.hv_reps):
        ds.hv(C, v, Hv, want_vHv=False)
    torch.cuda.synchronize()
    hv_s = (time.perf_counter() - t0) / args.hv_reps
    prof_hv = tron.tron_profile_read(ds.handle)
    fg_reps = max(3, args.hv_reps // 4)
    t0 = time.perf_counter()
    for _ in range(fg_reps):
        ds.fun_grad(loss, C, w, g)
    torch.cuda.synchronize()
    fg_s = (time.perf_counter() - t0) / fg_reps
    prof_fg = tron.tron_profile_read(ds.handle)
    tron.tron_profile_enable(ds.handle, False)

    kernels = {k: {"ms": v_["ms"] / v_["calls"], "calls": v_["calls"]} for k, v_ in prof_hv.items()}
    kernels_fg = {k: {"ms": v_["ms"] / v_["calls"], "calls": v_["calls"]} for k, v_ in prof_fg.items()}
    dominant = max((k for k in kernels if k in ("dense_hv", "spmv_fwd_a1", "spmv_bwd_hv")), key=lambda k: kernels[k]["ms"])
    dom_ms = kernels[dominant]["ms"]
    achieved = algorithmic_bytes(ds, dominant) / (dom_ms * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": dominant, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": achieved / HBM_PEAK_GBS, "traffic": None,
                "ms_per_launch": dom_ms, "algorithmic_bytes_per_launch": algorithmic_bytes(ds, dominant)}
    per_kernel = {}
    for k, rec in {**kernels, **kernels_fg}.items():
        try:
            gbs = algorithmic_bytes(ds, k) / (rec["ms"] * 1e-3) / 1e9
            per_kernel[k] = {"ms": rec["ms"], "GB/s": gbs, "frac": gbs / HBM_PEAK_GBS}
        except KeyError:
            per_kernel[k] = {"ms": rec["ms"]}

    # attainable streaming rates on this device, for context (and the known-size kernels the hardware
    # byte counters are scaled with): a 2 GiB read-only sum and a 1 GiB -> 1 GiB copy
    probe_n = 1 << 28
    probe_src = torch.empty(probe_n, dtype=torch.float64, device="cuda").normal_()
    ms_probe, _ = tron.tron_probe_read_bandwidth(probe_src, probe_n, reps=10)
    half = probe_n // 2
    ms_copy = tron.tron_probe_copy_bandwidth(probe_src[half:], probe_src[:half], half, reps=10)
    probe = {"read_GB/s": probe_n * 8 / (ms_probe * 1e-3) / 1e9, "read_bytes": probe_n * 8,
             "copy_GB/s": 2 * half * 8 / (ms_copy * 1e-3) / 1e9, "copy_bytes_read": half * 8, "copy_bytes_written": half * 8}
    del probe_src

    out = {
        "metric": "Hessian-vector products/sec (sustained over full TRON solves) + % HBM peak; end-to-end TRON solve seconds",
        "value": n_hv / elapsed, "unit": "Hv/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": solve_s * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f64", "data": "synthetic",
        "config": {"workload": name, "n": ds.n, "d": ds.d, "nnz": ds.nnz, "layout": "dense" if ds.dense else "csr+csr^T",
                   "loss": "l2svm" if loss == dg.LOSS_L2SVM else "lr", "C": C, "eps": eps, "scale": args.scale, "tune": args.tune},
        "solve": {"seconds": solve_s, "outer_iters": res.outer_iters, "cg_iters": res.cg_iters_total, "n_fun": res.n_fun,
                  "n_grad": res.n_grad, "n_hv": res.n_hv, "f": res.f, "gnorm": res.gnorm, "gnorm0": res.gnorm0,
                  "converged": res.converged},
        "hv_call": {"per_s": 1.0 / hv_s, "ms": hv_s * 1e3, "GB/s": hv_call_bytes(ds) / hv_s / 1e9,
                    "frac_hbm_peak": hv_call_bytes(ds) / hv_s / 1e9 / HBM_PEAK_GBS},
        "fun_grad_call": {"per_s": 1.0 / fg_s, "ms": fg_s * 1e3},
        "kernels": per_kernel,
        "roofline": roofline,
        "stream_probe": probe,
    }
    if not args.no_cpu_baseline:
        log("timing the CPU oracle (one thread, bounded sample)")
        out["cpu_baseline"] = cpu_baseline(workload, loss, C)
    else:
        out["cpu_baseline"] = None
    ds.close()
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
