#!/usr/bin/env python3
"""Benchmark of the TRON hot path on one MI355X.

A "step" is one full trust-region Newton solve from w = 0 on a resident synthetic workload: it
exercises every stage of the path (z = Xw, loss terms, f reduction, gradient, the Hessian-vector
products of the CG loop, the CG vector updates and the host driver).  `value` is the number of
Hessian-vector products completed per second of solve wall-clock (all stages included); the
stand-alone tron_hv and tron_fun_grad rates, the solve seconds and the HBM roofline of the dominant
kernel are reported next to it.  One JSON line is printed on stdout; progress goes to stderr.

    python bench.py [--workload c3|c5|c4|c2|c1] [--also c5|none] [--steps K] [--warmup W] [--gpus 1]

The primary workload (default c3, the large sparse config) fills the top-level fields; the workload
named by --also (default c5, the large dense config) is measured the same way and reported under
"also".
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

# (workload, library profiler slot) -> (kernel name in rocprofv3 output, profiles/ file that holds its byte counters).
# The counters were read on exactly that workload at full size; any other run reports traffic = null.
ROCPROF_NAMES = {
    ("c5", "dense_hv"): ("k_dense_hv<6, 4, 4, true, true, false, false>", "dense_hv_fun_grad_c5.md"),
    ("c5", "dense_fun_grad"): ("k_dense_fun_grad<6, 4, 4, true, 1>", "dense_hv_fun_grad_c5.md"),
    # config 3 has one value per instance: its layouts keep no value stream and run the "unit" kernels
    ("c3", "spmv_head"): ("k_head_sell", "csr_spmv_c3.md"),
    ("c3", "spmv_fwd"): ("k_csr_spmv_part<true, false, false, true>", "csr_spmv_c3.md"),
    ("c3", "spmv_bwd"): ("k_csr_spmv_part<false, false, false, true>", "csr_spmv_c3.md"),
    ("c3", "spmv_tiles"): ("k_hot_tiles_unit", "csr_spmv_c3.md"),
    # the same matrix with the general layout forced (csr_unit = 0: 32-bit / 16-bit indices + fp64 values)
    ("c3_values", "spmv_head"): ("k_csr_spmv_part<true, true, false, false>", "csr_spmv_c3_values.md"),
    ("c3_values", "spmv_fwd"): ("k_csr_spmv_part<true, false, false, false>", "csr_spmv_c3_values.md"),
    ("c3_values", "spmv_bwd"): ("k_csr_spmv_part<false, false, false, false>", "csr_spmv_c3_values.md"),
    ("c3_values", "spmv_tiles"): ("k_hot_tiles<false>", "csr_spmv_c3_values.md"),
}


def log(msg: str) -> None:
    print(f"[bench {time.strftime('%H:%M:%S')}] {msg}", file=sys.stderr, flush=True)


def make_workload(name: str, scale: float):
    """Seeded synthetic workload, generated on the host."""
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
    # other loss / storage mixes of the paper's dataset table: dense logistic regression at the shapes of its two
    # dense UCI sets (5M x 18 and 11M x 28), and the L2-SVM on the url-shaped sparse matrix
    if name == "susy_shape":
        return dg.config5(n=max(1000, int(round(5_000_000 * scale))), d=18)
    if name == "higgs_shape":
        return dg.config5(n=max(1000, int(round(11_000_000 * scale))), d=28)
    if name == "c3_svm":
        return dg.config3(scale)
    raise SystemExit(f"unknown workload {name!r}")


def workload_params(name: str):
    """(loss, C, eps) of a workload."""
    import datagen as dg
    if name in ("c4", "c5"):
        return dg.LOSS_L2SVM, 0.1, 0.01
    if name == "c3_svm":
        return dg.LOSS_L2SVM, 1.0, 0.01
    return dg.LOSS_LR, 1.0, 0.01


def upload(tron, workload):
    """Creates the device dataset; config 5 is streamed in 1M-row chunks."""
    import datagen as dg
    if isinstance(workload, dg.DenseStream):
        ds = tron.Dataset(tron.tron_dataset_create_dense_empty(workload.n, workload.d))
        t0 = time.time()
        for row0, X, y in workload.chunks():
            tron.tron_dataset_write_rows(ds.handle, row0, X.shape[0], X, y)
            if (row0 // workload.chunk_rows) % 40 == 0:
                log(f"  uploaded rows {row0 + X.shape[0]:,} / {workload.n:,} ({time.time() - t0:.0f} s)")
        return ds
    return tron.Dataset.from_problem(workload)


def format_bytes(ds, stat, kernel: str) -> float:
    """Bytes one launch of the named kernel has to move in the format the handle actually stores (the library's own
    count: index / value streams, flag bits, tables, every needed vector element once, partial sums and results
    written).  This is the numerator of every reported HBM fraction: the kernel cannot move fewer bytes, so the
    fraction cannot exceed 1."""
    key = {"dense_hv": "hv_bytes", "dense_fun_grad": "fun_grad_bytes", "spmv_head": "fwd_bytes_head",
           "spmv_fwd": "fwd_bytes_ranges", "spmv_tiles": "bwd_bytes_tiles", "spmv_bwd": "bwd_bytes_ranges",
           "spmv_gather": "fwd_bytes_gather", "spmv_tile_reduce": "bwd_bytes_tile_reduce"}.get(kernel)
    if kernel == "spmv_combine":   # two launches per call (forward with D, transposed with the addend): their mean
        return 0.5 * (stat("fwd_bytes_combine") + 8.0 * ds.n + stat("bwd_bytes_combine") + 8.0 * ds.d)
    if key is None:
        raise KeyError(kernel)
    v = float(stat(key))
    if v <= 0.0:
        raise KeyError(kernel)
    return v


def work_bytes(ds, stat, kernel: str) -> float:
    """The format-independent count of the method's description: 12 B per nonzero (int32 column + fp64 value) and 8 B
    per vector element touched; X once for the fused dense pass.  Reported as a rate of work done ("work_GB/s"), never
    as an HBM fraction: layouts without a value stream move fewer bytes than this."""
    n, d = ds.n, ds.d
    if kernel == "dense_hv":
        return 8.0 * n * d + 8.0 * n
    if kernel == "dense_fun_grad":
        return 8.0 * n * d + 16.0 * n
    if kernel == "spmv_head":
        return 12.0 * stat("fwd_head_nnz") + 8.0 * n
    if kernel == "spmv_fwd":
        return 12.0 * (stat("fwd_csr_nnz") - stat("fwd_head_nnz")) + 8.0 * d + 8.0 * n
    if kernel == "spmv_tiles":
        return 12.0 * stat("bwd_tile_nnz") + 8.0 * n
    if kernel == "spmv_bwd":
        return 12.0 * stat("bwd_csr_nnz") + 8.0 * n + 8.0 * d
    raise KeyError(kernel)


def hv_work_bytes(ds) -> float:
    if ds.dense:
        return 8.0 * ds.n * ds.d + 8.0 * ds.n
    return 24.0 * ds.nnz + 32.0 * ds.n + 32.0 * ds.d


def measured_traffic(profile_key, slot: str):
    """HBM-side bytes per launch from the committed rocprofv3 counter summaries (FETCH_SIZE + WRITE_SIZE, scaled);
    None unless this run is the workload the summary was taken on."""
    if profile_key is None or (profile_key, slot) not in ROCPROF_NAMES:
        return None
    kname, fname = ROCPROF_NAMES[(profile_key, slot)]
    path = os.path.join(ROOT, "profiles", fname)
    if not os.path.exists(path):
        return None
    in_traffic = False
    column = None   # index of the "traffic GB" cell (older summaries: fetched + written)
    for line in open(path):
        if line.startswith("## "):
            in_traffic = "traffic" in line
            column = None
        if not in_traffic or not line.startswith("|"):
            continue
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if cells and cells[0] == "kernel":
            column = cells.index("traffic GB") if "traffic GB" in cells else None
            fetched = cells.index("fetched GB") if "fetched GB" in cells else (cells.index("fetched GB (scaled)") if "fetched GB (scaled)" in cells else None)
            written = cells.index("written GB") if "written GB" in cells else (cells.index("written GB (scaled)") if "written GB (scaled)" in cells else None)
            continue
        if cells and cells[0] == f"`{kname}`":
            try:
                if column is not None:
                    total = float(cells[column]) * 1e9
                elif fetched is not None and written is not None:
                    total = (float(cells[fetched]) + float(cells[written])) * 1e9
                else:
                    return None
            except (ValueError, IndexError):
                return None
            return total if total > 0.0 else None    # a row of zeros: the kernel was not in that profile
    return None


def pin_to_one_core():
    """Pins this process to one of the cores it may run on (the oracle is single-threaded; pinning keeps it from
    migrating).  Returns (core, previous affinity) -- restore with os.sched_setaffinity(0, previous)."""
    prev = os.sched_getaffinity(0)
    core = max(prev)   # away from core 0, where the runtime's helper threads tend to sit
    os.sched_setaffinity(0, {core})
    return core, prev


def cpu_baseline(workload, loss, C, eps=None, budget_s: float = 15.0, full_solve: bool = False):
    """The CPU oracle timed on this host, one thread pinned to one core, on a bounded sample of the same workload;
    with full_solve also one complete oracle solve (config 3: about half a minute)."""
    core, prev = pin_to_one_core()
    try:
        return _cpu_baseline(workload, loss, C, eps, budget_s, full_solve, core)
    finally:
        os.sched_setaffinity(0, prev)


def _cpu_baseline(workload, loss, C, eps, budget_s, full_solve, core):
    import numpy as np
    import datagen as dg
    from oracle import Oracle

    if isinstance(workload, dg.DenseStream):
        rows = min(workload.n, 4_000_000)
        X, y = workload.rows(0, rows)
        o = Oracle(n=rows, d=workload.d, y=y, X=X)
        scale = rows / workload.n
        sample = f"first {rows:,} of {workload.n:,} rows; rate scaled by {scale:.5f}"
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
    cpu_model = "unknown"
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                cpu_model = line.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    out = {
        "value": scale / med, "unit": "Hv/s", "cores": 1, "pinned_to_core": core, "kind": "oracle", "host_cpu": cpu_model,
        "host_nproc": os.cpu_count(),
        "sample": f"{len(times)} oracle Hv calls, {sample}; median {med:.3f} s per sampled call; "
                  f"one fun+grad took {t_fg:.3f} s",
        "fun_grad_per_s": scale / t_fg,
    }
    if full_solve and scale == 1.0:
        log("  oracle: one full solve")
        t0 = time.perf_counter()
        ref = o.tron(loss, C, eps)
        t_solve = time.perf_counter() - t0
        out["solve"] = {"seconds": t_solve, "outer_iters": ref.outer_iters, "cg_iters": ref.cg_iters_total, "f": ref.f,
                        "converged": ref.converged, "hv_per_s_over_the_solve": ref.n_hv / t_solve}
        out["sample"] += f"; one full oracle solve took {t_solve:.1f} s"
    else:
        out["solve"] = None   # the sample is a part of the matrix: no whole solve is timed
    return out


def run_workload(args, wname: str) -> dict:
    import torch
    import datagen as dg
    import paper_2008_03433_amd as tron

    t0 = time.time()
    log(f"generating workload {wname} (scale {args.scale:g}) with {dg.num_threads()} host threads")
    workload = make_workload(wname, args.scale)
    loss, C, eps = workload_params(wname)
    log(f"generated in {time.time() - t0:.1f} s; building the device dataset")
    t0 = time.time()
    ds = upload(tron, workload)
    setup_s = time.time() - t0
    log(f"dataset resident: n={ds.n:,} d={ds.d:,} nnz={ds.nnz:,} dense={ds.dense} ({setup_s:.1f} s)")
    name = workload.name if hasattr(workload, "name") else (f"c5_dense_svm_{ds.n}" if wname == "c5" else f"{wname}_dense_{ds.n}x{ds.d}")
    if wname == "c3_svm":
        name += "_l2svm"

    def stat(key):
        return tron.tron_dataset_stat(ds.handle, key)

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
    solve_times = []
    for _ in range(args.steps):
        t1 = time.perf_counter()
        res = one_solve()          # returns after the solver's last scalar read-back: the stream is idle
        solve_times.append(time.perf_counter() - t1)
        n_hv += res.n_hv
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    solve_s = elapsed / args.steps
    log(f"solve: {solve_s * 1e3:.2f} ms, outer={res.outer_iters} cg={res.cg_iters_total} f={res.f:.10g} converged={res.converged}")

    # ---- the same solve with the diagonally preconditioned inner solver (reported beside, not part of `value`)
    def one_pcg_solve():
        w.zero_()
        return ds.solve(loss, C, eps, w, precond_blend=0.01)
    one_pcg_solve()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    pres = one_pcg_solve()
    pcg_s = time.perf_counter() - t1
    log(f"preconditioned solve: {pcg_s * 1e3:.2f} ms, outer={pres.outer_iters} cg={pres.cg_iters_total} f={pres.f:.10g}")

    # ---- stand-alone call rates: wall-clock without instrumentation, then per-kernel times with HIP events
    #      recorded on the handle's stream by the library's profiler
    g = torch.empty_like(w)
    v = torch.randn(ds.d, dtype=torch.float64, device="cuda")
    Hv = torch.empty_like(v)
    w.zero_()
    ds.fun_grad(loss, C, w, g)
    hv_fmt, fg_fmt = float(stat("hv_bytes")), float(stat("fun_grad_bytes"))   # for the D cached now (w = 0: every row active)
    for _ in range(3):
        ds.hv(C, v, Hv, want_vHv=False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.hv_reps):
        ds.hv(C, v, Hv, want_vHv=False)
    torch.cuda.synchronize()
    hv_s = (time.perf_counter() - t0) / args.hv_reps
    # per-call times with events on the handle's stream (it is torch's current stream)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.hv_reps)]
    for a, b in evs:
        a.record()
        ds.hv(C, v, Hv, want_vHv=False)
        b.record()
    torch.cuda.synchronize()
    hv_each = sorted(a.elapsed_time(b) for a, b in evs)
    fg_reps = max(3, args.hv_reps // 4)
    t0 = time.perf_counter()
    for _ in range(fg_reps):
        ds.fun_grad(loss, C, w, g)
    torch.cuda.synchronize()
    fg_s = (time.perf_counter() - t0) / fg_reps
    tron.tron_profile_enable(ds.handle, True)
    for _ in range(args.hv_reps):
        ds.hv(C, v, Hv, want_vHv=False)
    prof_hv = tron.tron_profile_read(ds.handle)
    for _ in range(fg_reps):
        ds.fun_grad(loss, C, w, g)
    prof_fg = tron.tron_profile_read(ds.handle)
    tron.tron_profile_enable(ds.handle, False)

    kernels = {k: {"ms": r["ms"] / r["calls"], "calls_per_hv": r["calls"] / args.hv_reps} for k, r in prof_hv.items()}
    kernels_fg = {k: {"ms": r["ms"] / r["calls"], "calls_per_fun_grad": r["calls"] / fg_reps} for k, r in prof_fg.items()}
    # HBM fractions are computed from the bytes the stored format makes the kernel move (library count, read while the
    # D of the timed calls is cached); the format-independent 12 B / nonzero count is reported beside them as a rate of
    # work ("work_GB/s"), which can exceed the peak for layouts without a value stream and is never called a fraction.
    profile_key = None
    if args.scale == 1.0 and wname in ("c3", "c5"):
        profile_key = wname if (ds.dense or stat("unit_values")) else "c3_values"

    def kernel_roofline(k, ms, table_name):
        fb = format_bytes(ds, stat, k) if k != "dense_hv" else hv_fmt
        if k == "dense_fun_grad":
            fb = fg_fmt
        rec = {"kernel": k, "in": table_name, "bound": "hbm", "achieved": fb / (ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
               "frac": fb / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "traffic": measured_traffic(profile_key, k), "ms_per_launch": ms,
               "format_bytes_per_launch": fb}
        try:
            rec["work_GB/s"] = work_bytes(ds, stat, k) / (ms * 1e-3) / 1e9
        except KeyError:
            pass
        return rec

    def with_rates(table, table_name):
        outk = {}
        for k, rec in table.items():
            outk[k] = dict(rec)
            try:
                r = kernel_roofline(k, rec["ms"], table_name)
                outk[k].update({"GB/s": r["achieved"], "frac": r["frac"], "format_bytes": r["format_bytes_per_launch"]})
                if "work_GB/s" in r:
                    outk[k]["work_GB/s"] = r["work_GB/s"]
            except KeyError:
                pass
        return outk

    big = [k for k in kernels if k in ("dense_hv", "spmv_head", "spmv_fwd", "spmv_bwd", "spmv_tiles")]
    dominant = max(big, key=lambda k: kernels[k]["ms"])
    roofline = kernel_roofline(dominant, kernels[dominant]["ms"], "kernels_hv")
    roofline["workload"] = name
    # every other large kernel of the two calls, and the calls as a whole
    roofline["also"] = [dict(kernel_roofline(k, kernels[k]["ms"], "kernels_hv"), workload=name) for k in big if k != dominant]
    roofline["also"] += [dict(kernel_roofline(k, kernels_fg[k]["ms"], "kernels_fun_grad"), workload=name)
                         for k in kernels_fg if k in ("dense_fun_grad",)]
    roofline["also"].append({"kernel": "one tron_hv call (all its kernels)", "workload": name, "bound": "hbm",
                             "achieved": hv_fmt / hv_s / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                             "frac": hv_fmt / hv_s / 1e9 / HBM_PEAK_GBS, "ms_per_launch": hv_s * 1e3,
                             "format_bytes_per_launch": hv_fmt, "work_GB/s": hv_work_bytes(ds) / hv_s / 1e9, "traffic": None})
    if not ds.dense:
        roofline["note"] = ("frac = bytes the kernel must move in the stored format / time / 8 TB/s." +
                            (" Every instance of this matrix has one value for all its entries, so the layouts keep no value stream "
                             "(2-4 B per nonzero): the head-partition and tile kernels are bound by LDS gathers and instruction issue, "
                             "the range kernels by L2 requests, not by HBM bytes." if stat("unit_values") else ""))

    out = {
        "metric": "Hessian-vector products/sec (sustained over full TRON solves) + % HBM peak; end-to-end TRON solve seconds",
        "value": n_hv / elapsed, "unit": "Hv/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": solve_s * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f64", "data": "synthetic",
        "config": {"workload": name, "n": ds.n, "d": ds.d, "nnz": ds.nnz, "layout": "dense" if ds.dense else "csr+csr^T",
                   "loss": "l2svm" if loss == dg.LOSS_L2SVM else "lr", "C": C, "eps": eps, "scale": args.scale,
                   "tune": args.tune, "setup_seconds": setup_s},
        "solve": {"seconds": solve_s, "outer_iters": res.outer_iters, "cg_iters": res.cg_iters_total, "n_fun": res.n_fun,
                  "n_grad": res.n_grad, "n_hv": res.n_hv, "f": res.f, "gnorm": res.gnorm, "gnorm0": res.gnorm0,
                  "converged": res.converged, "min_seconds": min(solve_times)},
        "solve_preconditioned": {"precond_blend": 0.01, "seconds": pcg_s, "outer_iters": pres.outer_iters,
                                 "cg_iters": pres.cg_iters_total, "n_hv": pres.n_hv, "f": pres.f, "gnorm": pres.gnorm,
                                 "converged": pres.converged},
        "hv_call": {"per_s": 1.0 / hv_s, "ms": hv_s * 1e3, "GB/s": hv_fmt / hv_s / 1e9,
                    "frac_hbm_peak": hv_fmt / hv_s / 1e9 / HBM_PEAK_GBS, "format_bytes": hv_fmt,
                    "work_bytes": hv_work_bytes(ds), "work_GB/s": hv_work_bytes(ds) / hv_s / 1e9,
                    "event_ms_median": hv_each[len(hv_each) // 2], "event_ms_min": hv_each[0]},
        "fun_grad_call": {"per_s": 1.0 / fg_s, "ms": fg_s * 1e3, "format_bytes": fg_fmt, "GB/s": fg_fmt / fg_s / 1e9,
                          "frac_hbm_peak": fg_fmt / fg_s / 1e9 / HBM_PEAK_GBS},
        "kernels_hv": with_rates(kernels, "kernels_hv"),
        "kernels_fun_grad": with_rates(kernels_fg, "kernels_fun_grad"),
        "roofline": roofline,
    }
    if not ds.dense:
        out["layout"] = {k: stat(k) for k in ("fwd_parts", "bwd_parts", "fwd_csr_nnz", "fwd_head_nnz", "fwd_lds_columns", "bwd_csr_nnz",
                                             "bwd_tile_nnz", "bwd_tile_rows", "bwd_tiles", "unit_values")}
    if not args.no_cpu_baseline:
        log("timing the CPU oracle (one thread, bounded sample)")
        out["cpu_baseline"] = cpu_baseline(workload, loss, C, eps, full_solve=(wname == "c3"))
    else:
        out["cpu_baseline"] = None
    ds.close()
    del ds, w, g, v, Hv
    torch.cuda.empty_cache()
    return out


def small_config(args, wname: str) -> dict:
    """The small configurations (cache-resident / launch-bound): solve and call times, and the oracle's full solve."""
    sub = run_workload(argparse.Namespace(**{**vars(args), "no_cpu_baseline": True, "steps": 5, "warmup": 1}), wname)
    out = {"config": sub["config"]["workload"], "solve_ms": sub["ms_per_step"], "solve_min_ms": sub["solve"]["min_seconds"] * 1e3,
           "outer_iters": sub["solve"]["outer_iters"], "cg_iters": sub["solve"]["cg_iters"], "f": sub["solve"]["f"],
           "hv_ms": sub["hv_call"]["ms"], "hv_format_GB/s": sub["hv_call"]["GB/s"], "hv_frac_hbm_peak": sub["hv_call"]["frac_hbm_peak"],
           "hv_work_GB/s": sub["hv_call"]["work_GB/s"],
           "fun_grad_ms": sub["fun_grad_call"]["ms"], "solve_preconditioned": sub["solve_preconditioned"],
           "kernels_hv": sub["kernels_hv"], "cpu_baseline": None}
    if not args.no_cpu_baseline:
        import datagen as dg
        from oracle import Oracle
        workload = make_workload(wname, 1.0)
        loss, C, eps = workload_params(wname)
        o = Oracle.from_problem(workload)
        t0 = time.perf_counter()
        ref = o.tron(loss, C, eps)
        t_solve = time.perf_counter() - t0
        out["cpu_baseline"] = {"kind": "oracle", "cores": 1, "solve_seconds": t_solve, "f": ref.f,
                               "outer_iters": ref.outer_iters, "cg_iters": ref.cg_iters_total,
                               "value": ref.n_hv / t_solve, "unit": "Hv/s", "sample": "one full solve"}
    return out


def active_set_sweep() -> dict:
    """Dense L2-SVM Hessian-vector time against the active fraction |I|/n, two ways: the pass over X that does not read
    the rows outside the active set, and the pass over a compacted copy X_I built on the device (the paper's choice,
    Section 5).  20M x 24 rows of the config-5 generator; w is moved along the class direction to shrink the active set.
    ideal_ms = 8 |I| d bytes at the 6.5 TB/s the all-active pass sustains."""
    import numpy as np
    import torch
    import datagen as dg
    import paper_2008_03433_amd as tron
    n, d = 20_000_000, 24
    p = dg.config5(n=n, d=d)
    ds = upload(tron, p)
    mu = p.mu / np.linalg.norm(p.mu)
    v = torch.randn(d, dtype=torch.float64, device="cuda")
    Hv = torch.empty_like(v)

    def time_hv(reps=20):
        for _ in range(3):
            ds.hv(0.1, v, Hv, want_vHv=False)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            ds.hv(0.1, v, Hv, want_vHv=False)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / reps * 1e3

    points = []
    try:
        for scale in (0.0, 1.0, 3.0, 12.0, 40.0):
            w = torch.tensor(scale * mu, dtype=torch.float64, device="cuda")
            tron.tron_tuning_set("dense_compact", 0)
            ds.fun_grad(dg.LOSS_L2SVM, 0.1, w, None)
            skip_ms = time_hv()
            skip_bytes = tron.tron_dataset_stat(ds.handle, "hv_bytes")
            rec = {"w_norm": scale, "hv_ms": skip_ms, "hv_format_bytes": skip_bytes}
            if scale > 0.0:
                tron.tron_tuning_set("dense_compact", 1)
                tron.tron_profile_enable(ds.handle, True)
                for _ in range(3):
                    ds.fun_grad(dg.LOSS_L2SVM, 0.1, w, None)
                prof = tron.tron_profile_read(ds.handle)
                tron.tron_profile_enable(ds.handle, False)
                rows = tron.tron_dataset_stat(ds.handle, "dense_compact_rows")
                rec.update({"active_rows": rows, "active_fraction": rows / n, "hv_compacted_ms": time_hv(),
                            "hv_compacted_format_bytes": tron.tron_dataset_stat(ds.handle, "hv_bytes"),
                            "compact_build_ms": prof["dense_compact"]["ms"] / prof["dense_compact"]["calls"],
                            "ideal_ms": 8.0 * rows * d / 6.5e12 * 1e3})
                rec["products_to_amortise_the_copy"] = (rec["compact_build_ms"] / (skip_ms - rec["hv_compacted_ms"])
                                                        if skip_ms > rec["hv_compacted_ms"] else None)
            else:
                rec.update({"active_rows": n, "active_fraction": 1.0, "ideal_ms": 8.0 * n * d / 6.5e12 * 1e3})
            points.append(rec)
    finally:
        tron.tron_tuning_set("dense_compact", -1)
    ds.close()
    return {"n": n, "d": d, "points": points}


def cross_validation(X, y, label: str, folds: int = 3, Cs=(0.1, 1.0), eps: float = 0.01, reps: int = 3) -> dict:
    """Cross-validation folds over one resident matrix (Section 2.1 of the paper): problem (fold f, C) trains the L2-SVM
    on the rows outside fold f.  Batched: every problem advances on the same pass over X (tron_batch_solve).  One at a
    time: the same problems solved one after the other by tron_solve, each on its own compacted copy of its rows (what
    the paper does for X_I, Section 5).  X, y: CUDA tensors."""
    import torch
    import datagen as dg
    import paper_2008_03433_amd as tron
    n, d = X.shape
    K = folds * len(Cs)
    u = torch.from_numpy(dg.uniforms(200803433, 77, n)).cuda()
    fold = torch.clamp((u * folds).to(torch.int32), max=folds - 1)
    C_list = [float(c) for c in Cs for _ in range(folds)]
    member = torch.zeros(n, dtype=torch.int32, device="cuda")
    for k in range(K):
        member |= (fold != (k % folds)).to(torch.int32) << k
    ds = tron.Dataset(tron.tron_dataset_create_dense(n, d, X, y))
    b = tron.Batch(ds, K, member)
    best, res = float("inf"), None
    for _ in range(reps):
        W = torch.zeros((K, d), dtype=torch.float64, device="cuda")
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        res = b.solve(dg.LOSS_L2SVM, C_list, eps, W)
        best = min(best, time.perf_counter() - t0)
    rounds = max(r.n_fun + r.n_hv for r in res)
    # one round at the final iterates, by kernel
    V = torch.randn((K, d), dtype=torch.float64, device="cuda")
    HV = torch.empty_like(V)
    tron.tron_profile_enable(ds.handle, True)
    for _ in range(10):
        b.hv(C_list, V, HV, want_vHv=False)
    prof_hv = tron.tron_profile_read(ds.handle)
    for _ in range(5):
        b.fun_grad(dg.LOSS_L2SVM, C_list, W, None)
    prof_fg = tron.tron_profile_read(ds.handle)
    tron.tron_profile_enable(ds.handle, False)
    hv_pass_ms = prof_hv["batch_pass"]["ms"] / prof_hv["batch_pass"]["calls"]
    fg_pass_ms = prof_fg["batch_pass"]["ms"] / prof_fg["batch_pass"]["calls"]
    advance_ms = prof_hv["batch_advance"]["ms"] / prof_hv["batch_advance"]["calls"]
    batch_f = [r.f for r in res]
    # the same rounds for the logistic loss (fp64 D per row and problem instead of one bit; the function/gradient round
    # evaluates exp / log1p per row and problem)
    b.fun_grad(dg.LOSS_LR, C_list, W, None)
    tron.tron_profile_enable(ds.handle, True)
    for _ in range(10):
        b.hv(C_list, V, HV, want_vHv=False)
    lr_hv = tron.tron_profile_read(ds.handle)
    for _ in range(5):
        b.fun_grad(dg.LOSS_LR, C_list, W, None)
    lr_fg = tron.tron_profile_read(ds.handle)
    tron.tron_profile_enable(ds.handle, False)
    lr_hv_pass_ms = lr_hv["batch_pass"]["ms"] / lr_hv["batch_pass"]["calls"]
    lr_fg_pass_ms = lr_fg["batch_pass"]["ms"] / lr_fg["batch_pass"]["calls"]
    b.close()
    ds.close()
    # one problem at a time on compacted copies
    seq_solve, seq_hv, seq_f, seq_hv_count = 0.0, 0.0, [], 0
    for f in range(folds):
        keep = fold != f
        sub = tron.Dataset(tron.tron_dataset_create_dense(int(keep.sum()), d, X[keep].contiguous(), y[keep].contiguous()))
        for c in Cs:
            t_best, r1 = float("inf"), None
            for _ in range(reps):
                w = torch.zeros(d, dtype=torch.float64, device="cuda")
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                r1 = sub.solve(dg.LOSS_L2SVM, float(c), eps, w)
                t_best = min(t_best, time.perf_counter() - t0)
            seq_solve += t_best
            seq_f.append((list(Cs).index(c) * folds + f, r1.f))
            seq_hv_count += r1.n_hv
            v, hv = V[0].contiguous(), torch.empty(d, dtype=torch.float64, device="cuda")
            for _ in range(3):
                sub.hv(float(c), v, hv, want_vHv=False)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(10):
                sub.hv(float(c), v, hv, want_vHv=False)
            torch.cuda.synchronize()
            seq_hv += (time.perf_counter() - t0) / 10
        sub.close()
        del sub
        torch.cuda.empty_cache()
    agree = max(abs(batch_f[k] - fk) / abs(fk) for k, fk in seq_f)
    return {"workload": label, "n": n, "d": d, "folds": folds, "C": list(Cs), "problems": K, "loss": "l2svm", "eps": eps,
            # the library's rule per loss: the matrix units from eight problems on (L2-SVM), from five (logistic)
            "pass_kernel": "fp64 matrix instructions" if K >= 8 else "vector units",
            "logistic_pass_kernel": "fp64 matrix instructions" if K >= 5 else "vector units",
            "batched": {"solve_ms": best * 1e3, "rounds": rounds, "hv_pass_ms": hv_pass_ms, "fun_grad_pass_ms": fg_pass_ms,
                        "advance_ms": advance_ms, "logistic_hv_pass_ms": lr_hv_pass_ms, "logistic_fun_grad_pass_ms": lr_fg_pass_ms,
                        "hv_per_second_all_problems": K / ((hv_pass_ms + advance_ms) * 1e-3),
                        "X_read_GB/s": 8.0 * n * d / (hv_pass_ms * 1e-3) / 1e9,
                        "outer_iters": [r.outer_iters for r in res], "cg_iters": [r.cg_iters_total for r in res],
                        "converged": all(r.converged for r in res)},
            "one_at_a_time": {"solve_ms_total": seq_solve * 1e3, "hv_ms_total": seq_hv * 1e3, "cg_iters_total": seq_hv_count,
                              "note": "tron_solve / tron_hv on a compacted copy of each problem's rows, one after the other"},
            "speedup_solve": seq_solve / best, "speedup_hv_round": seq_hv * 1e3 / (hv_pass_ms + advance_ms),
            "max_rel_diff_f": agree}


def cross_validation_configs(which: str = "all") -> dict:
    import torch
    import datagen as dg
    out = {}
    if which in ("all", "c4"):
        p4 = dg.config4()
        out["c4_shape"] = cross_validation(torch.from_numpy(p4.X).cuda(), torch.from_numpy(p4.y).cuda(), p4.name)
    if which == "c4":
        return out
    n, d = 20_000_000, 24
    p = dg.config5(n=n, d=d)
    X = torch.empty((n, d), dtype=torch.float64, device="cuda")
    y = torch.empty(n, dtype=torch.float64, device="cuda")
    for row0, Xc, yc in p.chunks():
        X[row0:row0 + Xc.shape[0]] = torch.from_numpy(Xc).cuda()
        y[row0:row0 + Xc.shape[0]] = torch.from_numpy(yc).cuda()
    out["20M_x_24"] = cross_validation(X, y, f"config-5 generator, {n} x {d}", reps=2)
    # twelve problems (3 folds x 4 values of C): more than the pass on the vector units holds, so the two skinny products of
    # a tile run on the fp64 matrix units
    out["20M_x_24_12_problems"] = cross_validation(X, y, f"config-5 generator, {n} x {d}", Cs=(0.03, 0.1, 0.3, 1.0), reps=2)
    return out


def stream_probe() -> dict:
    """Attainable streaming rates on this device (also the known-size kernels the byte counters are scaled with)."""
    import torch
    import paper_2008_03433_amd as tron
    probe_n = 1 << 28
    src = torch.empty(probe_n, dtype=torch.float64, device="cuda").normal_()
    ms_read, _ = tron.tron_probe_read_bandwidth(src, probe_n, reps=10)
    half = probe_n // 2
    ms_copy = tron.tron_probe_copy_bandwidth(src[half:], src[:half], half, reps=10)
    return {"read_GB/s": probe_n * 8 / (ms_read * 1e-3) / 1e9, "read_bytes": probe_n * 8,
            "copy_GB/s": 2 * half * 8 / (ms_copy * 1e-3) / 1e9, "copy_bytes_read": half * 8, "copy_bytes_written": half * 8}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    names = ["c1", "c2", "c3", "c4", "c5", "susy_shape", "higgs_shape", "c3_svm"]
    ap.add_argument("--workload", default="c3", choices=names)
    ap.add_argument("--also", default=None, choices=names + ["none"],
                    help="second workload reported under 'also' (default: c5 when the primary is c3)")
    ap.add_argument("--scale", type=float, default=1.0, help="shrink the workload (debugging only; reported)")
    ap.add_argument("--hv-reps", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--only-cv", nargs="?", const="all", default=None, choices=["all", "c4", "20M"],
                    help="run the cross-validation (multi-problem) measurements only (optionally one of the two sizes)")
    ap.add_argument("--only-active-set", action="store_true", help="run the active-set sweep (dense L2-SVM, 20M x 24) only")
    ap.add_argument("--tune", action="append", default=[], metavar="KNOB=VALUE", help="library tuning knob (see tron_tuning_set)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        return 2

    import torch
    import paper_2008_03433_amd as tron

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the library has no CPU fallback", file=sys.stderr)
        return 3
    torch.cuda.set_device(0)
    tron.load_library()
    for kv in args.tune:
        k, v_ = kv.split("=")
        tron.tron_tuning_set(k, int(v_))

    if args.only_active_set:
        print(json.dumps({"active_set": active_set_sweep(), "stream_probe": stream_probe()}), flush=True)
        return 0
    if args.only_cv:
        print(json.dumps({"cross_validation": cross_validation_configs(args.only_cv), "stream_probe": stream_probe()}), flush=True)
        return 0
    out = run_workload(args, args.workload)
    out["stream_probe"] = stream_probe()
    also = args.also if args.also is not None else ("c5" if args.workload == "c3" and args.scale == 1.0 else "none")
    if also != "none" and also != args.workload:
        sub = run_workload(args, also)
        keep = ("value", "unit", "ms_per_step", "config", "solve", "solve_preconditioned", "hv_call", "fun_grad_call", "kernels_hv", "kernels_fun_grad", "roofline", "cpu_baseline")
        out["also"] = {also: {k: sub[k] for k in keep}}
        # the second workload's rooflines travel inside the primary roofline object as well
        extra = dict(sub["roofline"])
        out["roofline"]["also"].append({k: v for k, v in extra.items() if k != "also"})
        out["roofline"]["also"] += extra.get("also", [])
    if args.workload == "c3" and args.scale == 1.0 and args.also is None:
        out["others"] = {w: small_config(args, w) for w in ("c1", "c2", "c4")}
        # the other loss / storage mixes (GPU only: their oracle solves take minutes)
        quiet = argparse.Namespace(**{**vars(args), "no_cpu_baseline": True})
        out["mixes"] = {w: small_config(quiet, w) for w in ("susy_shape", "higgs_shape", "c3_svm")}
        out["active_set"] = active_set_sweep()
        # config 3 again with the general 12-byte layout (its own layouts keep no value stream, see roofline.note)
        tron.tron_tuning_set("csr_unit", 0)
        try:
            sub = run_workload(argparse.Namespace(**{**vars(args), "no_cpu_baseline": True, "steps": 2, "warmup": 1}), "c3")
            out["c3_with_value_stream"] = {"hv_call": sub["hv_call"], "solve_ms": sub["ms_per_step"], "kernels_hv": sub["kernels_hv"],
                                           "layout": sub["layout"], "roofline": sub["roofline"]}
            for r in [sub["roofline"]] + sub["roofline"].get("also", []):
                out["roofline"]["also"].append(dict({k: v for k, v in r.items() if k != "also"},
                                                    workload=sub["config"]["workload"] + " with the value stream (csr_unit = 0)"))
        finally:
            tron.tron_tuning_set("csr_unit", 1)
        out["cross_validation"] = cross_validation_configs()
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
