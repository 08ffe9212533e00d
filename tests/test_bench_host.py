"""Host logic of bench.py that needs no GPU: the committed rocprofv3 summaries are read back as bytes per launch."""
import importlib.util
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench():
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_traffic_is_read_from_the_committed_summaries_in_bytes():
    b = _bench()
    # what the kernels of each profiled workload move per launch lies between a few MB and a few tens of GB, and
    # within a factor of two of known sizes: c5 is 44.2 GB of matrix, the tile kernel of c3 without values reads 0.42 GB
    seen = {}
    for (workload, slot) in b.ROCPROF_NAMES:
        t = b.measured_traffic(workload, slot)
        assert t is not None and 1e6 < t < 1e11, (workload, slot, t)
        seen[(workload, slot)] = t
    assert 0.9 < seen[("c5", "dense_hv")] / (8.0 * 230_000_000 * 24) < 1.1
    assert 0.3e9 < seen[("c3", "spmv_tiles")] < 0.6e9
    assert seen[("c3_values", "spmv_tiles")] > 2.0 * seen[("c3", "spmv_tiles")]   # the value stream triples the bytes
    assert b.measured_traffic(None, "spmv_tiles") is None and b.measured_traffic("c3", "no_such_kernel") is None


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in (r.stdout + r.stderr)
