"""CPU-only checks of the boundary: the library loads, exports every symbol include/tron.h declares,
the Python binding covers the same names, and calls fail loudly (no fallback) without a GPU."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2008_03433_amd as tron
from paper_2008_03433_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "tron.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"TRON_API\s+[\w\s\*]+?\b(tron_\w+)\s*\(", text)))


def test_header_declares_the_three_callbacks():
    names = _declared()
    for required in ("tron_fun_grad", "tron_hv", "tron_solve", "tron_dataset_create_csr", "tron_dataset_create_dense",
                     "tron_dataset_destroy", "tron_last_error"):
        assert required in names


def test_library_exports_every_declared_symbol():
    lib = tron.load_library()
    for name in _declared():
        assert hasattr(lib, name), f"{name} is declared in include/tron.h but not exported"


def test_binding_covers_every_declared_symbol():
    for name in _declared():
        assert name in binding._SIGNATURES, f"binding has no signature for {name}"
        assert hasattr(tron, name), f"package does not expose {name}"


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2008_03433_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                src = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in src and "from oracle" not in src and "tron_oracle" not in src


def _has_gpu():
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


@pytest.mark.skipif(_has_gpu(), reason="checks the no-GPU behaviour")
def test_no_gpu_means_error_not_fallback():
    with pytest.raises(tron.TronError) as e:
        tron.tron_dataset_create_dense(4, 2, np.zeros((4, 2)), np.ones(4), stream=0)
    assert e.value.code == binding.EDEVICE
    assert "no CPU fallback" in str(e.value)


def test_argument_errors_are_reported_before_touching_the_device():
    lib = tron.load_library()
    out = ctypes.c_void_p()
    assert lib.tron_dataset_create_csr(0, 5, None, None, None, None, 0, None, ctypes.byref(out)) == binding.EINVAL
    assert lib.tron_dataset_create_dense(4, 2, None, None, 0, None, ctypes.byref(out)) == binding.EINVAL
    assert lib.tron_fun_grad(None, 0, 1.0, None, None, None) == binding.EINVAL
    assert lib.tron_hv(None, 1.0, None, None, None) == binding.EINVAL
    assert lib.tron_solve(None, None, None, None) == binding.EINVAL
    assert lib.tron_tuning_set(b"no_such_knob", 1) == binding.EINVAL
    assert "tron_tuning_set" in tron.tron_last_error()
    assert lib.tron_batch_create(None, 3, None, 0, ctypes.byref(out)) == binding.EINVAL
    assert lib.tron_batch_fun_grad(None, 0, None, None, None, None) == binding.EINVAL
    assert lib.tron_batch_hv(None, None, None, None, None) == binding.EINVAL
    assert lib.tron_batch_solve(None, None, None, None, None, None) == binding.EINVAL
    lib.tron_batch_destroy(None)
    lib.tron_dataset_destroy(None)  # NULL is ignored
