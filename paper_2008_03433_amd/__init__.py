"""MI355X-native TRON hot path (function/gradient, Hessian-vector product, full solve) for
L2-regularised logistic regression and the L2-loss SVM.

The arithmetic lives in ``libtron_hip.so`` (hand-written HIP for gfx950 behind the C ABI of
``include/tron.h``); this package is argument marshalling only.  PyTorch supplies device
memory and the stream.  There is no CPU fallback: importing works anywhere, calling needs
the built library and a GPU.
"""
from .binding import (  # noqa: F401
    LOSS_LR, LOSS_L2SVM, TronError, Dataset, SolveResult, lib_path, load_library,
    tron_dataset_create_csr, tron_dataset_create_dense, tron_dataset_create_dense_empty,
    tron_dataset_write_rows, tron_dataset_destroy, tron_dataset_shape, tron_dataset_stat, tron_fun_grad, tron_hv, tron_hv_static,
    tron_solve, tron_hess_diag, tron_last_error, tron_profile_enable, tron_profile_read, tron_probe_read_bandwidth,
    tron_probe_copy_bandwidth, tron_tuning_set, Batch, BATCH_MAX, BATCH_MAX_D, tron_batch_create, tron_batch_destroy,
    tron_batch_fun_grad, tron_batch_hv, tron_batch_solve,
)
