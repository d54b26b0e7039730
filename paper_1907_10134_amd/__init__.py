"""MI355X-native BPPSA hot path: thin Python binding over the C-ABI library.

The functions here only marshal arguments (device pointers, sizes, the current
HIP stream) into libbppsa.so; every step of the path runs in the library's HIP
kernels.  There is no CPU fallback: if the library is not built, importing
`binding` raises.
"""
from . import binding  # noqa: F401
from .binding import (  # noqa: F401
    BppsaError, RNN_TANH, GRU, forward, head_seed, build_jacobians, scan,
    scan_workspace_bytes, param_grads, param_grads_workspace_bytes, lib_path,
    CsrMatrix, csr_conv3x3, csr_conv2d, csr_linear, csr_relu, csr_maxpool2x2, spmv, SpscanPlan, SpscanCache, spscan,
    calibration_copy, rnn_scan_fused, scan_static, scan_h20_diag, scan_h128_diag, scan_h128_schedule,
    check_scan, gru_scan_fused, gru_scan_fused_workspace_bytes, head_backward, adam_step, rnn_param_count, RnnTrainer, RNN_PARAM_ORDER,
)
