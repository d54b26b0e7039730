"""CPU-only: the C-ABI library loads, exports every symbol the header declares, and rejects
bad arguments on the host before touching a GPU."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "bppsa.h")
LIB = os.path.join(ROOT, "paper_1907_10134_amd", "libbppsa.so")


def _declared():
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    return sorted(set(re.findall(r"\b(bppsa_[a-z0-9_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        import __graft_entry__
        __graft_entry__.build()
    return ctypes.CDLL(LIB)


def test_header_declares_the_hot_path_calls():
    names = _declared()
    for must in ("bppsa_build_jacobians", "bppsa_scan", "bppsa_param_grads", "bppsa_spscan"):
        assert must in names
    assert len(names) >= 20


def test_every_declared_symbol_is_exported(lib):
    for name in _declared():
        assert hasattr(lib, name), name


def test_strerror(lib):
    lib.bppsa_strerror.restype = ctypes.c_char_p
    assert lib.bppsa_strerror(0) == b"BPPSA_OK"
    for code in range(1, 7):
        assert lib.bppsa_strerror(code).startswith(b"BPPSA_E")
    assert b"unknown" in lib.bppsa_strerror(99)


def test_workspace_queries_are_pure_host_functions(lib):
    lib.bppsa_scan_workspace_bytes.restype = ctypes.c_size_t
    lib.bppsa_param_grads_workspace_bytes.restype = ctypes.c_size_t
    small = lib.bppsa_scan_workspace_bytes(16, 2, 20)
    big = lib.bppsa_scan_workspace_bytes(30000, 16, 20)
    assert 0 < small <= big and big < 64 << 20
    assert lib.bppsa_scan_workspace_bytes(0, 2, 20) == 0
    assert lib.bppsa_scan_workspace_bytes(16, 2, 1 << 20) == 0
    assert lib.bppsa_param_grads_workspace_bytes(0, 1000, 16, 20, 1) > 0
    assert lib.bppsa_param_grads_workspace_bytes(1, 4096, 16, 128, 1) > 4096 * 16 * 4 * 128 * 4
    assert lib.bppsa_param_grads_workspace_bytes(7, 10, 1, 1, 1) == 0


def test_bad_arguments_are_rejected_before_any_launch(lib):
    null = ctypes.c_void_p()
    one = ctypes.c_void_p(256)          # a non-null pointer that is never dereferenced
    EINVAL, ESHAPE, EWORKSPACE, EOVERFLOW, EUNSUPPORTED = 1, 2, 3, 4, 6
    lib.bppsa_scan.argtypes = [ctypes.c_int] * 3 + [ctypes.c_void_p] * 5 + [ctypes.c_size_t, ctypes.c_void_p]
    assert lib.bppsa_scan(0, 1, 1, one, one, one, null, null, 0, null) == EINVAL
    assert lib.bppsa_scan(4, 1, 4, null, one, one, null, null, 0, null) == EINVAL
    assert lib.bppsa_scan(1 << 30, 1 << 20, 128, one, one, one, null, null, 0, null) == EOVERFLOW
    assert lib.bppsa_scan(100, 1, 4096, one, one, one, null, null, 0, null) == EUNSUPPORTED
    assert lib.bppsa_scan(1000, 16, 20, one, one, one, null, null, 0, null) == EWORKSPACE
    assert lib.bppsa_scan(1000, 16, 20, one, one, one, null, one, 512, null) == EWORKSPACE
    lib.bppsa_build_jacobians.argtypes = [ctypes.c_int] * 5 + [ctypes.c_void_p] * 8
    assert lib.bppsa_build_jacobians(0, 4, 1, 4, 1, null, null, null, one, null, null, one, null) == EINVAL
    assert lib.bppsa_build_jacobians(5, 4, 1, 4, 1, one, null, null, one, null, null, one, null) == EUNSUPPORTED
    assert lib.bppsa_build_jacobians(1, 4, 1, 4, 1, one, null, null, one, null, null, one, null) == EINVAL
    lib.bppsa_param_grads.argtypes = [ctypes.c_int] * 5 + [ctypes.c_void_p] * 12 + [ctypes.c_size_t, ctypes.c_void_p]
    args = [one] * 3 + [null] * 4 + [one] * 4
    assert lib.bppsa_param_grads(0, 4, 1, 4, 1, *args, null, 0, null) == EWORKSPACE
    assert lib.bppsa_param_grads(0, 4, 1, 4, 0, *args, one, 1 << 20, null) == EINVAL
    lib.bppsa_csr_maxpool2x2.argtypes = [ctypes.c_int] * 3 + [ctypes.c_void_p] * 5
    assert lib.bppsa_csr_maxpool2x2(1, 3, 4, one, one, one, one, null) == ESHAPE
    lib.bppsa_csr_conv3x3_indptr.argtypes = [ctypes.c_int] * 4 + [ctypes.c_void_p] * 3
    assert lib.bppsa_csr_conv3x3_indptr(4096, 4096, 64, 64, null, one, null) == EOVERFLOW
    geom = (ctypes.c_int32 * 8)
    lib.bppsa_csr_conv2d_indptr.argtypes = [ctypes.c_int] * 4 + [ctypes.c_void_p] * 4
    assert lib.bppsa_csr_conv2d_indptr(1, 1, 8, 8, null, null, one, null) == EINVAL                   # no geometry
    assert lib.bppsa_csr_conv2d_indptr(1, 1, 8, 8, geom(3, 3, 0, 1, 1, 1, 1, 1), null, one, null) == EINVAL   # stride 0
    assert lib.bppsa_csr_conv2d_indptr(1, 1, 8, 8, geom(3, 3, 1, 1, -1, 0, 1, 1), null, one, null) == EINVAL  # negative padding
    assert lib.bppsa_csr_conv2d_indptr(1, 1, 4, 4, geom(7, 7, 1, 1, 0, 0, 1, 1), null, one, null) == ESHAPE   # kernel larger than the image
    assert lib.bppsa_csr_conv2d_indptr(1, 1, 8, 8, geom(3, 3, 1, 1, 0, 0, 4, 1), null, one, null) == ESHAPE   # dilated kernel too tall
    assert lib.bppsa_csr_conv2d_indptr(512, 512, 64, 64, geom(5, 5, 1, 1, 2, 2, 1, 1), null, one, null) == EOVERFLOW
    lib.bppsa_adam_step.argtypes = [ctypes.c_int64] + [ctypes.c_void_p] * 4 + [ctypes.c_int] + [ctypes.c_double] * 4 + [ctypes.c_void_p]
    assert lib.bppsa_adam_step(10, one, one, one, one, 0, 1e-5, 0.9, 0.999, 1e-8, null) == EINVAL     # steps count from 1
    assert lib.bppsa_adam_step(10, one, one, one, one, 1, 1e-5, 1.0, 0.999, 1e-8, null) == EINVAL     # beta1 = 1
    lib.bppsa_head_backward.argtypes = [ctypes.c_int] * 3 + [ctypes.c_void_p] * 9
    assert lib.bppsa_head_backward(4000, 20, 10, one, one, one, one, one, null, null, null, null) == ESHAPE
    lib.bppsa_rnn_param_count.restype = ctypes.c_size_t
    assert lib.bppsa_rnn_param_count(20, 1, 10) == 20 + 400 + 40 + 200 + 10
    lib.bppsa_head_seed.argtypes = [ctypes.c_int] * 3 + [ctypes.c_void_p] * 7
    assert lib.bppsa_head_seed(1, 4, 65, one, one, one, one, one, null, null) == ESHAPE
    lib.bppsa_rnn_scan_fused.argtypes = [ctypes.c_int] * 3 + [ctypes.c_void_p] * 6 + [ctypes.c_size_t, ctypes.c_void_p]
    assert lib.bppsa_rnn_scan_fused(0, 1, 20, one, one, one, one, null, one, 1 << 30, null) == EINVAL
    assert lib.bppsa_rnn_scan_fused(8, 2, 20, null, one, one, one, null, one, 1 << 30, null) == EINVAL
    assert lib.bppsa_rnn_scan_fused(8, 2, 16, one, one, one, one, null, one, 1 << 30, null) == EUNSUPPORTED
    assert lib.bppsa_rnn_scan_fused(1000, 16, 20, one, one, one, one, null, one, 512, null) == EWORKSPACE
    assert lib.bppsa_rnn_scan_fused(1000, 16, 20, one, one, one, one, null, ctypes.c_void_p(260), 1 << 30, null) == EINVAL
    lib.bppsa_calibration_copy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p]
    assert lib.bppsa_calibration_copy(null, one, 16, null) == EINVAL
    assert lib.bppsa_calibration_copy(one, one, 0, null) == EINVAL
    assert lib.bppsa_calibration_copy(one, one, 6, null) == ESHAPE
    assert lib.bppsa_calibration_copy(ctypes.c_void_p(260), one, 16, null) == ESHAPE


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr


@pytest.mark.gpu
def test_calibration_copy_copies_exactly():
    import torch
    import paper_1907_10134_amd as bp
    src = torch.arange(4 * 100003, dtype=torch.float32, device="cuda")
    dst = torch.zeros_like(src)
    bp.calibration_copy(src, dst)
    torch.cuda.synchronize()
    assert torch.equal(src, dst)
    with pytest.raises(bp.BppsaError):
        bp.calibration_copy(src[:6], dst[:6])
