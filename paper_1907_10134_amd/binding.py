"""ctypes binding with the same names as the C ABI in include/bppsa.h.

Argument marshalling only.  Tensors must be fp32 (int32 for labels / indices),
contiguous and resident on the GPU; PyTorch supplies device memory and the
stream, nothing else.
"""
from __future__ import annotations

import ctypes
import os

import torch

RNN_TANH = 0
GRU = 1

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libbppsa.so")


class BppsaError(RuntimeError):
    def __init__(self, code, where, detail=None):
        self.code = code
        super().__init__("%s failed: %s" % (where, detail or _lib.bppsa_strerror(code).decode()))


def _load(path=_LIB_PATH):
    if not os.path.exists(path):
        raise ImportError(
            "libbppsa.so is not built (expected at %s); run "
            "`python -c 'import __graft_entry__ as g; g.build()'` first - there is no "
            "CPU fallback" % path)
    lib = ctypes.CDLL(path)
    c_int, c_void_p, c_size_t = ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t
    lib.bppsa_strerror.restype = ctypes.c_char_p
    lib.bppsa_strerror.argtypes = [c_int]
    lib.bppsa_forward.restype = c_int
    lib.bppsa_forward.argtypes = [c_int] * 5 + [c_void_p] * 7
    lib.bppsa_head_seed.restype = c_int
    lib.bppsa_head_seed.argtypes = [c_int] * 3 + [c_void_p] * 7
    lib.bppsa_build_jacobians.restype = c_int
    lib.bppsa_build_jacobians.argtypes = [c_int] * 5 + [c_void_p] * 8
    lib.bppsa_scan_workspace_bytes.restype = c_size_t
    lib.bppsa_scan_workspace_bytes.argtypes = [c_int] * 3
    lib.bppsa_scan.restype = c_int
    lib.bppsa_scan.argtypes = [c_int] * 3 + [c_void_p] * 5 + [c_size_t, c_void_p]
    lib.bppsa_scan_h20_diag.restype = c_int
    lib.bppsa_scan_h20_diag.argtypes = [c_int] * 2 + [c_void_p] * 5 + [c_size_t, c_void_p, c_int, c_int, c_void_p]
    lib.bppsa_scan_h128_diag.restype = c_int
    lib.bppsa_scan_h128_diag.argtypes = [c_int] * 2 + [c_void_p] * 5 + [c_size_t, c_void_p, c_int, c_int, c_int]
    lib.bppsa_scan_h128_schedule.restype = c_int
    lib.bppsa_scan_h128_schedule.argtypes = [c_int] * 4 + [ctypes.POINTER(H128Schedule)]
    lib.bppsa_scan_static.restype = c_int
    lib.bppsa_scan_static.argtypes = [c_int] * 3 + [c_void_p] * 5
    lib.bppsa_rnn_scan_fused.restype = c_int
    lib.bppsa_rnn_scan_fused.argtypes = [c_int] * 3 + [c_void_p] * 6 + [c_size_t, c_void_p]
    lib.bppsa_param_grads_workspace_bytes.restype = c_size_t
    lib.bppsa_param_grads_workspace_bytes.argtypes = [c_int] * 5
    lib.bppsa_param_grads.restype = c_int
    lib.bppsa_param_grads.argtypes = [c_int] * 5 + [c_void_p] * 12 + [c_size_t, c_void_p]
    c_i32p = c_void_p
    lib.bppsa_csr_conv3x3_indptr.restype = c_int
    lib.bppsa_csr_conv3x3_indptr.argtypes = [c_int] * 4 + [c_void_p] * 3
    lib.bppsa_csr_conv3x3_fill.restype = c_int
    lib.bppsa_csr_conv3x3_fill.argtypes = [c_int] * 4 + [c_void_p] * 6
    lib.bppsa_csr_conv2d_indptr.restype = c_int
    lib.bppsa_csr_conv2d_indptr.argtypes = [c_int] * 4 + [ctypes.POINTER(Conv2dGeometry)] + [c_void_p] * 3
    lib.bppsa_csr_conv2d_fill.restype = c_int
    lib.bppsa_csr_conv2d_fill.argtypes = [c_int] * 4 + [ctypes.POINTER(Conv2dGeometry)] + [c_void_p] * 6
    lib.bppsa_csr_relu.restype = c_int
    lib.bppsa_csr_relu.argtypes = [c_int] + [c_void_p] * 5
    lib.bppsa_csr_maxpool2x2.restype = c_int
    lib.bppsa_csr_maxpool2x2.argtypes = [c_int] * 3 + [c_void_p] * 5
    lib.bppsa_csr_linear_indptr.restype = c_int
    lib.bppsa_csr_linear_indptr.argtypes = [c_int] * 2 + [c_void_p] * 3
    lib.bppsa_csr_linear_fill.restype = c_int
    lib.bppsa_csr_linear_fill.argtypes = [c_int] * 2 + [c_void_p] * 6
    lib.bppsa_spmv.restype = c_int
    lib.bppsa_spmv.argtypes = [ctypes.POINTER(CsrDesc), c_void_p, c_void_p, c_void_p]
    lib.bppsa_spscan_plan_create.restype = c_int
    lib.bppsa_spscan_plan_create.argtypes = [c_int, ctypes.POINTER(CsrDesc), c_int, c_void_p, c_size_t,
                                             c_void_p, ctypes.POINTER(c_void_p)]
    lib.bppsa_spscan_plan_destroy.restype = None
    lib.bppsa_spscan_plan_destroy.argtypes = [c_void_p]
    lib.bppsa_spscan_plan_arena_used.restype = c_size_t
    lib.bppsa_spscan_plan_arena_used.argtypes = [c_void_p]
    lib.bppsa_spscan_plan_num_products.restype = c_int
    lib.bppsa_spscan_plan_num_products.argtypes = [c_void_p]
    lib.bppsa_spscan_plan_product.restype = c_int
    lib.bppsa_spscan_plan_product.argtypes = [c_void_p, c_int, ctypes.POINTER(CsrDesc),
                                              ctypes.POINTER(c_int), ctypes.POINTER(c_int)]
    lib.bppsa_spscan_plan_flops.restype = c_int
    lib.bppsa_spscan_plan_flops.argtypes = [c_void_p, ctypes.POINTER(ctypes.c_int64),
                                            ctypes.POINTER(ctypes.c_int64)]
    c_double = ctypes.c_double
    lib.bppsa_gru_scan_fused_workspace_bytes.restype = c_size_t
    lib.bppsa_gru_scan_fused_workspace_bytes.argtypes = [c_int] * 3
    lib.bppsa_gru_scan_fused.restype = c_int
    lib.bppsa_gru_scan_fused.argtypes = [c_int] * 4 + [c_void_p] * 10 + [c_size_t, c_void_p]
    lib.bppsa_head_backward.restype = c_int
    lib.bppsa_head_backward.argtypes = [c_int] * 3 + [c_void_p] * 8 + [c_void_p]
    lib.bppsa_adam_step.restype = c_int
    lib.bppsa_adam_step.argtypes = [ctypes.c_int64] + [c_void_p] * 4 + [c_int] + [c_double] * 4 + [c_void_p]
    lib.bppsa_rnn_param_count.restype = c_size_t
    lib.bppsa_rnn_param_count.argtypes = [c_int] * 3
    lib.bppsa_rnn_train_workspace_bytes.restype = c_size_t
    lib.bppsa_rnn_train_workspace_bytes.argtypes = [c_int] * 4
    lib.bppsa_rnn_train_step.restype = c_int
    lib.bppsa_rnn_train_step.argtypes = [c_int] * 5 + [c_void_p, c_void_p, ctypes.POINTER(RnnTrainState), c_int] + \
        [c_double] * 4 + [c_void_p]
    lib.bppsa_spscan_plan_num_steps.restype = c_int
    lib.bppsa_spscan_plan_num_steps.argtypes = [c_void_p]
    lib.bppsa_spscan_plan_step_flops.restype = c_int
    lib.bppsa_spscan_plan_step_flops.argtypes = [c_void_p, c_int, ctypes.POINTER(SpscanStep)]
    lib.bppsa_spscan_cache_create.restype = c_int
    lib.bppsa_spscan_cache_create.argtypes = [ctypes.POINTER(c_void_p)]
    lib.bppsa_spscan_cache_destroy.restype = None
    lib.bppsa_spscan_cache_destroy.argtypes = [c_void_p]
    lib.bppsa_spscan_cache_stats.restype = c_int
    lib.bppsa_spscan_cache_stats.argtypes = [c_void_p, ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int64),
                                             ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(c_size_t)]
    lib.bppsa_spscan_plan_create_cached.restype = c_int
    lib.bppsa_spscan_plan_create_cached.argtypes = [c_void_p, c_int, ctypes.POINTER(CsrDesc), c_int, c_void_p,
                                                    c_size_t, c_void_p, ctypes.POINTER(c_void_p)]
    lib.bppsa_spscan_run.restype = c_int
    lib.bppsa_spscan_run.argtypes = [c_void_p, ctypes.POINTER(CsrDesc), c_void_p,
                                     ctypes.POINTER(c_void_p), c_void_p]
    lib.bppsa_spscan.restype = c_int
    lib.bppsa_spscan.argtypes = [c_int, ctypes.POINTER(CsrDesc), c_void_p, ctypes.POINTER(c_void_p),
                                 c_int, c_void_p, c_size_t, c_void_p]
    lib.bppsa_calibration_copy.restype = c_int
    lib.bppsa_calibration_copy.argtypes = [c_void_p, c_void_p, ctypes.c_int64, c_void_p]
    return lib


class CsrDesc(ctypes.Structure):
    """Mirror of the C struct bppsa_csr (host struct, device array pointers)."""
    _fields_ = [("rows", ctypes.c_int32), ("cols", ctypes.c_int32), ("nnz", ctypes.c_int64),
                ("indptr", ctypes.c_void_p), ("indices", ctypes.c_void_p), ("data", ctypes.c_void_p)]


class H128Schedule(ctypes.Structure):
    """bppsa_h128_schedule."""
    _fields_ = [(k, ctypes.c_int32) for k in ("segment_steps", "segments", "chain_steps", "slab_segments", "slabs",
                                              "last_slab_steps")] + \
               [("matrix_products", ctypes.c_int64), ("model_us", ctypes.c_double)]


class Conv2dGeometry(ctypes.Structure):
    """Mirror of the C struct bppsa_conv2d_geometry."""
    _fields_ = [(k, ctypes.c_int32) for k in ("kh", "kw", "stride_h", "stride_w", "pad_h", "pad_w", "dil_h", "dil_w")]


class RnnTrainState(ctypes.Structure):
    """Mirror of the C struct bppsa_rnn_train_state (host struct, device pointers)."""
    _fields_ = [(k, ctypes.c_void_p) for k in ("params", "grads", "adam_m", "adam_v", "h", "G", "seed", "loss",
                                                "Jt", "workspace")] + [("workspace_bytes", ctypes.c_size_t)]


class SpscanStep(ctypes.Structure):
    """Mirror of the C struct bppsa_spscan_step."""
    _fields_ = [("kind", ctypes.c_int32), ("phase", ctypes.c_int32), ("level", ctypes.c_int32),
                ("matrix", ctypes.c_int32), ("flops", ctypes.c_int64), ("numeric_kind", ctypes.c_int32)]


_lib = _load()


def lib_path() -> str:
    return _LIB_PATH


def _ptr(t, dtype=torch.float32, name="tensor"):
    if t is None:
        return None
    if not isinstance(t, torch.Tensor):
        raise TypeError("%s must be a torch.Tensor" % name)
    if not t.is_cuda:
        raise ValueError("%s must live on the GPU" % name)
    if t.dtype != dtype:
        raise ValueError("%s must be %s, got %s" % (name, dtype, t.dtype))
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    return t.data_ptr()


def _stream(stream=None):
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream


def _check(code, where):
    if code != 0:
        raise BppsaError(code, where)


def _workspace(nbytes, device, stream=None):
    # 256-byte aligned by the caching allocator (its blocks are 512-byte aligned).  A workspace
    # made here for a stream other than the current one is tied to that stream, so the allocator
    # does not hand its memory out again while the call is still running there.
    ws = torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)
    if stream is not None and stream != torch.cuda.current_stream(device):
        ws.record_stream(stream)
    return ws


_last_h20_workspace = None      # the workspace of the latest H = 20 scan that allocated its own


def check_scan(workspace=None):
    """Synchronise and read the error word of an H = 20 scan's workspace (its first 4 bytes): raises
    BppsaError if a bounded wait inside the kernel expired, in which case G is invalid.  With no
    argument, checks the workspace the latest scan()/rnn_scan_fused() call allocated for itself."""
    ws = _last_h20_workspace if workspace is None else workspace
    if ws is None:
        return
    torch.cuda.synchronize(ws.device)
    if int(ws[:4].view(torch.int32).item()) != 0:
        raise BppsaError(5, "bppsa_scan", "a bounded wait inside the H = 20 scan expired; G is invalid")


def forward(cell, x, w_ih, w_hh, b_ih, b_hh, h, stream=None):
    """bppsa_forward: fills h[1..T] from h[0], x and the weights.  h is [T+1,B,H]."""
    T1, B, H = h.shape
    I = x.shape[2]
    _check(_lib.bppsa_forward(cell, T1 - 1, B, H, I, _ptr(x), _ptr(w_ih), _ptr(w_hh),
                              _ptr(b_ih), _ptr(b_hh), _ptr(h), _stream(stream)), "bppsa_forward")
    return h


def head_seed(h_last, w_out, b_out, labels, seed=None, loss=None, stream=None):
    """bppsa_head_seed: seed[B,H] = dL/dh_T of the softmax cross-entropy head."""
    B, H = h_last.shape
    C = w_out.shape[0]
    if seed is None:
        seed = torch.empty((B, H), dtype=torch.float32, device=h_last.device)
    if loss is None:
        loss = torch.empty((1,), dtype=torch.float32, device=h_last.device)
    _check(_lib.bppsa_head_seed(B, H, C, _ptr(h_last), _ptr(w_out), _ptr(b_out),
                                _ptr(labels, torch.int32), _ptr(seed), _ptr(loss),
                                _stream(stream)), "bppsa_head_seed")
    return seed, loss


def build_jacobians(cell, h, x=None, w_ih=None, w_hh=None, b_ih=None, b_hh=None, Jt=None,
                    stream=None):
    """bppsa_build_jacobians: Jt[T,B,H,H], Jt[t] = (dh[t+1]/dh[t])^T."""
    T1, B, H = h.shape
    T = T1 - 1
    I = x.shape[2] if x is not None else 1
    if Jt is None:
        Jt = torch.empty((T, B, H, H), dtype=torch.float32, device=h.device)
    _check(_lib.bppsa_build_jacobians(cell, T, B, H, I, _ptr(h), _ptr(x), _ptr(w_ih), _ptr(w_hh),
                                      _ptr(b_ih), _ptr(b_hh), _ptr(Jt), _stream(stream)),
           "bppsa_build_jacobians")
    return Jt


def scan_workspace_bytes(T, B, H):
    return int(_lib.bppsa_scan_workspace_bytes(T, B, H))


def scan(Jt, seed, G=None, g0=None, workspace=None, stream=None):
    """bppsa_scan: G[t-1] = dL/dh[t], t = 1..T; optional g0 = dL/dh[0]."""
    T, B, H, _ = Jt.shape
    if G is None:
        G = torch.empty((T, B, H), dtype=torch.float32, device=Jt.device)
    if workspace is None:
        workspace = _workspace(scan_workspace_bytes(T, B, H), Jt.device, stream)
        if H == 20:
            global _last_h20_workspace
            _last_h20_workspace = workspace
    _check(_lib.bppsa_scan(T, B, H, _ptr(Jt), _ptr(seed), _ptr(G), _ptr(g0),
                           workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                           _stream(stream)), "bppsa_scan")
    return G


def scan_h20_diag(Jt, seed, G=None, g0=None, workspace=None, stream=None, absent_dies=0, unit_halves=0,
                  lookback_stats=None):
    """bppsa_scan_h20_diag: the H = 20 scan with chosen dies standing aside / a forced unit length;
    lookback_stats, if given, is an int64 tensor of 3 that receives (hops, look-backs, max hops)."""
    T, B, H, _ = Jt.shape
    if G is None:
        G = torch.empty((T, B, H), dtype=torch.float32, device=Jt.device)
    if workspace is None:
        workspace = _workspace(scan_workspace_bytes(T, B, H), Jt.device)
    _check(_lib.bppsa_scan_h20_diag(T, B, _ptr(Jt), _ptr(seed), _ptr(G), _ptr(g0), workspace.data_ptr(),
                                    workspace.numel() * workspace.element_size(), _stream(stream),
                                    int(absent_dies), int(unit_halves), _ptr(lookback_stats, torch.int64)),
           "bppsa_scan_h20_diag")
    return G


def scan_h128_diag(Jt, seed, G=None, g0=None, workspace=None, stream=None, chain_segments=0, slab_segments=0,
                   last_slab_steps=0):
    """bppsa_scan_h128_diag: the H = 128 scan with a forced schedule (segments walked by the serial
    chain, segments per slab of totals, segment length inside the last slab)."""
    T, B, H, _ = Jt.shape
    if G is None:
        G = torch.empty((T, B, H), dtype=torch.float32, device=Jt.device)
    if workspace is None:
        workspace = _workspace(scan_workspace_bytes(T, B, H), Jt.device, stream)
    _check(_lib.bppsa_scan_h128_diag(T, B, _ptr(Jt), _ptr(seed), _ptr(G), _ptr(g0), workspace.data_ptr(),
                                     workspace.numel() * workspace.element_size(), _stream(stream),
                                     int(chain_segments), int(slab_segments), int(last_slab_steps)),
           "bppsa_scan_h128_diag")
    return G


def scan_h128_schedule(T, B, want_g0=False, generated=False):
    """bppsa_scan_h128_schedule as a dict: how bppsa_scan (or bppsa_gru_scan_fused) walks such a chain."""
    out = H128Schedule()
    _check(_lib.bppsa_scan_h128_schedule(int(T), int(B), int(bool(want_g0)), int(bool(generated)), ctypes.byref(out)),
           "bppsa_scan_h128_schedule")
    return {name: getattr(out, name) for name, _ in H128Schedule._fields_}


def scan_static(Jt, seed, G, g0=None, stream=None):
    """bppsa_scan_static: bppsa_scan on the library's fixed scratch array; allocates nothing,
    so G (and g0) must be passed in."""
    T, B, H, _ = Jt.shape
    _check(_lib.bppsa_scan_static(T, B, H, _ptr(Jt), _ptr(seed), _ptr(G), _ptr(g0), _stream(stream)),
           "bppsa_scan_static")
    return G


def rnn_scan_fused(h, w_hh, seed, G=None, g0=None, workspace=None, stream=None):
    """bppsa_rnn_scan_fused: the tanh-RNN scan with the Jacobians generated in the kernel."""
    T1, B, H = h.shape
    T = T1 - 1
    if G is None:
        G = torch.empty((T, B, H), dtype=torch.float32, device=h.device)
    if workspace is None:
        workspace = _workspace(scan_workspace_bytes(T, B, H), h.device, stream)
        global _last_h20_workspace
        _last_h20_workspace = workspace
    _check(_lib.bppsa_rnn_scan_fused(T, B, H, _ptr(h, name="h"), _ptr(w_hh, name="w_hh"), _ptr(seed, name="seed"),
                                     _ptr(G, name="G"), _ptr(g0),
                                     workspace.data_ptr(), workspace.numel(), _stream(stream)),
           "bppsa_rnn_scan_fused")
    return G


def gru_scan_fused_workspace_bytes(T, B, H):
    return int(_lib.bppsa_gru_scan_fused_workspace_bytes(T, B, H))


def gru_scan_fused(h, x, w_ih, w_hh, b_ih, b_hh, seed, G=None, g0=None, workspace=None, stream=None):
    """bppsa_gru_scan_fused: the H = 128 GRU scan with the Jacobians generated inside its kernels."""
    T1, B, H = h.shape
    T = T1 - 1
    I = x.shape[2]
    if G is None:
        G = torch.empty((T, B, H), dtype=torch.float32, device=h.device)
    if workspace is None:
        workspace = _workspace(gru_scan_fused_workspace_bytes(T, B, H), h.device)
    _check(_lib.bppsa_gru_scan_fused(T, B, H, I, _ptr(h, name="h"), _ptr(x, name="x"), _ptr(w_ih), _ptr(w_hh),
                                     _ptr(b_ih), _ptr(b_hh), _ptr(seed, name="seed"), _ptr(G, name="G"), _ptr(g0),
                                     workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                     _stream(stream)), "bppsa_gru_scan_fused")
    return G


def param_grads_workspace_bytes(cell, T, B, H, I):
    return int(_lib.bppsa_param_grads_workspace_bytes(cell, T, B, H, I))


def param_grads(cell, h, x, G, w_ih=None, w_hh=None, b_ih=None, b_hh=None, out=None,
                workspace=None, stream=None):
    """bppsa_param_grads: returns (dW_ih, dW_hh, db_ih, db_hh)."""
    T1, B, H = h.shape
    T = T1 - 1
    I = x.shape[2]
    R = H if cell == RNN_TANH else 3 * H
    dev = h.device
    if out is None:
        out = (torch.empty((R, I), dtype=torch.float32, device=dev),
               torch.empty((R, H), dtype=torch.float32, device=dev),
               torch.empty((R,), dtype=torch.float32, device=dev),
               torch.empty((R,), dtype=torch.float32, device=dev))
    if workspace is None:
        workspace = _workspace(param_grads_workspace_bytes(cell, T, B, H, I), dev)
    dW_ih, dW_hh, db_ih, db_hh = out
    _check(_lib.bppsa_param_grads(cell, T, B, H, I, _ptr(h), _ptr(x), _ptr(G), _ptr(w_ih),
                                  _ptr(w_hh), _ptr(b_ih), _ptr(b_hh), _ptr(dW_ih), _ptr(dW_hh),
                                  _ptr(db_ih), _ptr(db_hh), workspace.data_ptr(),
                                  workspace.numel() * workspace.element_size(), _stream(stream)),
           "bppsa_param_grads")
    return out


# --------------------------------------------------------------------------
# Training iteration
# --------------------------------------------------------------------------

def head_backward(h_last, w_out, b_out, labels, seed=None, loss=None, dW_out=None, db_out=None, stream=None):
    """bppsa_head_backward: (seed, loss, dW_out, db_out) of the softmax cross-entropy head."""
    B, H = h_last.shape
    C = w_out.shape[0]
    dev = h_last.device
    seed = torch.empty((B, H), dtype=torch.float32, device=dev) if seed is None else seed
    loss = torch.empty((1,), dtype=torch.float32, device=dev) if loss is None else loss
    dW_out = torch.empty((C, H), dtype=torch.float32, device=dev) if dW_out is None else dW_out
    db_out = torch.empty((C,), dtype=torch.float32, device=dev) if db_out is None else db_out
    _check(_lib.bppsa_head_backward(B, H, C, _ptr(h_last), _ptr(w_out), _ptr(b_out), _ptr(labels, torch.int32),
                                    _ptr(seed), _ptr(loss), _ptr(dW_out), _ptr(db_out), _stream(stream)),
           "bppsa_head_backward")
    return seed, loss, dW_out, db_out


def adam_step(theta, grad, m, v, step, lr=1e-5, beta1=0.9, beta2=0.999, eps=1e-8, stream=None):
    """bppsa_adam_step: in-place update of theta, m, v (flat fp32 tensors of equal length)."""
    _check(_lib.bppsa_adam_step(theta.numel(), _ptr(theta), _ptr(grad), _ptr(m), _ptr(v), int(step), lr, beta1,
                                beta2, eps, _stream(stream)), "bppsa_adam_step")
    return theta


def rnn_param_count(H, I, C):
    return int(_lib.bppsa_rnn_param_count(H, I, C))


RNN_PARAM_ORDER = ("w_ih", "w_hh", "b_ih", "b_hh", "w_out", "b_out")


def rnn_param_shapes(H, I, C):
    return {"w_ih": (H, I), "w_hh": (H, H), "b_ih": (H,), "b_hh": (H,), "w_out": (C, H), "b_out": (C,)}


class RnnTrainer:
    """Device buffers of bppsa_rnn_train_step for fixed (T, B, H, I, C); step() enqueues one iteration.

    params / grads / adam_m / adam_v are flat tensors in the library's layout (views(name) gives the
    shaped view of one parameter); with materialise=False the H = 20 scan generates the Jacobians
    itself and no Jt buffer exists."""

    def __init__(self, T, B, H, I, C, params, materialise=True, device="cuda"):
        self.dims = (T, B, H, I, C)
        n = rnn_param_count(H, I, C)
        f32 = dict(dtype=torch.float32, device=device)
        self.params = torch.cat([params[k].reshape(-1).to(**f32) for k in RNN_PARAM_ORDER]).contiguous()
        assert self.params.numel() == n
        self.grads = torch.zeros((n,), **f32)
        self.adam_m = torch.zeros((n,), **f32)
        self.adam_v = torch.zeros((n,), **f32)
        self.h = torch.zeros((T + 1, B, H), **f32)
        self.G = torch.empty((T, B, H), **f32)
        self.seed = torch.empty((B, H), **f32)
        self.loss = torch.zeros((1,), **f32)
        self.Jt = torch.empty((T, B, H, H), **f32) if materialise else None
        self.workspace = _workspace(int(_lib.bppsa_rnn_train_workspace_bytes(T, B, H, I)), torch.device(device))
        self.t = 0
        self._st = RnnTrainState(self.params.data_ptr(), self.grads.data_ptr(), self.adam_m.data_ptr(),
                                 self.adam_v.data_ptr(), self.h.data_ptr(), self.G.data_ptr(), self.seed.data_ptr(),
                                 self.loss.data_ptr(), self.Jt.data_ptr() if materialise else None,
                                 self.workspace.data_ptr(), self.workspace.numel() * self.workspace.element_size())

    def view(self, flat, name):
        T, B, H, I, C = self.dims
        off = 0
        for k in RNN_PARAM_ORDER:
            shape = rnn_param_shapes(H, I, C)[k]
            size = 1
            for d in shape:
                size *= d
            if k == name:
                return flat[off:off + size].view(shape)
            off += size
        raise KeyError(name)

    def step(self, x, labels, lr=1e-5, beta1=0.9, beta2=0.999, eps=1e-8, stream=None):
        T, B, H, I, C = self.dims
        self.t += 1
        _check(_lib.bppsa_rnn_train_step(T, B, H, I, C, _ptr(x), _ptr(labels, torch.int32), ctypes.byref(self._st),
                                         self.t, lr, beta1, beta2, eps, _stream(stream)), "bppsa_rnn_train_step")
        return self.loss


# --------------------------------------------------------------------------
# Sparse path
# --------------------------------------------------------------------------

class CsrMatrix:
    """Device CSR arrays (int32 indptr/indices, fp32 data) plus the shape."""

    def __init__(self, rows, cols, indptr, indices, data):
        self.rows, self.cols = int(rows), int(cols)
        self.indptr, self.indices, self.data = indptr, indices, data
        self.nnz = int(indices.numel())

    def desc(self):
        return CsrDesc(self.rows, self.cols, self.nnz, _ptr(self.indptr, torch.int32),
                       _ptr(self.indices, torch.int32) if self.nnz else None,
                       _ptr(self.data) if self.nnz else None)


def _i32(n, dev):
    return torch.empty((max(int(n), 1),), dtype=torch.int32, device=dev)[:int(n)]


def _two_call(rows, cols, dev, call_indptr, call_fill):
    indptr = torch.empty((rows + 1,), dtype=torch.int32, device=dev)
    call_indptr(indptr)
    nnz = int(indptr[-1].item())          # the two-call pattern: read nnz, then size the arrays
    indices = torch.empty((nnz,), dtype=torch.int32, device=dev)
    data = torch.empty((nnz,), dtype=torch.float32, device=dev)
    if nnz:
        call_fill(indptr, indices, data)
    return CsrMatrix(rows, cols, indptr, indices, data)


def csr_conv3x3(weight, mask, h, w, stream=None):
    """bppsa_csr_conv3x3_indptr + _fill.  weight [co,ci,3,3] fp32, mask same shape uint8 or None."""
    co, ci = weight.shape[:2]
    st = _stream(stream)
    mp = _ptr(mask, torch.uint8, "mask")
    return _two_call(
        ci * h * w, co * h * w, weight.device,
        lambda ip: _check(_lib.bppsa_csr_conv3x3_indptr(ci, co, h, w, mp, _ptr(ip, torch.int32), st),
                          "bppsa_csr_conv3x3_indptr"),
        lambda ip, ix, d: _check(_lib.bppsa_csr_conv3x3_fill(ci, co, h, w, _ptr(weight), mp,
                                                             _ptr(ip, torch.int32), _ptr(ix, torch.int32),
                                                             _ptr(d), st), "bppsa_csr_conv3x3_fill"))


def csr_conv2d(weight, mask, h, w, stride=(1, 1), padding=(0, 0), dilation=(1, 1), stream=None):
    """bppsa_csr_conv2d_indptr + _fill.  weight [co,ci,kh,kw] fp32, mask same shape uint8 or None."""
    co, ci, kh, kw = weight.shape
    g = Conv2dGeometry(kh, kw, stride[0], stride[1], padding[0], padding[1], dilation[0], dilation[1])
    oh = (h + 2 * padding[0] - dilation[0] * (kh - 1) - 1) // stride[0] + 1
    ow = (w + 2 * padding[1] - dilation[1] * (kw - 1) - 1) // stride[1] + 1
    st = _stream(stream)
    mp = _ptr(mask, torch.uint8, "mask")
    return _two_call(
        ci * h * w, co * max(oh, 0) * max(ow, 0), weight.device,
        lambda ip: _check(_lib.bppsa_csr_conv2d_indptr(ci, co, h, w, ctypes.byref(g), mp, _ptr(ip, torch.int32), st),
                          "bppsa_csr_conv2d_indptr"),
        lambda ip, ix, d: _check(_lib.bppsa_csr_conv2d_fill(ci, co, h, w, ctypes.byref(g), _ptr(weight), mp,
                                                            _ptr(ip, torch.int32), _ptr(ix, torch.int32),
                                                            _ptr(d), st), "bppsa_csr_conv2d_fill"))


def csr_linear(weight, mask, stream=None):
    """bppsa_csr_linear_indptr + _fill.  weight [out,in]."""
    out, inn = weight.shape
    st = _stream(stream)
    mp = _ptr(mask, torch.uint8, "mask")
    return _two_call(
        inn, out, weight.device,
        lambda ip: _check(_lib.bppsa_csr_linear_indptr(out, inn, mp, _ptr(ip, torch.int32), st),
                          "bppsa_csr_linear_indptr"),
        lambda ip, ix, d: _check(_lib.bppsa_csr_linear_fill(out, inn, _ptr(weight), mp, _ptr(ip, torch.int32),
                                                            _ptr(ix, torch.int32), _ptr(d), st),
                                 "bppsa_csr_linear_fill"))


def csr_relu(x, stream=None):
    d = x.numel()
    dev = x.device
    indptr = torch.empty((d + 1,), dtype=torch.int32, device=dev)
    indices = torch.empty((d,), dtype=torch.int32, device=dev)
    data = torch.empty((d,), dtype=torch.float32, device=dev)
    _check(_lib.bppsa_csr_relu(d, _ptr(x), _ptr(indptr, torch.int32), _ptr(indices, torch.int32), _ptr(data),
                               _stream(stream)), "bppsa_csr_relu")
    return CsrMatrix(d, d, indptr, indices, data)


def csr_maxpool2x2(x, stream=None):
    c, h, w = x.shape
    dev = x.device
    n_out = c * (h // 2) * (w // 2)
    indptr = torch.empty((c * h * w + 1,), dtype=torch.int32, device=dev)
    indices = torch.empty((n_out,), dtype=torch.int32, device=dev)
    data = torch.empty((n_out,), dtype=torch.float32, device=dev)
    _check(_lib.bppsa_csr_maxpool2x2(c, h, w, _ptr(x), _ptr(indptr, torch.int32), _ptr(indices, torch.int32),
                                     _ptr(data), _stream(stream)), "bppsa_csr_maxpool2x2")
    return CsrMatrix(c * h * w, n_out, indptr, indices, data)


def spmv(A, x, y=None, stream=None):
    if y is None:
        y = torch.empty((A.rows,), dtype=torch.float32, device=x.device)
    d = A.desc()
    _check(_lib.bppsa_spmv(ctypes.byref(d), _ptr(x), _ptr(y), _stream(stream)), "bppsa_spmv")
    return y


def _desc_array(jts):
    arr = (CsrDesc * len(jts))()
    for k, m in enumerate(jts):
        arr[k] = m.desc()
    return arr


def _grads_array(grads):
    arr = (ctypes.c_void_p * len(grads))()
    for k, g in enumerate(grads):
        arr[k] = None if g is None else _ptr(g)
    return arr


class SpscanCache:
    """Host handle of bppsa_spscan_cache_create: symbolic phases kept across plans."""

    def __init__(self):
        self._h = ctypes.c_void_p()
        _check(_lib.bppsa_spscan_cache_create(ctypes.byref(self._h)), "bppsa_spscan_cache_create")

    def stats(self):
        """(plans served from the cache, plans that ran the symbolic phase, products computed, device bytes)."""
        h, m, p, b = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64(), ctypes.c_size_t()
        _check(_lib.bppsa_spscan_cache_stats(self._h, ctypes.byref(h), ctypes.byref(m), ctypes.byref(p),
                                             ctypes.byref(b)), "bppsa_spscan_cache_stats")
        return h.value, m.value, p.value, b.value

    def close(self):
        if self._h:
            _lib.bppsa_spscan_cache_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        self.close()


class _DeviceArray:
    """Device memory owned by the library, exposed to torch.as_tensor without a copy."""

    def __init__(self, ptr, count, typestr, owner):
        self.owner = owner
        self.__cuda_array_interface__ = {"shape": (count,), "typestr": typestr, "data": (ptr, False),
                                         "version": 2, "strides": None}


class SpscanPlan:
    """Host handle of bppsa_spscan_plan_create (or, with `cache`, bppsa_spscan_plan_create_cached);
    device storage lives in `arena` (a uint8 tensor) and, for the product structures of a cached
    plan, in the cache."""

    def __init__(self, jts, up_levels, arena, stream=None, cache=None):
        self.n = len(jts)
        self.arena = arena
        self.cache = cache
        self._h = ctypes.c_void_p()
        descs = _desc_array(jts)
        if cache is None:
            _check(_lib.bppsa_spscan_plan_create(self.n, descs, int(up_levels), arena.data_ptr(),
                                                 arena.numel(), _stream(stream), ctypes.byref(self._h)),
                   "bppsa_spscan_plan_create")
        else:
            _check(_lib.bppsa_spscan_plan_create_cached(cache._h, self.n, descs, int(up_levels), arena.data_ptr(),
                                                        arena.numel(), _stream(stream), ctypes.byref(self._h)),
                   "bppsa_spscan_plan_create_cached")

    def close(self):
        if self._h:
            _lib.bppsa_spscan_plan_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        self.close()

    def arena_used(self):
        return int(_lib.bppsa_spscan_plan_arena_used(self._h))

    def num_products(self):
        return int(_lib.bppsa_spscan_plan_num_products(self._h))

    def flops(self):
        mm, mv = ctypes.c_int64(), ctypes.c_int64()
        _check(_lib.bppsa_spscan_plan_flops(self._h, ctypes.byref(mm), ctypes.byref(mv)), "bppsa_spscan_plan_flops")
        return mm.value, mv.value

    def steps(self):
        """The planned steps in issue order: dicts with kind, phase, level, matrix, flops, numeric_kind."""
        out = []
        for k in range(int(_lib.bppsa_spscan_plan_num_steps(self._h))):
            st = SpscanStep()
            _check(_lib.bppsa_spscan_plan_step_flops(self._h, k, ctypes.byref(st)), "bppsa_spscan_plan_step_flops")
            out.append({"kind": ("mv", "mm")[st.kind], "phase": ("up", "linear", "down", "tail")[st.phase],
                        "level": st.level, "matrix": st.matrix, "flops": st.flops, "numeric_kind": st.numeric_kind})
        return out

    def _view(self, ptr, count, dtype):
        off = ptr - self.arena.data_ptr()
        if 0 <= off and off + 4 * count <= self.arena.numel():
            return self.arena[off:off + 4 * count].view(dtype)
        if count == 0:
            return torch.empty((0,), dtype=dtype, device=self.arena.device)
        typestr = "<i4" if dtype == torch.int32 else "<f4"
        return torch.as_tensor(_DeviceArray(ptr, count, typestr, self.cache), device=self.arena.device)

    def product(self, idx):
        """(CsrMatrix view into the arena, left operand id, right operand id)."""
        d, l, r = CsrDesc(), ctypes.c_int(), ctypes.c_int()
        _check(_lib.bppsa_spscan_plan_product(self._h, idx, ctypes.byref(d), ctypes.byref(l), ctypes.byref(r)),
               "bppsa_spscan_plan_product")
        m = CsrMatrix(d.rows, d.cols, self._view(d.indptr, d.rows + 1, torch.int32),
                      self._view(d.indices, d.nnz, torch.int32), self._view(d.data, d.nnz, torch.float32))
        return m, l.value, r.value

    def run(self, jts, seed, grads, stream=None):
        descs = _desc_array(jts)
        _check(_lib.bppsa_spscan_run(self._h, descs, _ptr(seed), _grads_array(grads), _stream(stream)),
               "bppsa_spscan_run")
        return grads


def spscan(jts, seed, grads, up_levels, workspace, stream=None):
    """bppsa_spscan: one-shot plan + run + destroy (synchronises)."""
    descs = _desc_array(jts)
    _check(_lib.bppsa_spscan(len(jts), descs, _ptr(seed), _grads_array(grads), int(up_levels),
                             workspace.data_ptr(), workspace.numel(), _stream(stream)), "bppsa_spscan")
    return grads


def calibration_copy(src, dst, stream=None):
    """dst[:] = src for two fp32 tensors of equal size: the known-size copy used to scale traffic counters."""
    if src.numel() != dst.numel():
        raise ValueError("calibration_copy: sizes differ")
    _check(_lib.bppsa_calibration_copy(_ptr(src, name="src"), _ptr(dst, name="dst"), src.numel(),
                                       _stream(stream)), "bppsa_calibration_copy")
    return dst
