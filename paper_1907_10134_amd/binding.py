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
    def __init__(self, code, where):
        self.code = code
        super().__init__("%s failed: %s" % (where, _lib.bppsa_strerror(code).decode()))


def _load():
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            "libbppsa.so is not built (expected at %s); run "
            "`python -c 'import __graft_entry__ as g; g.build()'` first - there is no "
            "CPU fallback" % _LIB_PATH)
    lib = ctypes.CDLL(_LIB_PATH)
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
    lib.bppsa_param_grads_workspace_bytes.restype = c_size_t
    lib.bppsa_param_grads_workspace_bytes.argtypes = [c_int] * 5
    lib.bppsa_param_grads.restype = c_int
    lib.bppsa_param_grads.argtypes = [c_int] * 5 + [c_void_p] * 12 + [c_size_t, c_void_p]
    return lib


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


def _workspace(nbytes, device):
    # 256-byte aligned by the caching allocator (its blocks are 512-byte aligned)
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


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
        workspace = _workspace(scan_workspace_bytes(T, B, H), Jt.device)
    _check(_lib.bppsa_scan(T, B, H, _ptr(Jt), _ptr(seed), _ptr(G), _ptr(g0),
                           workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                           _stream(stream)), "bppsa_scan")
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
