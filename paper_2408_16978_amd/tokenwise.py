"""Thin ctypes binding of libfpdt_tokenwise.so (include/fpdt_tokenwise.h): argument marshalling
only.  Tensors are torch tensors used as memory handles; there is no fallback."""
import ctypes
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libfpdt_tokenwise.so")
_lib = None


class FpdtTwError(RuntimeError):
    def __init__(self, status, text):
        super().__init__("fpdt_tw status %d: %s" % (status, text))
        self.status = status


def load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError("libfpdt_tokenwise.so is not built: run `python -m paper_2408_16978_amd.build`")
    L = ctypes.CDLL(LIB_PATH)
    vp, i64, ci, cf, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_float, ctypes.c_size_t
    L.fpdt_tw_loss_workspace_bytes.restype = sz
    L.fpdt_tw_loss_workspace_bytes.argtypes = [i64, ci, ci, ci]
    L.fpdt_tw_loss_fwd_bwd.restype = ci
    L.fpdt_tw_loss_fwd_bwd.argtypes = [vp, vp, vp, cf, vp, vp, vp, vp, i64, ci, ci, ci, vp, sz, vp]
    L.fpdt_tw_last_error.restype = ctypes.c_char_p
    _lib = L
    return L


def fpdt_tw_last_error() -> str:
    return load().fpdt_tw_last_error().decode()


def fpdt_tw_loss_workspace_bytes(rows, hidden, vocab, n_chunks) -> int:
    return int(load().fpdt_tw_loss_workspace_bytes(rows, hidden, vocab, n_chunks))


def _ptr(t):
    return None if t is None else t.data_ptr()


def fpdt_tw_loss_fwd_bwd(H, W, target, grad_scale, loss, lse, dH, dW, n_chunks, workspace, stream=None):
    """H [rows, hidden] bf16, W [vocab, hidden] bf16, target [rows] int32; loss, lse [rows] fp32;
    dH [rows, hidden] bf16 or None; dW [vocab, hidden] fp32 (accumulated into) or None."""
    rows, hidden = H.shape
    vocab = W.shape[0]
    if stream is None:
        stream = torch.cuda.current_stream()
    st = load().fpdt_tw_loss_fwd_bwd(_ptr(H), _ptr(W), _ptr(target), float(grad_scale), _ptr(loss), _ptr(lse),
                                     _ptr(dH), _ptr(dW), rows, hidden, vocab, n_chunks, _ptr(workspace),
                                     0 if workspace is None else workspace.numel() * workspace.element_size(),
                                     stream.cuda_stream)
    if st != 0:
        raise FpdtTwError(st, fpdt_tw_last_error())
