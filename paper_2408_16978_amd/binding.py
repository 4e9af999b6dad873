"""Thin ctypes binding of libfpdt.so: argument marshalling only.

Function names match the C ABI (include/fpdt.h).  Tensors are torch tensors used purely as
memory handles (device memory, or pinned host memory for the offload flags); every step of
the attention path runs inside the library's HIP kernels.  There is no fallback: if the
library has not been built, loading raises.
"""
import ctypes
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libfpdt.so")

FPDT_OK, FPDT_ERR_INVALID_ARG, FPDT_ERR_UNSUPPORTED, FPDT_ERR_WORKSPACE, FPDT_ERR_HIP = range(5)
FPDT_DTYPE_F32, FPDT_DTYPE_BF16 = 0, 1
FPDT_KV_ON_HOST = 1 << 0
FPDT_ACT_ON_HOST = 1 << 1
FPDT_BWD_KV_OUTER = 1 << 2
FPDT_BWD_Q_OUTER = 1 << 3
FPDT_PAIRWISE = 1 << 4
FPDT_BWD_STORE_DS = 1 << 5
FPDT_CHUNK_MULTIPLE = 256
FPDT_NOALLOC_SCRATCH_BYTES = 32 << 20
FPDT_PREFERRED_CHUNK = 65536
FPDT_PROF_FWD, FPDT_PROF_DKDV, FPDT_PROF_DQ, FPDT_PROF_H2D, FPDT_PROF_D2H = range(5)
FPDT_DEBUG_POISON_STAGING, FPDT_DEBUG_DELAY_COPIES = 1, 2

_lib = None


class FpdtError(RuntimeError):
    def __init__(self, status, text):
        super().__init__("fpdt status %d: %s" % (status, text))
        self.status = status


def load():
    """Load libfpdt.so (built by paper_2408_16978_amd.build); raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError("libfpdt.so is not built: run `python -m paper_2408_16978_amd.build` "
                          "(there is no CPU or PyTorch fallback)")
    L = ctypes.CDLL(LIB_PATH)
    vp, i64, ci, cu, cf, sz = (ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_uint,
                               ctypes.c_float, ctypes.c_size_t)
    L.fpdt_attn_workspace_bytes.restype = sz
    L.fpdt_attn_workspace_bytes.argtypes = [i64, i64, ci, ci, ci, ci, cu, ci]
    L.fpdt_attn_pick_chunk.restype = i64
    L.fpdt_attn_pick_chunk.argtypes = [i64, ci, ci, ci, ci, cu, sz]
    L.fpdt_attn_fwd.restype = ci
    L.fpdt_attn_fwd.argtypes = [vp, vp, vp, vp, vp, i64, i64, ci, ci, ci, cf, ci, cu, vp, sz, vp]
    L.fpdt_attn_fwd_noalloc.restype = ci
    L.fpdt_attn_fwd_noalloc.argtypes = [vp, vp, vp, vp, vp, i64, i64, ci, ci, ci, cf, ci, cu, vp]
    L.fpdt_attn_bwd.restype = ci
    L.fpdt_attn_bwd.argtypes = [vp] * 9 + [i64, i64, ci, ci, ci, cf, ci, cu, vp, sz, vp]
    L.fpdt_attn_fwd_blocksparse.restype = ci
    L.fpdt_attn_fwd_blocksparse.argtypes = [vp, vp, vp, vp, vp, i64, i64, ci, ci, ci, cf, ci, cu, vp, vp, sz, vp]
    L.fpdt_attn_bwd_blocksparse.restype = ci
    L.fpdt_attn_bwd_blocksparse.argtypes = [vp] * 9 + [i64, i64, ci, ci, ci, cf, ci, cu, vp, vp, sz, vp]
    L.fpdt_attn_merge.restype = ci
    L.fpdt_attn_merge.argtypes = [vp] * 6 + [i64, ci, ci, ci, vp]
    L.fpdt_last_link_bytes.restype = ci
    L.fpdt_last_link_bytes.argtypes = [ctypes.POINTER(ctypes.c_uint64)] * 2
    L.fpdt_profile_enable.restype = ci
    L.fpdt_profile_enable.argtypes = [ci]
    L.fpdt_profile_read.restype = ci
    L.fpdt_profile_read.argtypes = [ci, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i64)]
    L.fpdt_calibrate_mfma.restype = ci
    L.fpdt_calibrate_mfma.argtypes = [ci, ci, vp, sz, ctypes.POINTER(ctypes.c_double),
                                      ctypes.POINTER(ctypes.c_double), vp]
    L.fpdt_debug_configure.restype = ci
    L.fpdt_debug_configure.argtypes = [cu]
    L.fpdt_last_error.restype = ctypes.c_char_p
    L.fpdt_version.restype = ctypes.c_char_p
    _lib = L
    return L


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return FPDT_DTYPE_F32
    if t.dtype == torch.bfloat16:
        return FPDT_DTYPE_BF16
    raise TypeError("fpdt: tensors must be float32 or bfloat16, got %s" % t.dtype)


def _stream_handle(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _check(status):
    if status != FPDT_OK:
        raise FpdtError(status, fpdt_last_error())


def fpdt_version() -> str:
    return load().fpdt_version().decode()


def fpdt_last_error() -> str:
    return load().fpdt_last_error().decode()


def fpdt_last_link_bytes():
    h, d = ctypes.c_uint64(0), ctypes.c_uint64(0)
    load().fpdt_last_link_bytes(ctypes.byref(h), ctypes.byref(d))
    return int(h.value), int(d.value)


def fpdt_debug_configure(flags: int):
    """Event-ordering checks of the offload pipeline (poisoned staging buffers, delayed copies)."""
    _check(load().fpdt_debug_configure(flags))


def fpdt_profile_enable(on: bool):
    _check(load().fpdt_profile_enable(int(on)))


def fpdt_profile_read(kind: int):
    """(total milliseconds, launches) of one kind since the last read; waits for the events."""
    ms, n = ctypes.c_double(0.0), ctypes.c_int64(0)
    _check(load().fpdt_profile_read(kind, ctypes.byref(ms), ctypes.byref(n)))
    return float(ms.value), int(n.value)


FPDT_CAL_KINDS = ("mfma_reg_2w", "mfma_reg_1w", "softmax_reg_2w", "softmax_reg_1w", "mfma_lds1_2w",
                  "mfma_lds2_1w", "softmax_lds1_2w", "softmax_lds2_1w")
FPDT_CAL_WORKSPACE_BYTES = 1 << 20


def fpdt_calibrate_mfma(kind: int, iters: int = 20000, stream=None):
    """(TFLOP/s, milliseconds) of one calibration loop (see include/fpdt.h)."""
    ws = torch.empty(FPDT_CAL_WORKSPACE_BYTES, dtype=torch.uint8, device="cuda")
    tf, ms = ctypes.c_double(0.0), ctypes.c_double(0.0)
    _check(load().fpdt_calibrate_mfma(kind, iters, ws.data_ptr(), ws.numel(), ctypes.byref(tf),
                                      ctypes.byref(ms), _stream_handle(stream)))
    return float(tf.value), float(ms.value)


def fpdt_attn_workspace_bytes(S, chunk, Hq, Hkv, D, dtype, flags=0, is_bwd=False) -> int:
    return int(load().fpdt_attn_workspace_bytes(S, chunk, Hq, Hkv, D, dtype, flags, int(is_bwd)))


def fpdt_attn_pick_chunk(S, Hq, Hkv, D, dtype, flags=0, max_workspace_bytes=0) -> int:
    """Recommended chunk size (0 if none: see fpdt_last_error)."""
    return int(load().fpdt_attn_pick_chunk(S, Hq, Hkv, D, dtype, flags, max_workspace_bytes))


def fpdt_attn_fwd(Q, K, V, O, LSE, chunk, scale, flags=0, workspace=None, stream=None):
    """Enqueue the forward.  Q,O [S,Hq,D]; K,V [S,Hkv,D]; LSE [Hq,S] fp32.  `workspace` is a
    device uint8 tensor of at least fpdt_attn_workspace_bytes(...) bytes."""
    S, Hq, D = Q.shape
    Hkv = K.shape[1]
    ws_ptr = _ptr(workspace)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = load().fpdt_attn_fwd(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(LSE), S, chunk, Hq, Hkv, D,
                              float(scale), _dtype_code(Q), flags, ws_ptr, ws_bytes,
                              _stream_handle(stream))
    _check(st)


def fpdt_attn_fwd_noalloc(Q, K, V, O, LSE, chunk, scale, flags=0, stream=None):
    """fpdt_attn_fwd on the library's built-in scratch array: no workspace argument, no allocation."""
    S, Hq, D = Q.shape
    Hkv = K.shape[1]
    st = load().fpdt_attn_fwd_noalloc(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(LSE), S, chunk, Hq, Hkv,
                                      D, float(scale), _dtype_code(Q), flags, _stream_handle(stream))
    _check(st)


def fpdt_attn_bwd(Q, K, V, O, LSE, dO, dQ, dK, dV, chunk, scale, flags=0, workspace=None,
                  stream=None):
    """Enqueue the backward.  dQ, dK, dV are fully overwritten."""
    S, Hq, D = Q.shape
    Hkv = K.shape[1]
    ws_ptr = _ptr(workspace)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = load().fpdt_attn_bwd(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(LSE), _ptr(dO), _ptr(dQ),
                              _ptr(dK), _ptr(dV), S, chunk, Hq, Hkv, D, float(scale),
                              _dtype_code(Q), flags, ws_ptr, ws_bytes, _stream_handle(stream))
    _check(st)


def _mask_bytes(chunk_mask, u):
    """u*u bytes (row = query chunk) from any array-like / tensor; kept alive by the caller."""
    m = torch.as_tensor(chunk_mask).to("cpu")
    if tuple(m.shape) != (u, u):
        raise ValueError("chunk_mask must be [%d, %d], got %s" % (u, u, tuple(m.shape)))
    return (m != 0).to(torch.uint8).contiguous()


def fpdt_attn_fwd_blocksparse(Q, K, V, O, LSE, chunk, scale, chunk_mask, flags=0, workspace=None,
                              stream=None):
    """Forward with a [u, u] chunk mask (query chunk m reads key chunk i <= m iff mask[m, i])."""
    S, Hq, D = Q.shape
    Hkv = K.shape[1]
    m = _mask_bytes(chunk_mask, S // chunk)
    ws_ptr = _ptr(workspace)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = load().fpdt_attn_fwd_blocksparse(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(LSE), S, chunk, Hq,
                                          Hkv, D, float(scale), _dtype_code(Q), flags, m.data_ptr(),
                                          ws_ptr, ws_bytes, _stream_handle(stream))
    _check(st)


def fpdt_attn_bwd_blocksparse(Q, K, V, O, LSE, dO, dQ, dK, dV, chunk, scale, chunk_mask, flags=0,
                              workspace=None, stream=None):
    """Backward with the chunk mask the forward was given."""
    S, Hq, D = Q.shape
    Hkv = K.shape[1]
    m = _mask_bytes(chunk_mask, S // chunk)
    ws_ptr = _ptr(workspace)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = load().fpdt_attn_bwd_blocksparse(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(LSE), _ptr(dO),
                                          _ptr(dQ), _ptr(dK), _ptr(dV), S, chunk, Hq, Hkv, D,
                                          float(scale), _dtype_code(Q), flags, m.data_ptr(), ws_ptr,
                                          ws_bytes, _stream_handle(stream))
    _check(st)


def fpdt_attn_merge(O_a, LSE_a, O_b, LSE_b, O_out, LSE_out, stream=None):
    rows, Hq, D = O_a.shape
    st = load().fpdt_attn_merge(_ptr(O_a), _ptr(LSE_a), _ptr(O_b), _ptr(LSE_b), _ptr(O_out),
                                _ptr(LSE_out), rows, Hq, D, _dtype_code(O_a),
                                _stream_handle(stream))
    _check(st)


def alloc_workspace(S, chunk, Hq, Hkv, D, dtype, flags=0, is_bwd=False, device="cuda"):
    """Device workspace tensor of the size the library asks for (torch only owns the memory)."""
    n = fpdt_attn_workspace_bytes(S, chunk, Hq, Hkv, D, dtype, flags, is_bwd)
    if n == 0:
        # let the entry point report why
        return torch.empty(256, dtype=torch.uint8, device=device)
    return torch.empty(n, dtype=torch.uint8, device=device)
