"""ctypes front end of fpdt_oracle.c: unchunked causal attention in fp64.

TEST INFRASTRUCTURE ONLY (see the header of fpdt_oracle.c).  All arrays are
numpy float64; tensors are [rows, heads, D]; LSE / Delta are returned as
[Hq, rows] to match the library's LSE layout.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_LIB = None


def lib():
    global _LIB
    if _LIB is None:
        path = _build.build(force=False)
        L = ctypes.CDLL(path)
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int64)
        L.fpdt_oracle_threads.restype = ctypes.c_int
        L.fpdt_oracle_rows.restype = ctypes.c_int
        L.fpdt_oracle_rows.argtypes = [dp, dp, ip, ctypes.c_int64, dp, dp, ctypes.c_int64,
                                       ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_double,
                                       dp, dp, dp, dp]
        bp = ctypes.POINTER(ctypes.c_uint8)
        L.fpdt_oracle_rows_blocksparse.restype = ctypes.c_int
        L.fpdt_oracle_rows_blocksparse.argtypes = [dp, dp, ip, ctypes.c_int64, dp, dp, ctypes.c_int64,
                                                   ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                                   ctypes.c_double, ctypes.c_int64, bp, dp, dp, dp, dp]
        L.fpdt_oracle_cols_blocksparse.restype = ctypes.c_int
        L.fpdt_oracle_cols_blocksparse.argtypes = [dp, dp, dp, dp, ctypes.c_int64, dp, dp, ip,
                                                   ctypes.c_int64, ctypes.c_int64, ctypes.c_int,
                                                   ctypes.c_int, ctypes.c_int, ctypes.c_double,
                                                   ctypes.c_int64, bp, dp, dp]
        L.fpdt_oracle_cols.restype = ctypes.c_int
        L.fpdt_oracle_cols.argtypes = [dp, dp, dp, dp, ctypes.c_int64, dp, dp, ip, ctypes.c_int64,
                                       ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                       ctypes.c_double, dp, dp]
        _LIB = L
    return _LIB


def threads() -> int:
    """Number of OpenMP threads the oracle will use."""
    return int(lib().fpdt_oracle_threads())


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _dp(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double)) if a is not None else None


def _ip(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int64))


def _mask(chunk_mask, chunk, S):
    """(chunk, contiguous uint8 [u,u] or None, its ctypes pointer or None)"""
    if chunk_mask is None:
        return 0, None, None
    m = np.ascontiguousarray(np.asarray(chunk_mask) != 0, dtype=np.uint8)
    assert chunk and S % chunk == 0 and m.shape == (S // chunk, S // chunk)
    return int(chunk), m, m.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8))


def rows(Qr, K, V, row_idx, scale, dOr=None, chunk=None, chunk_mask=None):
    """Quantities indexed by a query row, for the listed rows only.

    Qr, dOr: [n, Hq, D] (rows `row_idx` of Q and dO); K, V: [S, Hkv, D].
    chunk, chunk_mask [u,u]: block-sparse variant (query chunk m reads key chunk
    i <= m iff chunk_mask[m, i]); None = dense.
    Returns dict with O [n,Hq,D], LSE [Hq,n] and, if dOr is given,
    Delta [Hq,n] and dQ [n,Hq,D].
    """
    Qr, K, V = _f64(Qr), _f64(K), _f64(V)
    idx = np.ascontiguousarray(row_idx, dtype=np.int64)
    n, Hq, D = Qr.shape
    S, Hkv, D2 = K.shape
    assert D2 == D and V.shape == K.shape and idx.shape == (n,)
    O = np.empty((n, Hq, D))
    LSE = np.empty((n, Hq))
    if dOr is not None:
        dOr = _f64(dOr)
        assert dOr.shape == Qr.shape
        Delta = np.empty((n, Hq))
        dQ = np.empty((n, Hq, D))
    else:
        Delta = dQ = None
    c, m, mp = _mask(chunk_mask, chunk, S)
    if m is None:
        rc = lib().fpdt_oracle_rows(_dp(Qr), _dp(dOr), _ip(idx), n, _dp(K), _dp(V), S, Hq, Hkv, D,
                                    float(scale), _dp(O), _dp(LSE), _dp(Delta), _dp(dQ))
    else:
        rc = lib().fpdt_oracle_rows_blocksparse(_dp(Qr), _dp(dOr), _ip(idx), n, _dp(K), _dp(V), S,
                                                Hq, Hkv, D, float(scale), c, mp, _dp(O), _dp(LSE),
                                                _dp(Delta), _dp(dQ))
    if rc != 0:
        raise ValueError("fpdt_oracle_rows rejected its arguments")
    out = {"O": O, "LSE": np.ascontiguousarray(LSE.T)}
    if dOr is not None:
        out["Delta"] = np.ascontiguousarray(Delta.T)
        out["dQ"] = dQ
    return out


def cols(Qw, dOw, LSEw, Deltaw, row_base, Kc, Vc, col_idx, S, scale, chunk=None, chunk_mask=None):
    """dK, dV for the listed key rows.

    Qw, dOw: [S-row_base, Hq, D] query rows row_base..S-1; LSEw, Deltaw:
    [Hq, S-row_base] for the same rows; Kc, Vc: [n, Hkv, D] listed key rows.
    Returns (dK, dV), each [n, Hkv, D].
    """
    Qw, dOw, Kc, Vc = _f64(Qw), _f64(dOw), _f64(Kc), _f64(Vc)
    lse = _f64(np.asarray(LSEw).T)
    delta = _f64(np.asarray(Deltaw).T)
    idx = np.ascontiguousarray(col_idx, dtype=np.int64)
    W, Hq, D = Qw.shape
    n, Hkv, _ = Kc.shape
    assert W == S - row_base and lse.shape == (W, Hq) and delta.shape == (W, Hq)
    dK = np.empty((n, Hkv, D))
    dV = np.empty((n, Hkv, D))
    c, m, mp = _mask(chunk_mask, chunk, S)
    if m is None:
        rc = lib().fpdt_oracle_cols(_dp(Qw), _dp(dOw), _dp(lse), _dp(delta), int(row_base), _dp(Kc),
                                    _dp(Vc), _ip(idx), n, int(S), Hq, Hkv, D, float(scale), _dp(dK),
                                    _dp(dV))
    else:
        rc = lib().fpdt_oracle_cols_blocksparse(_dp(Qw), _dp(dOw), _dp(lse), _dp(delta),
                                                int(row_base), _dp(Kc), _dp(Vc), _ip(idx), n, int(S),
                                                Hq, Hkv, D, float(scale), c, mp, _dp(dK), _dp(dV))
    if rc != 0:
        raise ValueError("fpdt_oracle_cols rejected its arguments")
    return dK, dV


def attn_fwd(Q, K, V, scale):
    """Full forward: O [S,Hq,D], LSE [Hq,S]."""
    S = Q.shape[0]
    r = rows(Q, K, V, np.arange(S), scale)
    return r["O"], r["LSE"]


def attn_fwd_bwd(Q, K, V, dO, scale, chunk=None, chunk_mask=None):
    """Full forward + backward: dict O, LSE, Delta, dQ, dK, dV."""
    S = Q.shape[0]
    r = rows(Q, K, V, np.arange(S), scale, dOr=dO, chunk=chunk, chunk_mask=chunk_mask)
    dK, dV = cols(Q, dO, r["LSE"], r["Delta"], 0, K, V, np.arange(S), S, scale, chunk=chunk,
                  chunk_mask=chunk_mask)
    r["dK"], r["dV"] = dK, dV
    return r


def tail_window(Qw, dOw, K, V, w, scale):
    """Exact fwd+bwd for the last `w` query rows and dK, dV of the last `w` keys.

    Query rows S-w..S-1 are the only ones that attend keys S-w..S-1, so their
    dK/dV are complete.  Qw, dOw: [w, Hq, D] (the last w rows); K, V whole.
    """
    S = K.shape[0]
    idx = np.arange(S - w, S)
    r = rows(Qw, K, V, idx, scale, dOr=dOw)
    dK, dV = cols(Qw, dOw, r["LSE"], r["Delta"], S - w, K[S - w:], V[S - w:], idx, S, scale)
    r["dK"], r["dV"] = dK, dV
    return r
