"""Convenience layer over the binding: buffer placement + one call per pass.

Allocation and placement only (device tensors, pinned host tensors, workspace); the
attention itself is the library's.  Used by the tests, the smoke check and the benchmark.
"""
from dataclasses import dataclass

import torch

from . import binding as B


def _place(t: torch.Tensor, on_host: bool) -> torch.Tensor:
    """Pinned host copy (offloaded tensors) or device copy of `t`."""
    if on_host:
        out = torch.empty(t.shape, dtype=t.dtype, pin_memory=True)
        out.copy_(t)
        return out
    return t.to("cuda") if not t.is_cuda else t


def _empty_like_placed(shape, dtype, on_host: bool) -> torch.Tensor:
    if on_host:
        return torch.empty(shape, dtype=dtype, pin_memory=True)
    return torch.empty(shape, dtype=dtype, device="cuda")


@dataclass
class Buffers:
    Q: torch.Tensor
    K: torch.Tensor
    V: torch.Tensor
    dO: torch.Tensor
    O: torch.Tensor
    LSE: torch.Tensor
    dQ: torch.Tensor
    dK: torch.Tensor
    dV: torch.Tensor
    ws_fwd: torch.Tensor
    ws_bwd: torch.Tensor
    chunk: int
    scale: float
    flags: int
    chunk_mask: object = None  # [u, u] block-sparse mask, or None for dense attention


def make_buffers(Q, K, V, dO, chunk, scale, flags=0, bwd=True, chunk_mask=None) -> Buffers:
    """Place inputs per the offload flags and allocate outputs + workspaces.  With a chunk mask
    the block-sparse entry points are used (pair-by-pair schedule)."""
    if chunk_mask is not None:
        flags |= B.FPDT_PAIRWISE
    S, Hq, D = Q.shape
    Hkv = K.shape[1]
    kvh = bool(flags & B.FPDT_KV_ON_HOST)
    acth = bool(flags & B.FPDT_ACT_ON_HOST)
    dt = B.FPDT_DTYPE_BF16 if Q.dtype == torch.bfloat16 else B.FPDT_DTYPE_F32
    fwd_flags = flags & ~(B.FPDT_BWD_KV_OUTER | B.FPDT_BWD_Q_OUTER | B.FPDT_BWD_STORE_DS)
    bufs = Buffers(
        Q=_place(Q, acth), K=_place(K, kvh), V=_place(V, kvh), dO=_place(dO, acth),
        O=_empty_like_placed((S, Hq, D), Q.dtype, acth),
        LSE=_empty_like_placed((Hq, S), torch.float32, acth),
        dQ=_empty_like_placed((S, Hq, D), Q.dtype, acth) if bwd else None,
        dK=_empty_like_placed((S, Hkv, D), Q.dtype, kvh) if bwd else None,
        dV=_empty_like_placed((S, Hkv, D), Q.dtype, kvh) if bwd else None,
        ws_fwd=B.alloc_workspace(S, chunk, Hq, Hkv, D, dt, fwd_flags, False),
        ws_bwd=B.alloc_workspace(S, chunk, Hq, Hkv, D, dt, flags, True) if bwd else None,
        chunk=chunk, scale=scale, flags=flags, chunk_mask=chunk_mask)
    return bufs


def forward(b: Buffers, stream=None):
    fwd_flags = b.flags & ~(B.FPDT_BWD_KV_OUTER | B.FPDT_BWD_Q_OUTER | B.FPDT_BWD_STORE_DS)
    if b.chunk_mask is not None:
        B.fpdt_attn_fwd_blocksparse(b.Q, b.K, b.V, b.O, b.LSE, b.chunk, b.scale, b.chunk_mask,
                                    fwd_flags, b.ws_fwd, stream)
    else:
        B.fpdt_attn_fwd(b.Q, b.K, b.V, b.O, b.LSE, b.chunk, b.scale, fwd_flags, b.ws_fwd, stream)


def backward(b: Buffers, stream=None):
    if b.chunk_mask is not None:
        B.fpdt_attn_bwd_blocksparse(b.Q, b.K, b.V, b.O, b.LSE, b.dO, b.dQ, b.dK, b.dV, b.chunk,
                                    b.scale, b.chunk_mask, b.flags, b.ws_bwd, stream)
    else:
        B.fpdt_attn_bwd(b.Q, b.K, b.V, b.O, b.LSE, b.dO, b.dQ, b.dK, b.dV, b.chunk, b.scale, b.flags,
                        b.ws_bwd, stream)
