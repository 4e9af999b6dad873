"""Comparison helpers shared by the GPU parity tests (not collected by pytest)."""
import numpy as np
import torch

from oracle import definition

F32_TOL = 1e-4        # max-abs, fp32 tensors
BF16_TOL = 2e-2       # per (row, head): max_d |x - ref| <= BF16_TOL * rms_d(ref[row, head, :])
BF16_LSE_TOL = 2e-2   # abs


def to64(t: torch.Tensor) -> np.ndarray:
    """The stored bits (bf16 or fp32) widened to fp64 -- what the oracle is fed."""
    return t.detach().cpu().to(torch.float64).numpy()


def oracle_full(Q, K, V, dO, scale):
    return definition.attn_fwd_bwd(to64(Q), to64(K), to64(V), to64(dO), scale)


def check(name, got, ref, is_bf16):
    """Raise AssertionError if `got` is outside the tolerance of `ref`.
    got/ref: [rows, heads, D] or, for LSE, [heads, rows]."""
    got = to64(got) if isinstance(got, torch.Tensor) else np.asarray(got, dtype=np.float64)
    assert got.shape == ref.shape, (name, got.shape, ref.shape)
    assert np.isfinite(got).all(), name + " has non-finite values"
    err = np.abs(got - ref)
    if not is_bf16:
        assert err.max() <= F32_TOL, "%s: max-abs %.3e > %.1e" % (name, err.max(), F32_TOL)
        return err.max()
    if name == "LSE":
        assert err.max() <= BF16_LSE_TOL, "LSE: max-abs %.3e" % err.max()
        return err.max()
    rms = np.sqrt((ref ** 2).mean(axis=-1))
    ratio = err.max(axis=-1) / np.maximum(rms, 1e-30)
    worst = ratio.max()
    assert worst <= BF16_TOL, "%s: worst row error %.3e x row-rms (limit %.1e) at %s" % (
        name, worst, BF16_TOL, np.unravel_index(ratio.argmax(), ratio.shape))
    return worst


def check_all(out, ref, is_bf16, names=("O", "LSE", "dQ", "dK", "dV")):
    return {n: check(n, out[n], ref[n], is_bf16) for n in names}
