"""Comparison helpers shared by the GPU parity tests (not collected by pytest)."""
import numpy as np
import torch

from oracle import definition

F32_TOL = 1e-4        # max-abs, fp32 tensors
# bf16 tensors, per (row, head) and element d:
#   |x - ref| <= BF16_TOL * rms_d(ref[row, head, :])   compute error, relative to the row's RMS
#              + BF16_HALF_ULP * |ref|                  storing the result as bf16 (half an ulp is between
#                                                       2^-9 |x| and 2^-8 |x|; the smaller figure is granted)
#              + BF16_FLOOR                             fp32 round-off where the exact value is ~0
BF16_TOL = 2e-2
BF16_HALF_ULP = 2.0 ** -9
BF16_FLOOR = 1e-5
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
    rms = np.sqrt((ref ** 2).mean(axis=-1, keepdims=True))
    budget = BF16_TOL * rms + BF16_HALF_ULP * np.abs(ref) + BF16_FLOOR
    used = err / budget
    worst = used.max()
    assert worst <= 1.0, "%s: error uses %.3f of its budget at %s (err %.3e, row rms %.3e)" % (
        name, worst, np.unravel_index(used.argmax(), used.shape), err.flat[used.argmax()],
        rms.flat[used.argmax() // ref.shape[-1]])
    return worst


def check_all(out, ref, is_bf16, names=("O", "LSE", "dQ", "dK", "dV")):
    return {n: check(n, out[n], ref[n], is_bf16) for n in names}
