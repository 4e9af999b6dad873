"""fpdt_attn_fwd_noalloc: the forward on the library's built-in scratch array, for callers that
cannot allocate.  It runs the kernels of fpdt_attn_fwd, so the two must agree bit for bit; two
calls in a row (the second one smaller, on a scratch array that still holds the first call's
contents), then the oracle, then the size limit."""
import pytest
import torch

import parity
from paper_2408_16978_amd import binding as B, inputs

pytestmark = pytest.mark.gpu


def _both(S, chunk, Hq, Hkv, D, dtype, flags, seed):
    Q, K, V, _ = inputs.make_qkvdo(S, Hq, Hkv, D, dtype, seed, device="cuda")
    scale = D ** -0.5
    dt = B.FPDT_DTYPE_BF16 if dtype == "bf16" else B.FPDT_DTYPE_F32
    O_ref = torch.empty_like(Q)
    LSE_ref = torch.empty((Hq, S), dtype=torch.float32, device="cuda")
    ws = B.alloc_workspace(S, chunk, Hq, Hkv, D, dt, flags, False)
    B.fpdt_attn_fwd(Q, K, V, O_ref, LSE_ref, chunk, scale, flags, ws)
    O = torch.full_like(Q, float("nan"))
    LSE = torch.full_like(LSE_ref, float("nan"))
    B.fpdt_attn_fwd_noalloc(Q, K, V, O, LSE, chunk, scale, flags)
    torch.cuda.synchronize()
    return (Q, K, V, scale), (O, LSE), (O_ref, LSE_ref)


def _same_bits(a, b):
    return torch.equal(a.view(torch.int16 if a.dtype == torch.bfloat16 else torch.int32),
                       b.view(torch.int16 if b.dtype == torch.bfloat16 else torch.int32))


def test_two_calls_in_a_row_match_the_workspace_entry_point():
    torch.cuda.set_device(0)
    # first call: Llama-8B head shape, 4 chunks in one launch; fills 16 MiB of the scratch array
    inp, got, ref = _both(16384, 4096, 8, 2, 128, "bf16", 0, seed=31)
    assert _same_bits(got[0], ref[0]) and _same_bits(got[1], ref[1])
    # second call: smaller, other head shape (D = 80 pads its value fragments), pair by pair with
    # carried state in the scratch array, which still holds the first call's packed operands
    inp, got, ref = _both(1024, 256, 4, 4, 80, "bf16", B.FPDT_PAIRWISE, seed=32)
    assert _same_bits(got[0], ref[0]) and _same_bits(got[1], ref[1])
    Q, K, V, scale = inp
    want = parity.definition.attn_fwd_bwd(parity.to64(Q), parity.to64(K), parity.to64(V),
                                          parity.to64(Q), scale)
    parity.check("O", got[0], want["O"], True)
    parity.check("LSE", got[1], want["LSE"], True)
    # third: the fp32 path on the same array
    inp, got, ref = _both(512, 128, 2, 2, 64, "f32", 0, seed=33)
    assert _same_bits(got[0], ref[0]) and _same_bits(got[1], ref[1])


def test_sizes_beyond_the_array_and_offload_flags_are_refused():
    torch.cuda.set_device(0)
    S, Hq, Hkv, D = 65536, 8, 2, 128  # needs 64 MiB of packed K/V
    assert B.fpdt_attn_workspace_bytes(S, S, Hq, Hkv, D, B.FPDT_DTYPE_BF16, 0, False) > B.FPDT_NOALLOC_SCRATCH_BYTES
    Q = torch.zeros((S, Hq, D), dtype=torch.bfloat16, device="cuda")
    K = torch.zeros((S, Hkv, D), dtype=torch.bfloat16, device="cuda")
    O = torch.full_like(Q, 7.0)
    LSE = torch.zeros((Hq, S), dtype=torch.float32, device="cuda")
    with pytest.raises(B.FpdtError) as e:
        B.fpdt_attn_fwd_noalloc(Q, K, K, O, LSE, S, D ** -0.5, 0)
    assert e.value.status == B.FPDT_ERR_WORKSPACE and "scratch" in str(e.value)
    with pytest.raises(B.FpdtError) as e:
        B.fpdt_attn_fwd_noalloc(Q[:1024], K[:1024], K[:1024], O[:1024], LSE[:, :1024].contiguous(), 256,
                                D ** -0.5, B.FPDT_KV_ON_HOST)
    assert e.value.status == B.FPDT_ERR_UNSUPPORTED
    torch.cuda.synchronize()
    assert bool((O == 7.0).all())  # nothing was enqueued
