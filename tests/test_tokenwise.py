"""Token-wise chunked neighbours (Sec. 5.4): oracle pins and host-side checks (no GPU), and GPU
parity of libfpdt_tokenwise.so against the oracle."""
import math
import os
import re

import numpy as np
import pytest
import torch

from oracle import tokenwise as otw
from paper_2408_16978_amd import tokenwise as TW

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


# ------------------------------------------------------------------ oracle pins (CPU)
def test_cross_entropy_oracle_against_torch_autograd():
    r = np.random.default_rng(1)
    rows, hidden, vocab = 37, 16, 53
    H, W = r.standard_normal((rows, hidden)), r.standard_normal((vocab, hidden))
    t = r.integers(0, vocab, rows)
    out = otw.cross_entropy(H, W, t, grad_scale=0.25)
    h = torch.tensor(H, requires_grad=True)
    w = torch.tensor(W, requires_grad=True)
    loss = torch.nn.functional.cross_entropy(h @ w.T, torch.tensor(t), reduction="none")
    (0.25 * loss.sum()).backward()
    np.testing.assert_allclose(out["loss"], loss.detach().numpy(), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(out["lse"], torch.logsumexp(h @ w.T, dim=1).detach().numpy(), rtol=1e-12)
    np.testing.assert_allclose(out["dH"], h.grad.numpy(), rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(out["dW"], w.grad.numpy(), rtol=1e-11, atol=1e-13)


def test_cross_entropy_oracle_closed_forms():
    r = np.random.default_rng(2)
    rows, hidden, vocab = 9, 4, 11
    H = r.standard_normal((rows, hidden))
    t = r.integers(0, vocab, rows)
    # W = 0: uniform distribution, loss = log(vocab), dH = 0, dW = (1/vocab - onehot)^T H
    out = otw.cross_entropy(H, np.zeros((vocab, hidden)), t)
    np.testing.assert_allclose(out["loss"], math.log(vocab), rtol=1e-15)
    np.testing.assert_allclose(out["dH"], 0.0, atol=1e-15)
    G = np.full((rows, vocab), 1.0 / vocab)
    G[np.arange(rows), t] -= 1.0
    np.testing.assert_allclose(out["dW"], G.T @ H, atol=1e-14)
    # the gradient with respect to the logits sums to zero per row: sum_v dW[v, :] = 0
    W = r.standard_normal((vocab, hidden))
    out = otw.cross_entropy(H, W, t)
    np.testing.assert_allclose(out["dW"].sum(axis=0), 0.0, atol=1e-13)
    # shifting every logit of a row by a constant (H -> H, W -> W + 1 u^T with H u = const) ...
    # simpler shift invariance: adding the same vector to every row of W adds H_r . v to all
    # logits of row r, which changes neither the loss nor dH's projection on that direction
    v = r.standard_normal(hidden)
    out2 = otw.cross_entropy(H, W + v, t)
    np.testing.assert_allclose(out2["loss"], out["loss"], atol=1e-12)


# ------------------------------------------------------------------ host-side ABI checks (CPU)
def test_tokenwise_library_exports_and_rejects_bad_arguments():
    text = open(os.path.join(ROOT, "include", "fpdt_tokenwise.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = sorted(set(re.findall(r"\b(fpdt_tw_[a-z_0-9]+)\s*\(", text)))
    assert {"fpdt_tw_loss_fwd_bwd", "fpdt_tw_loss_workspace_bytes", "fpdt_tw_last_error"} <= set(names)
    L = TW.load()
    for n in names:
        assert hasattr(L, n), n
        assert callable(getattr(TW, n)), n
    # chunk = ceil(rows / n_chunks): fp32 logits + bf16 gradient of one chunk, each 256-aligned
    assert TW.fpdt_tw_loss_workspace_bytes(1000, 64, 512, 3) == 334 * 512 * 4 + (334 * 512 * 2 + 255) // 256 * 256
    assert TW.fpdt_tw_loss_workspace_bytes(0, 64, 512, 1) == 0
    assert TW.fpdt_tw_loss_workspace_bytes(10, 64, 512, 11) == 0
    p = 0x1000
    call = lambda **kw: L.fpdt_tw_loss_fwd_bwd(*[kw.get(k, d) for k, d in (
        ("H", p), ("W", p), ("t", p), ("gs", 1.0), ("loss", p), ("lse", p), ("dH", p), ("dW", p), ("rows", 1024),
        ("hidden", 64), ("vocab", 512), ("n", 4), ("ws", 0x100000), ("wsb", 1 << 40), ("st", None))])
    assert call(H=None) == 1 and "NULL" in TW.fpdt_tw_last_error()
    assert call(rows=0) == 1
    assert call(n=0) == 1
    assert call(n=2000) == 1
    assert call(gs=float("nan")) == 1
    assert call(ws=None) == 3
    assert call(wsb=16) == 3
    assert call(ws=0x100010) == 3


# ------------------------------------------------------------------ GPU parity
def _case(rows, hidden, vocab, seed):
    g = torch.Generator().manual_seed(seed)
    H = torch.randn(rows, hidden, generator=g).to(torch.bfloat16)
    W = (torch.randn(vocab, hidden, generator=g) * hidden ** -0.5).to(torch.bfloat16)
    t = torch.randint(0, vocab, (rows,), generator=g, dtype=torch.int32)
    return H, W, t


@pytest.mark.gpu
@pytest.mark.parametrize("rows,hidden,vocab,n_chunks", [(1000, 256, 1536, 3), (512, 128, 4099, 8), (96, 64, 320, 1)])
def test_gpu_loss_matches_oracle(rows, hidden, vocab, n_chunks):
    print("[case] chunked loss", rows, hidden, vocab, n_chunks, flush=True)
    H, W, t = _case(rows, hidden, vocab, 31)
    ref = otw.cross_entropy(H.double().numpy(), W.double().numpy(), t.numpy(), grad_scale=1.0 / rows)
    Hd, Wd, td = H.cuda(), W.cuda(), t.cuda()
    loss = torch.empty(rows, device="cuda")
    lse = torch.empty(rows, device="cuda")
    dH = torch.empty_like(Hd)
    dW = torch.zeros(vocab, hidden, device="cuda")
    ws = torch.empty(TW.fpdt_tw_loss_workspace_bytes(rows, hidden, vocab, n_chunks), dtype=torch.uint8, device="cuda")
    TW.fpdt_tw_loss_fwd_bwd(Hd, Wd, td, 1.0 / rows, loss, lse, dH, dW, n_chunks, ws)
    torch.cuda.synchronize()
    # logits are exact bf16 products accumulated in fp32: loss and lse to fp32 round-off
    np.testing.assert_allclose(loss.cpu().numpy(), ref["loss"], atol=2e-4)
    np.testing.assert_allclose(lse.cpu().numpy(), ref["lse"], atol=2e-4)
    # gradients: the logit gradient is rounded to bf16 before its two GEMMs and dH is stored in
    # bf16: per row (dH) / per vocabulary row (dW) 2e-2 of the reference row's RMS + storage half-ulp
    for name, got, r in (("dH", dH.float().cpu().numpy(), ref["dH"]), ("dW", dW.cpu().numpy(), ref["dW"])):
        rms = np.sqrt((r ** 2).mean(axis=1, keepdims=True))
        budget = 2e-2 * rms + 2.0 ** -9 * np.abs(r) + 1e-9
        assert (np.abs(got - r) <= budget).all(), (name, float((np.abs(got - r) / budget).max()))
    # dW is accumulated into: a second call doubles it; the chunk count does not change anything
    # beyond fp32 summation order
    TW.fpdt_tw_loss_fwd_bwd(Hd, Wd, td, 1.0 / rows, loss, lse, dH, dW, n_chunks, ws)
    torch.cuda.synchronize()
    np.testing.assert_allclose(dW.cpu().numpy(), 2 * ref["dW"], atol=2 * float(np.abs(ref["dW"]).max()) * 2e-2 + 1e-9)
    if n_chunks > 1:
        loss1 = torch.empty(rows, device="cuda")
        ws1 = torch.empty(TW.fpdt_tw_loss_workspace_bytes(rows, hidden, vocab, 1), dtype=torch.uint8, device="cuda")
        TW.fpdt_tw_loss_fwd_bwd(Hd, Wd, td, 1.0 / rows, loss1, lse, None, None, 1, ws1)
        torch.cuda.synchronize()
        np.testing.assert_allclose(loss1.cpu().numpy(), loss.cpu().numpy(), atol=1e-5)
        assert ws.numel() < ws1.numel()


@pytest.mark.gpu
def test_gpu_loss_rejects_small_workspace():
    H, W, t = _case(64, 64, 128, 32)
    out = torch.empty(64, device="cuda")
    ws = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(TW.FpdtTwError) as e:
        TW.fpdt_tw_loss_fwd_bwd(H.cuda(), W.cuda(), t.cuda(), 1.0, out, out.clone(), None, None, 1, ws)
    assert e.value.status == 3
