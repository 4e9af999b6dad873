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


@pytest.mark.parametrize("swiglu", [False, True])
def test_ffn_and_linear_oracles_against_torch_autograd(swiglu):
    r = np.random.default_rng(3 + swiglu)
    rows, n_model, n_ffn = 23, 12, 29
    X, dY = r.standard_normal((rows, n_model)), r.standard_normal((rows, n_model))
    W1, W3 = r.standard_normal((n_ffn, n_model)), r.standard_normal((n_ffn, n_model))
    W2 = r.standard_normal((n_model, n_ffn))
    out = otw.ffn(X, W1, W2, W3 if swiglu else None, dY)
    x, w1, w3, w2 = (torch.tensor(a, requires_grad=True) for a in (X, W1, W3, W2))
    F = torch.nn.functional
    y = (F.silu(x @ w1.T) * (x @ w3.T)) @ w2.T if swiglu else F.gelu(x @ w1.T) @ w2.T
    (y * torch.tensor(dY)).sum().backward()
    np.testing.assert_allclose(out["Y"], y.detach().numpy(), rtol=1e-11, atol=1e-12)
    for k, t in (("dX", x), ("dW1", w1), ("dW2", w2)) + ((("dW3", w3),) if swiglu else ()):
        np.testing.assert_allclose(out[k], t.grad.numpy(), rtol=1e-10, atol=1e-11, err_msg=k)
    assert ("dW3" in out) == swiglu
    # the linear projection is the FFN's first GEMM: pin it the same way
    x2, w = torch.tensor(X, requires_grad=True), torch.tensor(W1, requires_grad=True)
    dy2 = r.standard_normal((rows, n_ffn))
    lin = otw.linear(X, W1, dY=dy2)
    ((x2 @ w.T) * torch.tensor(dy2)).sum().backward()
    np.testing.assert_allclose(lin["Y"], (x2 @ w.T).detach().numpy(), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(lin["dX"], x2.grad.numpy(), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(lin["dW"], w.grad.numpy(), rtol=1e-12, atol=1e-13)


def test_ffn_oracle_closed_forms_and_finite_differences():
    r = np.random.default_rng(5)
    rows, n_model, n_ffn = 5, 4, 6
    X = r.standard_normal((rows, n_model))
    W1, W3 = r.standard_normal((n_ffn, n_model)), r.standard_normal((n_ffn, n_model))
    W2 = r.standard_normal((n_model, n_ffn))
    # gelu(0) = silu(0) = 0: X = 0 gives Y = 0; gelu'(0) = silu'(0) = 1/2
    z = np.zeros_like(X)
    assert np.all(otw.ffn(z, W1, W2)["Y"] == 0) and np.all(otw.ffn(z, W1, W2, W3)["Y"] == 0)
    dY = r.standard_normal((rows, n_model))
    np.testing.assert_allclose(otw.ffn(z, W1, W2, None, dY)["dX"], 0.5 * dY @ W2 @ W1, atol=1e-14)
    # large positive pre-activations: gelu(a) -> a, so the block is the product of its two matrices
    Xp, W1p = np.abs(X) + 1, np.abs(W1) * 10 + 10
    np.testing.assert_allclose(otw.ffn(Xp, W1p, W2)["Y"], Xp @ W1p.T @ W2.T, rtol=1e-12)
    # large negative: gelu(a) -> 0
    np.testing.assert_allclose(otw.ffn(Xp, -W1p, W2)["Y"], 0, atol=1e-12)
    # SwiGLU is linear in W3 and in W2
    a = otw.ffn(X, W1, W2, W3)["Y"]
    np.testing.assert_allclose(otw.ffn(X, W1, W2, 3 * W3)["Y"], 3 * a, rtol=1e-13)
    # central finite differences of L = sum(Y * dY) in one coordinate of each argument
    eps = 1e-6
    for sw in (False, True):
        g = otw.ffn(X, W1, W2, W3 if sw else None, dY)
        L = lambda X_, W1_, W2_, W3_: float((otw.ffn(X_, W1_, W2_, W3_ if sw else None)["Y"] * dY).sum())
        for name, arr, idx in (("dX", 0, (2, 1)), ("dW1", 1, (3, 2)), ("dW2", 2, (1, 4))) + ((("dW3", 3, (5, 0)),) if sw else ()):
            args_p = [X.copy(), W1.copy(), W2.copy(), W3.copy()]
            args_m = [X.copy(), W1.copy(), W2.copy(), W3.copy()]
            args_p[arr][idx] += eps
            args_m[arr][idx] -= eps
            fd = (L(*args_p) - L(*args_m)) / (2 * eps)
            assert abs(fd - g[name][idx]) < 1e-6 * max(1.0, abs(fd)), (sw, name, fd, g[name][idx])


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
    # feed-forward workspace: [chunk, n_ffn] bf16 tiles, 2 (GELU) or 3 (SwiGLU), one more backward
    tile = (250 * 1024 * 2 + 255) // 256 * 256
    assert TW.fpdt_tw_ffn_workspace_bytes(1000, 256, 1024, TW.FPDT_TW_GELU, 4, False) == 2 * tile
    assert TW.fpdt_tw_ffn_workspace_bytes(1000, 256, 1024, TW.FPDT_TW_SWIGLU, 4, False) == 3 * tile
    assert TW.fpdt_tw_ffn_workspace_bytes(1000, 256, 1024, TW.FPDT_TW_SWIGLU, 4, True) == 4 * tile
    assert TW.fpdt_tw_ffn_workspace_bytes(1000, 256, 1024, 7, 4, True) == 0
    assert L.fpdt_tw_ffn_fwd(p, p, None, p, p, 1000, 256, 1024, TW.FPDT_TW_SWIGLU, 4, 0x100000, 1 << 40, None) == 1
    assert "W3" in TW.fpdt_tw_last_error()
    assert L.fpdt_tw_ffn_fwd(p, p, None, p, p, 1000, 256, 1024, TW.FPDT_TW_GELU, 4, 0x100000, 16, None) == 3
    assert L.fpdt_tw_ffn_bwd(p, p, None, p, p, None, None, None, None, 1000, 256, 1024, TW.FPDT_TW_GELU, 4,
                             0x100000, 1 << 40, None) == 1
    assert L.fpdt_tw_linear_fwd(p, p, None, 1000, 256, 768, 4, None) == 1
    assert L.fpdt_tw_linear_fwd(p, p, p, 1000, 256, 768, 0, None) == 1
    assert L.fpdt_tw_linear_bwd(p, p, p, None, None, 1000, 0, 768, 4, None) == 1


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


def _rowwise_ok(name, got, ref, rel=2e-2):
    """|got - ref| <= rel * rms(ref row) + half a bf16 ulp of ref (at most 2^-8 |ref|: 8 significand
    bits), element by element."""
    rms = np.sqrt((ref ** 2).mean(axis=1, keepdims=True))
    budget = rel * rms + 2.0 ** -8 * np.abs(ref) + 1e-9
    err = np.abs(got - ref)
    assert (err <= budget).all(), (name, float((err / budget).max()))


@pytest.mark.gpu
@pytest.mark.parametrize("rows,n_in,n_out,n_chunks", [(1000, 256, 768, 3), (333, 136, 520, 7)])
def test_gpu_linear_matches_oracle(rows, n_in, n_out, n_chunks):
    print("[case] chunked linear", rows, n_in, n_out, n_chunks, flush=True)
    g = torch.Generator().manual_seed(41)
    X = torch.randn(rows, n_in, generator=g).to(torch.bfloat16)
    W = (torch.randn(n_out, n_in, generator=g) * n_in ** -0.5).to(torch.bfloat16)
    dY = torch.randn(rows, n_out, generator=g).to(torch.bfloat16)
    ref = otw.linear(X.double().numpy(), W.double().numpy(), dY.double().numpy())
    Xd, Wd, dYd = X.cuda(), W.cuda(), dY.cuda()
    Y = torch.empty(rows, n_out, dtype=torch.bfloat16, device="cuda")
    dX = torch.empty_like(Xd)
    dW = torch.zeros(n_out, n_in, device="cuda")
    TW.fpdt_tw_linear_fwd(Xd, Wd, Y, n_chunks)
    TW.fpdt_tw_linear_bwd(Xd, Wd, dYd, dX, dW, n_chunks)
    torch.cuda.synchronize()
    # fp32 accumulation of exact products, one rounding to bf16 on store
    _rowwise_ok("Y", Y.float().cpu().numpy(), ref["Y"], rel=1e-4)
    _rowwise_ok("dX", dX.float().cpu().numpy(), ref["dX"], rel=1e-4)
    np.testing.assert_allclose(dW.cpu().numpy(), ref["dW"], atol=1e-4 * float(np.abs(ref["dW"]).max()))
    # one chunk gives the same bits for Y and dX (each row is its own dot products)
    Y1, dX1 = torch.empty_like(Y), torch.empty_like(dX)
    TW.fpdt_tw_linear_fwd(Xd, Wd, Y1, 1)
    TW.fpdt_tw_linear_bwd(Xd, Wd, dYd, dX1, None, 1)
    torch.cuda.synchronize()
    _rowwise_ok("Y vs one chunk", Y.float().cpu().numpy(), Y1.float().cpu().numpy().astype(np.float64), rel=1e-4)
    _rowwise_ok("dX vs one chunk", dX.float().cpu().numpy(), dX1.float().cpu().numpy().astype(np.float64), rel=1e-4)


@pytest.mark.gpu
@pytest.mark.parametrize("act,rows,n_model,n_ffn,n_chunks", [
    ("gelu", 1000, 256, 1024, 4), ("swiglu", 1000, 256, 688, 4), ("swiglu", 257, 128, 349, 5), ("gelu", 64, 64, 256, 1)])
def test_gpu_ffn_matches_oracle(act, rows, n_model, n_ffn, n_chunks):
    print("[case] chunked ffn", act, rows, n_model, n_ffn, n_chunks, flush=True)
    sw = act == "swiglu"
    code = TW.FPDT_TW_SWIGLU if sw else TW.FPDT_TW_GELU
    g = torch.Generator().manual_seed(43)
    X = torch.randn(rows, n_model, generator=g).to(torch.bfloat16)
    W1 = (torch.randn(n_ffn, n_model, generator=g) * n_model ** -0.5).to(torch.bfloat16)
    W3 = (torch.randn(n_ffn, n_model, generator=g) * n_model ** -0.5).to(torch.bfloat16)
    W2 = (torch.randn(n_model, n_ffn, generator=g) * n_ffn ** -0.5).to(torch.bfloat16)
    dY = torch.randn(rows, n_model, generator=g).to(torch.bfloat16)
    f64 = lambda t: t.double().numpy()
    ref = otw.ffn(f64(X), f64(W1), f64(W2), f64(W3) if sw else None, f64(dY))
    Xd, W1d, W2d, dYd = X.cuda(), W1.cuda(), W2.cuda(), dY.cuda()
    W3d = W3.cuda() if sw else None
    Y, dX = torch.empty_like(Xd), torch.empty_like(Xd)
    dW1 = torch.zeros(n_ffn, n_model, device="cuda")
    dW3 = torch.zeros(n_ffn, n_model, device="cuda") if sw else None
    dW2 = torch.zeros(n_model, n_ffn, device="cuda")
    wf = torch.empty(TW.fpdt_tw_ffn_workspace_bytes(rows, n_model, n_ffn, code, n_chunks, False), dtype=torch.uint8, device="cuda")
    wb = torch.empty(TW.fpdt_tw_ffn_workspace_bytes(rows, n_model, n_ffn, code, n_chunks, True), dtype=torch.uint8, device="cuda")
    TW.fpdt_tw_ffn_fwd(Xd, W1d, W3d, W2d, Y, code, n_chunks, wf)
    TW.fpdt_tw_ffn_bwd(Xd, W1d, W3d, W2d, dYd, dX, dW1, dW3, dW2, code, n_chunks, wb)
    torch.cuda.synchronize()
    # intermediates [chunk, n_ffn] are rounded to bf16 between GEMMs (relative 2^-9 each, independent
    # across the contraction): 2e-2 of the reference row's RMS covers them with a wide margin
    _rowwise_ok("Y", Y.float().cpu().numpy(), ref["Y"])
    _rowwise_ok("dX", dX.float().cpu().numpy(), ref["dX"])
    _rowwise_ok("dW1", dW1.cpu().numpy(), ref["dW1"])
    _rowwise_ok("dW2", dW2.cpu().numpy(), ref["dW2"])
    if sw:
        _rowwise_ok("dW3", dW3.cpu().numpy(), ref["dW3"])
    # the weight gradients are accumulated into, dX is overwritten
    TW.fpdt_tw_ffn_bwd(Xd, W1d, W3d, W2d, dYd, dX, dW1, None, None, code, n_chunks, wb)
    torch.cuda.synchronize()
    _rowwise_ok("dW1 twice", dW1.cpu().numpy(), 2 * ref["dW1"])
    _rowwise_ok("dX again", dX.float().cpu().numpy(), ref["dX"])
    _rowwise_ok("dW2 untouched", dW2.cpu().numpy(), ref["dW2"])
    if n_chunks > 1:
        w1 = TW.fpdt_tw_ffn_workspace_bytes(rows, n_model, n_ffn, code, 1, True)
        assert wb.numel() * 2 < w1


# ------------------------------------------------------------------ Llama-8B widths, sampled
@pytest.mark.gpu
def test_gpu_ffn_llama_widths_sampled_rows_and_weight_slices():
    """Model 4096, FFN 14336, SwiGLU, 8192 tokens in 4 chunks.  Rows are independent, so the
    oracle evaluated on sampled rows gives their Y and dX exactly; a hidden unit's weight
    gradients depend only on its own column of the intermediates, so the oracle evaluated on
    a slice of hidden units gives those rows of dW1 / dW3 and columns of dW2 exactly."""
    rows, n_model, n_ffn, n_chunks = 8192, 4096, 14336, 4
    print("[case] ffn llama widths", rows, n_model, n_ffn, n_chunks, flush=True)
    g = torch.Generator(device="cuda").manual_seed(47)
    bf = lambda *s, std=1.0: (torch.randn(*s, device="cuda", generator=g) * std).to(torch.bfloat16)
    X, dY = bf(rows, n_model), bf(rows, n_model)
    W1, W3, W2 = bf(n_ffn, n_model, std=n_model ** -0.5), bf(n_ffn, n_model, std=n_model ** -0.5), bf(n_model, n_ffn, std=n_ffn ** -0.5)
    code = TW.FPDT_TW_SWIGLU
    Y, dX = torch.empty_like(X), torch.empty_like(X)
    dW1, dW3, dW2 = (torch.zeros_like(w, dtype=torch.float32) for w in (W1, W3, W2))
    wb = torch.empty(TW.fpdt_tw_ffn_workspace_bytes(rows, n_model, n_ffn, code, n_chunks, True), dtype=torch.uint8, device="cuda")
    TW.fpdt_tw_ffn_fwd(X, W1, W3, W2, Y, code, n_chunks, wb)
    TW.fpdt_tw_ffn_bwd(X, W1, W3, W2, dY, dX, dW1, dW3, dW2, code, n_chunks, wb)
    torch.cuda.synchronize()
    f64 = lambda t: t.double().cpu().numpy()
    r = np.random.default_rng(5)
    rs = np.sort(r.choice(rows, 24, replace=False))
    rs[0], rs[-1] = 0, rows - 1
    ref = otw.ffn(f64(X[rs]), f64(W1), f64(W2), f64(W3), f64(dY[rs]))
    _rowwise_ok("Y rows", f64(Y[rs]), ref["Y"])
    _rowwise_ok("dX rows", f64(dX[rs]), ref["dX"])
    del ref
    fs = np.sort(r.choice(n_ffn, 12, replace=False))
    fs[0], fs[-1] = 0, n_ffn - 1
    ref = otw.ffn(f64(X), f64(W1[fs]), f64(W2[:, fs]), f64(W3[fs]), f64(dY))
    _rowwise_ok("dW1 slice", f64(dW1[fs]), ref["dW1"])
    _rowwise_ok("dW3 slice", f64(dW3[fs]), ref["dW3"])
    _rowwise_ok("dW2 slice", f64(dW2[:, fs]).T.copy(), ref["dW2"].T.copy())


@pytest.mark.gpu
def test_gpu_loss_llama_vocabulary():
    """Hidden 4096, vocabulary 128256 (Llama-3), 1024 tokens in 4 chunks, against the full oracle."""
    rows, hidden, vocab, n_chunks = 1024, 4096, 128256, 4
    print("[case] loss llama vocabulary", rows, hidden, vocab, n_chunks, flush=True)
    g = torch.Generator(device="cuda").manual_seed(53)
    H = torch.randn(rows, hidden, device="cuda", generator=g).to(torch.bfloat16)
    W = (torch.randn(vocab, hidden, device="cuda", generator=g) * hidden ** -0.5).to(torch.bfloat16)
    t = torch.randint(0, vocab, (rows,), device="cuda", generator=g, dtype=torch.int32)
    loss, lse = torch.empty(rows, device="cuda"), torch.empty(rows, device="cuda")
    dH = torch.empty_like(H)
    dW = torch.zeros(vocab, hidden, device="cuda")
    ws = torch.empty(TW.fpdt_tw_loss_workspace_bytes(rows, hidden, vocab, n_chunks), dtype=torch.uint8, device="cuda")
    TW.fpdt_tw_loss_fwd_bwd(H, W, t, 1.0 / rows, loss, lse, dH, dW, n_chunks, ws)
    torch.cuda.synchronize()
    print("[step] oracle", flush=True)
    ref = otw.cross_entropy(H.double().cpu().numpy(), W.double().cpu().numpy(), t.cpu().numpy(), grad_scale=1.0 / rows)
    print("[step] compare", flush=True)
    # 4096-term fp32 dot products of O(1) logits: a few 1e-5 of round-off each
    np.testing.assert_allclose(loss.cpu().numpy(), ref["loss"], atol=1e-3)
    np.testing.assert_allclose(lse.cpu().numpy(), ref["lse"], atol=1e-3)
    _rowwise_ok("dH", dH.float().cpu().numpy(), ref["dH"])
    # a vocabulary row that is nobody's target has a gradient of ~1024 probabilities of ~1e-5 each,
    # every one rounded to bf16 before the GEMM: same relative budget per row
    _rowwise_ok("dW", dW.cpu().numpy(), ref["dW"])


@pytest.mark.gpu
def test_gpu_tokenwise_calls_replay_from_a_graph():
    """FFN forward + backward and the fused loss captured in one HIP graph (library GEMMs and the
    row / activation kernels on the captured stream), replayed three times with eager work in
    between; every replay equals the eager result bit for bit."""
    rows, n_model, n_ffn, vocab, n_chunks = 1024, 256, 688, 1536, 4
    print("[case] token-wise graph", rows, n_model, n_ffn, vocab, flush=True)
    g = torch.Generator(device="cuda").manual_seed(61)
    bf = lambda *s, std=1.0: (torch.randn(*s, device="cuda", generator=g) * std).to(torch.bfloat16)
    X, dY = bf(rows, n_model), bf(rows, n_model)
    W1, W3, W2 = bf(n_ffn, n_model, std=n_model ** -0.5), bf(n_ffn, n_model, std=n_model ** -0.5), bf(n_model, n_ffn, std=n_ffn ** -0.5)
    Wv = bf(vocab, n_model, std=n_model ** -0.5)
    tgt = torch.randint(0, vocab, (rows,), device="cuda", generator=g, dtype=torch.int32)
    code = TW.FPDT_TW_SWIGLU
    Y, dX, dH = torch.empty_like(X), torch.empty_like(X), torch.empty_like(X)
    dW1, dW3, dW2 = (torch.zeros_like(w, dtype=torch.float32) for w in (W1, W3, W2))
    dWv = torch.zeros_like(Wv, dtype=torch.float32)
    loss, lse = torch.empty(rows, device="cuda"), torch.empty(rows, device="cuda")
    wb = torch.empty(TW.fpdt_tw_ffn_workspace_bytes(rows, n_model, n_ffn, code, n_chunks, True), dtype=torch.uint8, device="cuda")
    wl = torch.empty(TW.fpdt_tw_loss_workspace_bytes(rows, n_model, vocab, n_chunks), dtype=torch.uint8, device="cuda")

    def step():
        TW.fpdt_tw_ffn_fwd(X, W1, W3, W2, Y, code, n_chunks, wb)
        TW.fpdt_tw_ffn_bwd(X, W1, W3, W2, dY, dX, dW1, dW3, dW2, code, n_chunks, wb)
        TW.fpdt_tw_loss_fwd_bwd(Y, Wv, tgt, 1.0 / rows, loss, lse, dH, dWv, n_chunks, wl)

    outs = {"Y": Y, "dX": dX, "dH": dH, "dW1": dW1, "dW3": dW3, "dW2": dW2, "dWv": dWv, "loss": loss, "lse": lse}

    def reset():  # written outputs are poisoned, accumulated-into ones start from zero
        for n, t in outs.items():
            t.zero_() if n.startswith("dW") else t.fill_(float("nan"))

    step()  # first call: sizes the library's operand scratch pool and loads its kernels outside any capture
    reset()
    step()
    torch.cuda.synchronize()
    want = {n: t.clone() for n, t in outs.items()}
    gr = torch.cuda.CUDAGraph()
    with torch.cuda.graph(gr, stream=torch.cuda.Stream()):
        step()
    for rep in range(3):
        reset()
        torch.cuda.synchronize()
        gr.replay()
        torch.cuda.synchronize()
        for n, t in outs.items():
            assert torch.equal(t.view(torch.uint8), want[n].view(torch.uint8)), (n, rep)
