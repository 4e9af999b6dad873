"""Throughput and workspace of the token-wise chunked operations (include/fpdt_tokenwise.h) as a
function of the chunk count, at Llama-8B layer shapes.  Prints one JSON line per (operation,
chunk count).  `python -m paper_2408_16978_amd.bench_tokenwise [--rows 65536] [--chunks 1,4,16,64]`.
"""
import argparse
import json

import torch

from . import tokenwise as TW


def _time(fn, iters):
    fn()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(iters):
        fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / iters


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--rows", type=int, default=65536, help="tokens on this GPU")
    ap.add_argument("--n-model", type=int, default=4096)
    ap.add_argument("--n-ffn", type=int, default=14336)
    ap.add_argument("--n-qkv", type=int, default=6144, help="(Hq + 2 Hkv) * D")
    ap.add_argument("--vocab", type=int, default=128256)
    ap.add_argument("--chunks", default="1,2,4,8,16,64")
    ap.add_argument("--iters", type=int, default=3)
    ap.add_argument("--max-workspace-gib", type=float, default=64.0)
    a = ap.parse_args()
    if not torch.cuda.is_available():
        raise SystemExit("needs a GPU")
    TW.load()
    dev = "cuda"
    g = torch.Generator(device=dev).manual_seed(7)
    rows, nm, nf, nq, nv = a.rows, a.n_model, a.n_ffn, a.n_qkv, a.vocab
    bf = lambda *s, std=1.0: (torch.randn(*s, device=dev, generator=g) * std).to(torch.bfloat16)
    X, dY = bf(rows, nm), bf(rows, nm)
    W1, W3, W2 = bf(nf, nm, std=nm ** -0.5), bf(nf, nm, std=nm ** -0.5), bf(nm, nf, std=nf ** -0.5)
    Wq, Wv = bf(nq, nm, std=nm ** -0.5), bf(nv, nm, std=nm ** -0.5)
    tgt = torch.randint(0, nv, (rows,), device=dev, generator=g, dtype=torch.int32)
    Y, dX = torch.empty_like(X), torch.empty_like(X)
    Yq = torch.empty(rows, nq, dtype=torch.bfloat16, device=dev)
    dW1, dW3, dW2 = (torch.zeros_like(w, dtype=torch.float32) for w in (W1, W3, W2))
    dWq, dWv = torch.zeros_like(Wq, dtype=torch.float32), torch.zeros_like(Wv, dtype=torch.float32)
    loss, lse = torch.empty(rows, device=dev), torch.empty(rows, device=dev)
    cap = int(a.max_workspace_gib * 2 ** 30)
    for n in [int(c) for c in a.chunks.split(",")]:
        ops = []
        wf = TW.fpdt_tw_ffn_workspace_bytes(rows, nm, nf, TW.FPDT_TW_SWIGLU, n, False)
        wb = TW.fpdt_tw_ffn_workspace_bytes(rows, nm, nf, TW.FPDT_TW_SWIGLU, n, True)
        wl = TW.fpdt_tw_loss_workspace_bytes(rows, nm, nv, n)
        ops.append(("linear_fwd", 0, 2.0 * rows * nm * nq, lambda ws: TW.fpdt_tw_linear_fwd(X, Wq, Yq, n)))
        ops.append(("linear_bwd", 0, 4.0 * rows * nm * nq, lambda ws: TW.fpdt_tw_linear_bwd(X, Wq, Yq, dX, dWq, n)))
        ops.append(("ffn_swiglu_fwd", wf, 6.0 * rows * nm * nf,
                    lambda ws: TW.fpdt_tw_ffn_fwd(X, W1, W3, W2, Y, TW.FPDT_TW_SWIGLU, n, ws)))
        # backward = 2 recomputed GEMMs + dHh + dW2 + 2 dX + dW1 + dW3 = 8 GEMMs of 2 rows nm nf
        ops.append(("ffn_swiglu_bwd", wb, 16.0 * rows * nm * nf,
                    lambda ws: TW.fpdt_tw_ffn_bwd(X, W1, W3, W2, dY, dX, dW1, dW3, dW2, TW.FPDT_TW_SWIGLU, n, ws)))
        ops.append(("loss_fwd_bwd", wl, 6.0 * rows * nm * nv,
                    lambda ws: TW.fpdt_tw_loss_fwd_bwd(X, Wv, tgt, 1.0 / rows, loss, lse, dX, dWv, n, ws)))
        for name, wbytes, flops, fn in ops:
            rec = {"op": name, "rows": rows, "n_chunks": n, "workspace_gib": round(wbytes / 2 ** 30, 3)}
            if wbytes > cap:
                rec["skipped"] = "workspace above --max-workspace-gib"
            else:
                ws = torch.empty(max(wbytes, 256), dtype=torch.uint8, device=dev)
                ms = _time(lambda: fn(ws), a.iters)
                del ws
                rec.update(ms=round(ms, 3), tflops=round(flops / ms * 1e-9, 1))
            print(json.dumps(rec), flush=True)


if __name__ == "__main__":
    main()
