"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times:
sampled query rows (O, LSE, dQ) and the tail window of key rows (dK, dV) against the fp64
oracle, plus invariants that hold at any size over the whole tensors."""
import numpy as np
import pytest
import torch

from paper_2408_16978_amd import binding as B
from paper_2408_16978_amd import inputs, runner
from oracle import definition

import parity

pytestmark = pytest.mark.gpu


def sample_rows(cfg, n_random, seed):
    """Stratified: sequence ends, both sides of every kind of chunk boundary, 256-row tile
    boundaries, and uniform-random rows."""
    S, C = cfg.S, cfg.chunk
    rows = {0, 1, 2, 31, 32, 63, 64, 255, 256, 257, S - 1, S - 2, S - 257}
    for m in (1, cfg.u // 2, cfg.u - 1):
        if 0 < m < cfg.u:
            rows |= {m * C - 1, m * C, m * C + 1}
    rng = np.random.default_rng(seed)
    rows |= set(int(x) for x in rng.integers(0, S, size=n_random))
    return np.array(sorted(r for r in rows if 0 <= r < S), dtype=np.int64)


def run_config(name, n_random, tail, seed=7):
    cfg = inputs.CONFIGS[name]
    print("[case]", cfg, flush=True)
    Q, K, V, dO = inputs.make_qkvdo(cfg.S, cfg.Hq, cfg.Hkv, cfg.D, cfg.dtype, seed, device="cuda")
    flags = (B.FPDT_KV_ON_HOST if cfg.kv_on_host else 0) | (B.FPDT_ACT_ON_HOST if cfg.act_on_host else 0)
    b = runner.make_buffers(Q, K, V, dO, cfg.chunk, cfg.scale, flags)
    runner.forward(b)
    runner.backward(b)
    torch.cuda.synchronize()
    print("[gpu done]", name, flush=True)
    is_bf16 = cfg.dtype == "bf16"
    g = cfg.Hq // cfg.Hkv

    # ---- sampled query rows: O, LSE, dQ ----
    rows = sample_rows(cfg, n_random, seed)
    ridx = torch.from_numpy(rows)
    K64, V64 = parity.to64(K), parity.to64(V)
    ref = definition.rows(parity.to64(Q[ridx.cuda()]), K64, V64, rows, cfg.scale,
                          dOr=parity.to64(dO[ridx.cuda()]))
    got_O = b.O[ridx.to(b.O.device)]
    got_dQ = b.dQ[ridx.to(b.dQ.device)]
    got_LSE = b.LSE[:, ridx.to(b.LSE.device)]
    print("O", parity.check("O", got_O, ref["O"], is_bf16),
          "LSE", parity.check("LSE", got_LSE, ref["LSE"], is_bf16),
          "dQ", parity.check("dQ", got_dQ, ref["dQ"], is_bf16), flush=True)

    # ---- tail window of keys: dK, dV exact (only the last `tail` queries reach them) ----
    t = definition.tail_window(parity.to64(Q[cfg.S - tail:]), parity.to64(dO[cfg.S - tail:]), K64,
                               V64, tail, cfg.scale)
    print("dK", parity.check("dK", b.dK[cfg.S - tail:], t["dK"], is_bf16),
          "dV", parity.check("dV", b.dV[cfg.S - tail:], t["dV"], is_bf16), flush=True)
    del K64, V64

    # ---- invariants over the whole tensors (fp64 reductions of the GPU outputs) ----
    dVd = b.dV.cuda().double()
    want = dO.double().view(cfg.S, cfg.Hkv, g, cfg.D).sum(dim=(0, 2))
    got = dVd.sum(dim=0)
    # rows of p sum to one: sum_j dV_j = sum of dO over the group's heads and all rows.
    # Measured deviation is 2e-5 (S=256K) .. 7e-5 (S=1M) of the norm: bf16 rounding of dV and
    # the fp32 accumulation of the softmax normaliser over up to S keys.  A dropped or doubled
    # chunk pair would move it by 1/u or more (>= 3e-2).
    rel = (got - want).norm() / want.norm()
    print("sum-dV invariant: relative error", float(rel), flush=True)
    assert rel < 1e-3, "sum dV invariant"
    # gauge identity: sum_h Q_h^T dQ_h = dK^T K per KV head (D x D); ties the full dK tensor
    # to dQ, which the sampled rows pin.
    Qd, dQd = Q.double(), b.dQ.cuda().double()
    Kd, dKd = K.double(), b.dK.cuda().double()
    for kv in range(cfg.Hkv):
        lhs = sum(Qd[:, h].T @ dQd[:, h] for h in range(kv * g, (kv + 1) * g))
        rhs = dKd[:, kv].T @ Kd[:, kv]
        rel = (lhs - rhs).norm() / rhs.norm()
        print("gauge identity kv head", kv, "relative Frobenius error", float(rel), flush=True)
        assert rel < 2e-2
    # K/V untouched on the host, nothing non-finite anywhere
    for n in ("O", "LSE", "dQ", "dK", "dV"):
        assert torch.isfinite(getattr(b, n)).all(), n


def test_config2_gpt2p7b_64k():
    run_config("gpt2p7b_64k", n_random=48, tail=64)


def test_config3_llama8b_256k():
    run_config("llama8b_256k", n_random=48, tail=32)


def test_config5_llama70b_1m_all_offloaded():
    run_config("llama70b_1m", n_random=24, tail=16)


def test_config4_llama8b_2m_kv_offloaded():
    run_config("llama8b_2m", n_random=16, tail=8)


def test_uniform_average_closed_form_at_256k():
    """K == 0: O_i is the running mean of V and LSE_i = log(i+1) at any S (closed form)."""
    S, chunk, Hq, Hkv, D = 262144, 65536, 8, 2, 128
    print("[case] K=0 closed form", S, flush=True)
    Q, K, V, dO = inputs.make_qkvdo(S, Hq, Hkv, D, "bf16", 9, device="cuda")
    K.zero_()
    b = runner.make_buffers(Q, K, V, dO, chunk, D ** -0.5, 0, bwd=False)
    runner.forward(b)
    torch.cuda.synchronize()
    lse = torch.log(torch.arange(1, S + 1, device="cuda", dtype=torch.float64))
    assert (b.LSE.double() - lse[None, :]).abs().max() < 1e-3
    mean = V.double().cumsum(dim=0) / torch.arange(1, S + 1, device="cuda", dtype=torch.float64)[:, None, None]
    ref = mean.repeat_interleave(Hq // Hkv, dim=1)
    idx = torch.arange(0, S, 997, device="cuda")
    parity.check("O", b.O[idx], ref[idx].cpu().numpy(), True)


def test_blocksparse_256k_kv_offloaded_sampled():
    """Block-sparse K/V fetch (Sec. 5.5) at the Llama-8B head share, S = 256K in 8 chunks of 32K,
    K/V in pinned host memory, a seeded mask that keeps about half of the below-diagonal pairs:
    sampled query rows and the tail window of keys against the masked oracle."""
    S, chunk, Hq, Hkv, D = 262144, 32768, 8, 2, 128
    u, scale, tail = S // chunk, D ** -0.5, 32
    mask = np.tril(np.random.default_rng(21).random((u, u)) < 0.5)
    np.fill_diagonal(mask, True)
    mask[5, :5] = False  # one query chunk that keeps only its diagonal
    print("[case] block-sparse 256K, kept pairs", int(mask.sum()), "of", u * (u + 1) // 2, flush=True)
    Q, K, V, dO = inputs.make_qkvdo(S, Hq, Hkv, D, "bf16", 23, device="cuda")
    b = runner.make_buffers(Q, K, V, dO, chunk, scale, B.FPDT_KV_ON_HOST, chunk_mask=mask)
    runner.forward(b)
    runner.backward(b)
    torch.cuda.synchronize()
    h2d, _ = B.fpdt_last_link_bytes()
    print("[gpu done] backward fetched", h2d / 2 ** 20, "MiB", flush=True)

    rows = {0, 1, 255, 256, S - 1, S - 2}
    for m in range(1, u):
        rows |= {m * chunk - 1, m * chunk, m * chunk + 1, m * chunk + 255, m * chunk + 256}
    rows |= set(int(x) for x in np.random.default_rng(22).integers(0, S, size=24))
    rows = np.array(sorted(rows), dtype=np.int64)
    ridx = torch.from_numpy(rows).cuda()
    K64, V64 = parity.to64(K), parity.to64(V)
    ref = definition.rows(parity.to64(Q[ridx]), K64, V64, rows, scale, dOr=parity.to64(dO[ridx]),
                          chunk=chunk, chunk_mask=mask)
    print("O", parity.check("O", b.O[ridx], ref["O"], True),
          "LSE", parity.check("LSE", b.LSE[:, ridx], ref["LSE"], True),
          "dQ", parity.check("dQ", b.dQ[ridx], ref["dQ"], True), flush=True)
    # the last `tail` keys are reached by the last `tail` queries only (their chunk's diagonal pair)
    idx = np.arange(S - tail, S)
    Qw, dOw = parity.to64(Q[S - tail:]), parity.to64(dO[S - tail:])
    r = definition.rows(Qw, K64, V64, idx, scale, dOr=dOw, chunk=chunk, chunk_mask=mask)
    dK, dV = definition.cols(Qw, dOw, r["LSE"], r["Delta"], S - tail, K64[S - tail:], V64[S - tail:], idx, S,
                             scale, chunk=chunk, chunk_mask=mask)
    print("dK", parity.check("dK", b.dK[S - tail:], dK, True), "dV", parity.check("dV", b.dV[S - tail:], dV, True), flush=True)
    for n in ("O", "LSE", "dQ", "dK", "dV"):
        assert torch.isfinite(getattr(b, n)).all(), n
