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


# One forward + backward per workload, shared by that workload's tests (they run back to back);
# only the latest workload is kept, so device memory holds one set of tensors at a time.
_RUN = {}


def gpu_run(name, seed=7):
    if _RUN.get("name") != name:
        _RUN.clear()
        torch.cuda.empty_cache()
        cfg = inputs.CONFIGS[name]
        print("[case]", cfg, flush=True)
        Q, K, V, dO = inputs.make_qkvdo(cfg.S, cfg.Hq, cfg.Hkv, cfg.D, cfg.dtype, seed, device="cuda")
        flags = (B.FPDT_KV_ON_HOST if cfg.kv_on_host else 0) | (B.FPDT_ACT_ON_HOST if cfg.act_on_host else 0) | \
            (B.FPDT_BWD_STORE_DS if cfg.store_ds else 0)   # the launch configuration bench.py times
        b = runner.make_buffers(Q, K, V, dO, cfg.chunk, cfg.scale, flags)
        runner.forward(b)
        runner.backward(b)
        torch.cuda.synchronize()
        print("[gpu done]", name, flush=True)
        _RUN.update(name=name, cfg=cfg, seed=seed, Q=Q, K=K, V=V, dO=dO, b=b)
    r = _RUN
    return r["cfg"], r["Q"], r["K"], r["V"], r["dO"], r["b"]


def check_rows_and_tail(name, n_random, tail):
    """Sampled query rows (O, LSE, dQ) and the last `tail` keys (dK, dV; reached by the last `tail`
    queries only) against the oracle, unconditionally."""
    cfg, Q, K, V, dO, b = gpu_run(name)
    is_bf16 = cfg.dtype == "bf16"
    rows = sample_rows(cfg, n_random, _RUN["seed"])
    ridx = torch.from_numpy(rows)
    K64, V64 = parity.to64(K), parity.to64(V)
    ref = definition.rows(parity.to64(Q[ridx.cuda()]), K64, V64, rows, cfg.scale,
                          dOr=parity.to64(dO[ridx.cuda()]))
    got_O = b.O[ridx.to(b.O.device)]
    got_dQ = b.dQ[ridx.to(b.dQ.device)]
    got_LSE = b.LSE[:, ridx.to(b.LSE.device)]
    parity.check("O", got_O, ref["O"], is_bf16, strict=True, label=name + " sampled rows")
    parity.check("LSE", got_LSE, ref["LSE"], is_bf16)
    parity.check("dQ", got_dQ, ref["dQ"], is_bf16, strict=True, label=name + " sampled rows")
    t = definition.tail_window(parity.to64(Q[cfg.S - tail:]), parity.to64(dO[cfg.S - tail:]), K64,
                               V64, tail, cfg.scale)
    parity.check("dK", b.dK[cfg.S - tail:], t["dK"], is_bf16, strict=True, label=name + " tail window")
    parity.check("dV", b.dV[cfg.S - tail:], t["dV"], is_bf16, strict=True, label=name + " tail window")


def sample_cols(cfg, per_chunk, seed):
    """Key rows for the column check: `per_chunk` random keys in EVERY chunk, both sides of chunk
    boundaries and of 256-key workgroup boundaries, the first keys, and the whole last workgroup
    (256 keys: every wave of it, masked steps included)."""
    S, C = cfg.S, cfg.chunk
    rng = np.random.default_rng(seed + 100)
    cols = {0, 1, 63, 64, 255, 256}
    for m in range(cfg.u):
        cols |= set(int(m * C + x) for x in rng.integers(0, C, size=per_chunk))
    for m in (1, cfg.u // 2, cfg.u - 1):
        if 0 < m < cfg.u:
            cols |= {m * C - 1, m * C, m * C + 255, m * C + 256}
    cols |= set(range(S - 256, S))
    return np.array(sorted(c for c in cols if 0 <= c < S), dtype=np.int64)


def check_columns_conditional(name, per_chunk):
    """dK, dV of sampled key rows anywhere in the sequence (Sec. 4.2: every key chunk gathers from
    all later query chunks).  CONDITIONAL check: the oracle's column evaluator needs LSE_i and
    Delta_i of every query row i >= j, which the oracle itself cannot produce at these sizes
    (that is the whole S^2 forward), so it is fed the GPU forward's LSE and
    Delta = rowsum(dO * O_gpu) in fp64 (both pinned row by row through the sampled-row test; the
    first 256 rows take the oracle's own exact Delta, as the library does).  Everything else --
    scores, probabilities, dP, the sums over all later rows and over the group's heads -- is the
    oracle's fp64 arithmetic, so a key block that is skipped, doubled, mis-indexed or mis-carried
    between chunk pairs shows here wherever it sits."""
    cfg, Q, K, V, dO, b = gpu_run(name)
    S = cfg.S
    cols = sample_cols(cfg, per_chunk, _RUN["seed"])
    print("[columns]", name, len(cols), "key rows, first", int(cols[0]), flush=True)
    # Delta from the GPU's O, in fp64, chunk by chunk on the device that holds dO
    delta = torch.empty((S, cfg.Hq), dtype=torch.float64)
    step = 1 << 16
    for r0 in range(0, S, step):
        o = b.O[r0:r0 + step].cuda().double()
        delta[r0:r0 + step] = (o * dO[r0:r0 + step].double()).sum(dim=-1).cpu()
    lse = b.LSE.cpu().double()
    K64, V64 = parity.to64(K), parity.to64(V)
    head = np.arange(256)
    hidx = torch.from_numpy(head).cuda()
    exact = definition.rows(parity.to64(Q[hidx]), K64, V64, head, cfg.scale, dOr=parity.to64(dO[hidx]))
    delta[:256] = torch.from_numpy(exact["Delta"].T)
    Q64, dO64 = parity.to64(Q), parity.to64(dO)
    print("[columns] inputs widened", flush=True)
    dK, dV = definition.cols(Q64, dO64, lse.numpy(), delta.numpy().T, 0, K64[cols], V64[cols], cols, S,
                             cfg.scale)
    del Q64, dO64
    cidx = torch.from_numpy(cols)
    parity.check("dK", b.dK[cidx.to(b.dK.device)], dK, True, strict=True, label=name + " sampled key rows (conditional)")
    parity.check("dV", b.dV[cidx.to(b.dV.device)], dV, True, strict=True, label=name + " sampled key rows (conditional)")


def check_invariants(name):
    """Identities over the whole output tensors (fp64 reductions of the GPU results)."""
    cfg, Q, K, V, dO, b = gpu_run(name)
    g = cfg.Hq // cfg.Hkv
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
    # ... and per element (kv head, channel).  Two terms.  (a) Rounding noise: every dV element
    # carries an independent bf16 rounding (uniform within half an ulp: standard deviation
    # 2^-9 |x| / sqrt 3 at most) and the probabilities its MFMAs consume are rounded the same way,
    # a random walk over the keys with standard deviation 2^-9 / sqrt 3 * sqrt(2 sum_j dV_jd^2);
    # six of them.  (b) fp32 round-off of sums over up to S * g products per element (the
    # normaliser of each row, the dV accumulators): measured, the whole-tensor deviation is
    # 2.4e-5 .. 1.0e-4 of the norm of the expected vector (S = 256K, g = 4 .. S = 1M, g = 8), so
    # a single element is granted 4e-4 of that vector's rms.  A dropped or doubled chunk pair
    # moves an element by about rms / u (>= 3e-2 rms).
    noise = (2.0 ** -9 / 3 ** 0.5) * (2.0 * dVd.pow(2).sum(dim=0)).sqrt()
    dev = (got - want).abs() / (6.0 * noise + 4e-4 * want.pow(2).mean().sqrt())
    print("sum-dV invariant: worst element uses", float(dev.max()), "of its bound", flush=True)
    assert dev.max() <= 1.0, "sum dV invariant, per element"
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
    for n in ("O", "LSE", "dQ", "dK", "dV"):
        assert torch.isfinite(getattr(b, n)).all(), n


# (workload, random rows, unconditional tail keys, random key rows per chunk); the three checks of
# a workload run back to back on one forward + backward
LARGE = [("gpt2p7b_64k", 48, 64, 8), ("llama8b_256k", 48, 32, 16), ("llama8b_256k_one_launch", 24, 16, 4),
         ("llama70b_1m", 24, 16, 3), ("llama8b_2m", 16, 8, 2)]
CASES = [(name, kind, n_random, tail, per_chunk) for name, n_random, tail, per_chunk in LARGE
         for kind in ("rows", "columns", "invariants")]


@pytest.mark.parametrize("name,kind,n_random,tail,per_chunk", CASES,
                         ids=["%s-%s" % (c[0], c[1]) for c in CASES])
def test_full_size(name, kind, n_random, tail, per_chunk):
    if kind == "rows":
        check_rows_and_tail(name, n_random, tail)
    elif kind == "columns":
        check_columns_conditional(name, per_chunk)
    else:
        check_invariants(name)


def test_release_cached_run():
    _RUN.clear()
    torch.cuda.empty_cache()


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
