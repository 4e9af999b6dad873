"""GPU parity: the HIP path (through the C ABI) against the fp64 oracle, element by element,
on seeded inputs that span several tiles, several chunks and the diagonal."""
import numpy as np
import pytest
import torch

from paper_2408_16978_amd import binding as B
from paper_2408_16978_amd import inputs, runner
from oracle import chunked

import parity

pytestmark = pytest.mark.gpu


def run(Q, K, V, dO, chunk, scale, flags=0):
    b = runner.make_buffers(Q, K, V, dO, chunk, scale, flags)
    runner.forward(b)
    runner.backward(b)
    torch.cuda.synchronize()
    return {"O": b.O, "LSE": b.LSE, "dQ": b.dQ, "dK": b.dK, "dV": b.dV}


def announce(*a):
    print("[case]", *a, flush=True)


def test_tiny_fp32_config():
    """Config 1: S=1024, 4 chunks of 256, 2 = 2 heads, D=64, fp32; all five outputs."""
    cfg = inputs.CONFIGS["tiny"]
    announce(cfg)
    Q, K, V, dO = inputs.make_qkvdo(cfg.S, cfg.Hq, cfg.Hkv, cfg.D, cfg.dtype, seed=1)
    ref = parity.oracle_full(Q, K, V, dO, cfg.scale)
    for flags in (0, B.FPDT_BWD_Q_OUTER):
        out = run(Q, K, V, dO, cfg.chunk, cfg.scale, flags)
        print(parity.check_all(out, ref, False))


@pytest.mark.parametrize("S,chunk,Hq,Hkv,D", [(300, 100, 4, 2, 80), (768, 256, 8, 1, 128),
                                              (130, 130, 2, 2, 64), (64, 1, 2, 1, 64)])
def test_fp32_ragged_shapes(S, chunk, Hq, Hkv, D):
    announce("fp32", S, chunk, Hq, Hkv, D)
    Q, K, V, dO = inputs.make_qkvdo(S, Hq, Hkv, D, "f32", seed=2)
    scale = D ** -0.5
    ref = parity.oracle_full(Q, K, V, dO, scale)
    out = run(Q, K, V, dO, chunk, scale)
    print(parity.check_all(out, ref, False))


SHAPES = [(2, 2, 64), (4, 4, 80), (8, 2, 128), (8, 1, 128)]


@pytest.mark.parametrize("Hq,Hkv,D", SHAPES)
def test_bf16_resident_full(Hq, Hkv, D):
    """Everything resident, the chunk pairs walked inside one launch per kernel."""
    S, chunk = 2048, 256
    announce("bf16 resident", S, chunk, Hq, Hkv, D)
    Q, K, V, dO = inputs.make_qkvdo(S, Hq, Hkv, D, "bf16", seed=3)
    scale = D ** -0.5
    ref = parity.oracle_full(Q, K, V, dO, scale)
    out = run(Q, K, V, dO, chunk, scale)
    print(parity.check_all(out, ref, True))


@pytest.mark.parametrize("Hq,Hkv,D", SHAPES)
@pytest.mark.parametrize("order", [B.FPDT_BWD_KV_OUTER, B.FPDT_BWD_Q_OUTER])
def test_bf16_pairwise_full(Hq, Hkv, D, order):
    """Pair-by-pair schedule with carried fp32 state, 8 chunks, both loop orders."""
    S, chunk = 2048, 256
    announce("bf16 pairwise", S, chunk, Hq, Hkv, D, order)
    Q, K, V, dO = inputs.make_qkvdo(S, Hq, Hkv, D, "bf16", seed=4)
    scale = D ** -0.5
    ref = parity.oracle_full(Q, K, V, dO, scale)
    out = run(Q, K, V, dO, chunk, scale, B.FPDT_PAIRWISE | order)
    print(parity.check_all(out, ref, True))


@pytest.mark.parametrize("Hq,Hkv,D", SHAPES)
@pytest.mark.parametrize("order", [B.FPDT_BWD_KV_OUTER, B.FPDT_BWD_Q_OUTER])
def test_bf16_stored_ds_backward(Hq, Hkv, D, order):
    """FPDT_BWD_STORE_DS: the dK/dV kernel writes its dS tiles and dQ is one GEMM over them.
    dK and dV must be the bits of the recomputing schedule (same kernel arithmetic, plus stores);
    dQ is checked against the oracle like any other dQ."""
    S, chunk = 2048, 256
    announce("bf16 stored dS", S, chunk, Hq, Hkv, D, order)
    Q, K, V, dO = inputs.make_qkvdo(S, Hq, Hkv, D, "bf16", seed=14)
    scale = D ** -0.5
    ref = parity.oracle_full(Q, K, V, dO, scale)
    base = run(Q, K, V, dO, chunk, scale, B.FPDT_PAIRWISE | order)
    out = run(Q, K, V, dO, chunk, scale, B.FPDT_BWD_STORE_DS | order)
    for n in ("O", "LSE", "dK", "dV"):
        assert torch.equal(out[n], base[n]), n
    print(parity.check_all(out, ref, True))


@pytest.mark.parametrize("S,chunk,Hq,Hkv,D,flags", [
    (768, 256, 4, 4, 128, 0), (1280, 1280, 8, 2, 128, 0), (2304, 768, 4, 4, 80, 0), (2304, 768, 2, 1, 64, 0),
    (4096, 512, 8, 2, 128, B.FPDT_KV_ON_HOST), (4096, 512, 8, 1, 128, B.FPDT_KV_ON_HOST | B.FPDT_ACT_ON_HOST)])
def test_bf16_stored_ds_odd_sizes_and_offload(S, chunk, Hq, Hkv, D, flags):
    """Stored-dS backward at odd multiples of the tile size, as a single chunk, and under the
    offload pipelines (K/V on the host in the paper's loop order; everything on the host, Q-outer)."""
    announce("bf16 stored dS", S, chunk, Hq, Hkv, D, flags)
    Q, K, V, dO = inputs.make_qkvdo(S, Hq, Hkv, D, "bf16", seed=15)
    scale = D ** -0.5
    ref = parity.oracle_full(Q, K, V, dO, scale)
    out = run(Q, K, V, dO, chunk, scale, flags | B.FPDT_BWD_STORE_DS)
    print(parity.check_all(out, ref, True))


@pytest.mark.parametrize("S,chunk", [(768, 256), (1280, 1280), (2304, 768)])
@pytest.mark.parametrize("Hq,Hkv,D", [(4, 4, 128), (8, 2, 128), (4, 4, 80), (2, 1, 64)])
def test_bf16_odd_tile_counts_and_ungrouped_heads(S, chunk, Hq, Hkv, D):
    """Chunk and sequence lengths that are odd multiples of the 256-row tile (odd numbers of
    steps in every kernel's unrolled loops, a single chunk, three chunks), and one query head
    per KV head at D = 128; resident and pair-by-pair in both loop orders."""
    announce("bf16 odd sizes", S, chunk, Hq, Hkv, D)
    Q, K, V, dO = inputs.make_qkvdo(S, Hq, Hkv, D, "bf16", seed=8)
    scale = D ** -0.5
    ref = parity.oracle_full(Q, K, V, dO, scale)
    for flags in (0, B.FPDT_PAIRWISE | B.FPDT_BWD_KV_OUTER, B.FPDT_PAIRWISE | B.FPDT_BWD_Q_OUTER):
        out = run(Q, K, V, dO, chunk, scale, flags)
        print(parity.check_all(out, ref, True))


@pytest.mark.parametrize("kind", ["rising", "offset", "peaked"])
@pytest.mark.parametrize("Hq,Hkv,D", [(4, 4, 80), (8, 2, 128)])
def test_bf16_score_distributions_beyond_gaussian(kind, Hq, Hkv, D):
    """Running maxima that rise in every tile, scores with a large common offset, and peaked
    rows, in the one-launch and in the pair-by-pair schedule.  O, LSE and dV meet the plain bf16
    budget.  With such scores dS = p (dP - Delta) cancels almost completely, and the roundings the
    method itself prescribes (the stored bf16 O inside Delta, Sec. 3.1; dS rounded to bf16 for its
    MFMAs) then weigh more in dQ and dK than the plain budget allows, whatever the kernel does:
    their budget adds six standard deviations of that rounding noise (parity.backward_noise)."""
    S, chunk = 2048, 256
    announce("bf16", kind, S, chunk, Hq, Hkv, D)
    Q, K, V, dO = inputs.structured(kind, S, Hq, Hkv, D, "bf16", seed=6)
    scale = D ** -0.5
    ref = parity.oracle_full(Q, K, V, dO, scale)
    sigma = parity.backward_noise(Q, K, V, dO, ref, scale)
    for flags in (0, B.FPDT_PAIRWISE | B.FPDT_BWD_KV_OUTER):
        out = run(Q, K, V, dO, chunk, scale, flags)
        print(parity.check_all(out, ref, True, names=("O", "LSE", "dV")))
        for n in ("dQ", "dK"):
            parity.check_with_noise(n, out[n], ref[n], sigma[n], label=kind)


@pytest.mark.parametrize("flags", [B.FPDT_KV_ON_HOST | B.FPDT_BWD_KV_OUTER,
                                   B.FPDT_KV_ON_HOST | B.FPDT_BWD_Q_OUTER,
                                   B.FPDT_KV_ON_HOST | B.FPDT_ACT_ON_HOST])
def test_offload_is_bitwise_equal_to_pairwise(flags):
    """Same kernels in the same order: only the copies and events differ, so any difference
    is a pipeline bug (a missing wait shows as stale or poisoned data)."""
    S, chunk, Hq, Hkv, D = 4096, 512, 8, 2, 128
    announce("offload", S, chunk, flags)
    Q, K, V, dO = inputs.make_qkvdo(S, Hq, Hkv, D, "bf16", seed=5)
    scale = D ** -0.5
    order = B.FPDT_BWD_Q_OUTER if (flags & (B.FPDT_BWD_Q_OUTER | B.FPDT_ACT_ON_HOST)) else B.FPDT_BWD_KV_OUTER
    base = run(Q, K, V, dO, chunk, scale, B.FPDT_PAIRWISE | order)
    out = run(Q, K, V, dO, chunk, scale, flags)
    for n in ("O", "LSE", "dQ", "dK", "dV"):
        assert torch.equal(out[n].cpu(), base[n].cpu()), n
    h2d, d2h = B.fpdt_last_link_bytes()
    assert h2d > 0 and d2h > 0
    ref = parity.oracle_full(Q, K, V, dO, scale)
    print(parity.check_all(out, ref, True))


@pytest.mark.parametrize("flags", [B.FPDT_KV_ON_HOST | B.FPDT_BWD_KV_OUTER,
                                   B.FPDT_KV_ON_HOST | B.FPDT_BWD_Q_OUTER,
                                   B.FPDT_KV_ON_HOST | B.FPDT_ACT_ON_HOST])
def test_offload_event_ordering_with_poisoned_buffers_and_delayed_copies(flags):
    """Every staging buffer is filled with NaNs right before the copy into it and every copy is
    held back by a 48 MiB dummy copy on its stream: a kernel that does not wait for its data, or
    a copy / kernel that does not wait for a buffer to be released, changes the result."""
    S, chunk, Hq, Hkv, D = 4096, 512, 8, 2, 128
    announce("offload under poison + delay", S, chunk, flags)
    Q, K, V, dO = inputs.make_qkvdo(S, Hq, Hkv, D, "bf16", seed=6)
    scale = D ** -0.5
    order = B.FPDT_BWD_Q_OUTER if (flags & (B.FPDT_BWD_Q_OUTER | B.FPDT_ACT_ON_HOST)) else B.FPDT_BWD_KV_OUTER
    base = run(Q, K, V, dO, chunk, scale, B.FPDT_PAIRWISE | order)
    B.fpdt_debug_configure(B.FPDT_DEBUG_POISON_STAGING | B.FPDT_DEBUG_DELAY_COPIES)
    try:
        out = run(Q, K, V, dO, chunk, scale, flags)
    finally:
        B.fpdt_debug_configure(0)
    for n in ("O", "LSE", "dQ", "dK", "dV"):
        assert torch.isfinite(out[n].float()).all(), n
        assert torch.equal(out[n].cpu(), base[n].cpu()), n
    with pytest.raises(B.FpdtError):
        B.fpdt_debug_configure(1 << 7)


@pytest.mark.parametrize("S,Hq,Hkv,D,flags,forced", [(6144, 8, 2, 128, B.FPDT_KV_ON_HOST, 1536),
                                                      (4096, 4, 4, 80, 0, None)])
def test_picked_chunk_runs_to_parity(S, Hq, Hkv, D, flags, forced):
    """fpdt_attn_pick_chunk (Sec. 5.3) returns a chunk the entry points accept, within the
    workspace limit it was given, and forward + backward at that chunk match the oracle: once
    with a limit that forces a small chunk of a sequence that is not a power of two (K/V
    offloaded), once without a limit (the whole short sequence is one chunk)."""
    BF = B.FPDT_DTYPE_BF16
    limit = 0
    if forced:
        limit = max(B.fpdt_attn_workspace_bytes(S, forced, Hq, Hkv, D, BF, flags, b) for b in (False, True))
    chunk = B.fpdt_attn_pick_chunk(S, Hq, Hkv, D, BF, flags, limit)
    announce("picked chunk", S, Hq, Hkv, D, flags, limit, "->", chunk)
    assert chunk == (forced or S)
    Q, K, V, dO = inputs.make_qkvdo(S, Hq, Hkv, D, "bf16", seed=12)
    scale = D ** -0.5
    ref = parity.oracle_full(Q, K, V, dO, scale)
    out = run(Q, K, V, dO, chunk, scale, flags)
    print(parity.check_all(out, ref, True))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_merge_kernel(dtype):
    rows, Hq, D = 1000, 4, 80
    announce("merge", dtype)
    g = torch.Generator().manual_seed(6)
    td = inputs.torch_dtype(dtype)
    Oa = torch.randn(rows, Hq, D, generator=g).to(td)
    Ob = torch.randn(rows, Hq, D, generator=g).to(td)
    La = torch.randn(Hq, rows, generator=g) * 3
    Lb = torch.randn(Hq, rows, generator=g) * 3
    La[0, :10] = float("-inf")          # partial that saw no keys
    want_o = np.empty((rows, Hq, D))
    want_l = np.empty((Hq, rows))
    for h in range(Hq):
        with np.errstate(invalid="ignore"):
            o, l = chunked.merge(parity.to64(Oa)[:, h], La[h].double().numpy(),
                                 parity.to64(Ob)[:, h], Lb[h].double().numpy())
        want_o[:, h], want_l[h] = o, l
    want_o[:10, 0] = parity.to64(Ob)[:10, 0]
    dev = [t.cuda() for t in (Oa, La, Ob, Lb)]
    Oo = torch.empty_like(dev[0])
    Lo = torch.empty_like(dev[1])
    B.fpdt_attn_merge(dev[0], dev[1], dev[2], dev[3], Oo, Lo)
    torch.cuda.synchronize()
    tol = 1e-5 if dtype == "f32" else 2e-2
    assert np.abs(parity.to64(Oo) - want_o).max() <= tol
    assert np.abs(Lo.cpu().double().numpy() - want_l).max() <= 1e-5


def test_invalid_pointers_are_rejected_on_gpu():
    """Host pointer where device memory is expected, short workspace: error codes, no launch."""
    S, chunk, Hq, Hkv, D = 512, 256, 2, 2, 64
    Q, K, V, dO = inputs.make_qkvdo(S, Hq, Hkv, D, "bf16", seed=7)
    b = runner.make_buffers(Q, K, V, dO, chunk, D ** -0.5)
    with pytest.raises(B.FpdtError) as e:
        B.fpdt_attn_fwd(b.Q, K, b.V, b.O, b.LSE, chunk, D ** -0.5, 0, b.ws_fwd)   # K on pageable host
    assert e.value.status == B.FPDT_ERR_INVALID_ARG
    with pytest.raises(B.FpdtError) as e:
        B.fpdt_attn_fwd(b.Q, b.K, b.V, b.O, b.LSE, chunk, D ** -0.5, 0, b.ws_fwd[:1024])
    assert e.value.status == B.FPDT_ERR_WORKSPACE
    with pytest.raises(B.FpdtError) as e:   # device K where pinned host memory is required
        B.fpdt_attn_fwd(b.Q, b.K, b.V, b.O, b.LSE, chunk, D ** -0.5, B.FPDT_KV_ON_HOST,
                        B.alloc_workspace(S, chunk, Hq, Hkv, D, B.FPDT_DTYPE_BF16, B.FPDT_KV_ON_HOST))
    assert e.value.status == B.FPDT_ERR_INVALID_ARG


def test_calibration_loops_report_plausible_rates():
    """fpdt_calibrate_mfma: every loop runs, inside the range a 2.5 PFLOP/s part can deliver, and
    the loops that add LDS-fed operands and the softmax's vector work to the MFMAs are slower
    than the MFMAs alone (the clock wanders by several percent from launch to launch, so nothing
    finer than that is asserted)."""
    B.fpdt_calibrate_mfma(0, 8000)  # clocks up
    rates = [B.fpdt_calibrate_mfma(kind, 8000)[0] for kind in range(len(B.FPDT_CAL_KINDS))]
    announce("calibration", dict(zip(B.FPDT_CAL_KINDS, (round(r) for r in rates))))
    assert all(300.0 < r < 2600.0 for r in rates)
    assert max(rates[6], rates[7]) < 0.95 * max(rates[0], rates[1])


@pytest.mark.parametrize("flags", [0, B.FPDT_BWD_STORE_DS, B.FPDT_KV_ON_HOST | B.FPDT_BWD_STORE_DS])
def test_results_are_reproducible_bit_for_bit(flags):
    """No atomics and no order that depends on timing anywhere on the path: two runs of the same
    problem (buffers allocated afresh, so at other addresses) give the same bits."""
    S, chunk, Hq, Hkv, D = 4096, 1024, 8, 2, 128
    announce("reproducibility", S, chunk, flags)
    Q, K, V, dO = inputs.make_qkvdo(S, Hq, Hkv, D, "bf16", seed=16)
    first = {n: t.clone() for n, t in run(Q, K, V, dO, chunk, D ** -0.5, flags).items()}
    pad = torch.empty(3 << 20, dtype=torch.uint8, device="cuda")  # shifts the next allocations
    second = run(Q, K, V, dO, chunk, D ** -0.5, flags)
    for n in ("O", "LSE", "dQ", "dK", "dV"):
        assert torch.equal(first[n].cpu(), second[n].cpu()), n
    del pad
