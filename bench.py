#!/usr/bin/env python3
"""Benchmark of the chunked causal attention path (forward + backward) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config NAME] [--no-cpu-baseline]

A step is one pass of the whole hot path -- fpdt_attn_fwd then fpdt_attn_bwd -- over one
batch of seeded synthetic N(0,1) inputs of the named workload, inputs already resident (in
HBM, or in pinned host memory for the tensors the workload offloads).  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

T_START = time.perf_counter()
ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0  # MI355X dense bf16 MFMA peak

# Wall-clock budgets (seconds).  One pass of the default workload takes about half a minute, so
# the number of timed passes is min(--steps, what fits in TIMED_BUDGET_S), at least one; the
# whole run (import, input generation, warm-up, timed passes, link probe, oracle baseline) is
# meant to stay far inside a ten-minute limit.
TIMED_BUDGET_S = 105.0
WARMUP_BUDGET_S = 20.0


def hbm_traffic_per_launch(workload, kernel):
    """HBM bytes (read + written) per launch of `kernel`, from the tracked rocprofv3 --pmc summary
    of this workload (FETCH_SIZE and WRITE_SIZE runs, each scaled by what the same counter reads
    for the plain 1 GiB copy kernel of --calibrate-copy).  A profiler measurement, not a live one:
    None for a workload that has no such summary."""
    path = os.path.join(ROOT, "profiles", "attn_kernels_%s_hbm_traffic.txt" % workload)
    try:
        with open(path) as f:
            for line in f:
                if line.startswith("traffic_bytes_per_launch"):
                    for item in line.split()[1:]:
                        k, _, v = item.partition("=")
                        if k == kernel:
                            return float(v)
    except OSError:
        pass
    return None


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1)
    ap.add_argument("--warmup", type=int, default=0)
    ap.add_argument("--config", default="llama8b_2m")
    ap.add_argument("--chunk", type=int, default=0, help="override the workload's chunk size")
    ap.add_argument("--seq", type=int, default=0, help="override the workload's sequence length")
    ap.add_argument("--offload", choices=["none", "kv", "kv+act"], default=None,
                    help="override which tensors live in pinned host memory")
    ap.add_argument("--keep", type=float, default=None,
                    help="block-sparse attention (Sec. 5.5): keep each below-diagonal chunk pair "
                         "with this probability (seeded), always keep the diagonal")
    ap.add_argument("--bwd-order", choices=["kv", "q"], default=None,
                    help="backward chunk-pair loop order (Sec. 4.2); default: the library's choice")
    ap.add_argument("--bwd", choices=["stored-ds", "recompute"], default=None,
                    help="backward form (default: the workload's): stored-ds = FPDT_BWD_STORE_DS, dQ from "
                         "the dS tiles the dK/dV kernel writes (5 executed GEMMs per chunk pair, chunk^2 * Hq "
                         "* 2 bytes of workspace); recompute = dQ recomputes S and dP (7 GEMMs)")
    ap.add_argument("--time-budget", type=float, default=TIMED_BUDGET_S,
                    help="seconds of timed passes: fewer than --steps are timed if they do not fit "
                         "(never fewer than one)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-link-probe", action="store_true")
    ap.add_argument("--resident-compare", action="store_true",
                    help="also time the same pair schedule with K/V resident (exposed copy time)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device-to-device copy kernel (reference for "
                         "scaling the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    ap.add_argument("--calibrate-mfma", action="store_true",
                    help="run only the library's MFMA calibration loops (what this GPU sustains on the "
                         "kernels' MFMA instruction with random operands, alone, with the softmax's vector "
                         "instructions in between, and with operands freshly read from LDS) and print them")
    return ap.parse_args()


def link_probe(torch, nbytes):
    """Bare pinned-memory hipMemcpyAsync rate, GB/s, (h2d, d2h)."""
    host = torch.empty(nbytes, dtype=torch.uint8, pin_memory=True)
    dev = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    out = []
    for direction in ("h2d", "d2h"):
        best = 0.0
        for _ in range(3):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            if direction == "h2d":
                dev.copy_(host, non_blocking=True)
            else:
                host.copy_(dev, non_blocking=True)
            b.record()
            b.synchronize()
            best = max(best, nbytes / (a.elapsed_time(b) * 1e-3) / 1e9)
        out.append(best)
    return out


def cpu_baseline(torch, cfg, K, V, seed):
    """The fp64 oracle's row evaluator (forward + dQ side of the backward) on a bounded
    sample of the workload's own rows, timed on the host cores."""
    import numpy as np
    from oracle import definition
    from paper_2408_16978_amd import inputs
    limit = min(cfg.S, 262144)
    n_rows = 256  # about 15-20 s on 16 host cores
    rng = np.random.default_rng(1234)
    rows = np.sort(rng.integers(0, limit, size=n_rows))
    Kd = K[:limit].to(torch.float64).cpu().numpy()
    Vd = V[:limit].to(torch.float64).cpu().numpy()
    Qr = inputs.normal("Q", (n_rows, cfg.Hq, cfg.D), seed + 1, cfg.dtype).to(torch.float64).numpy()
    dOr = inputs.normal("dO", (n_rows, cfg.Hq, cfg.D), seed + 1, cfg.dtype).to(torch.float64).numpy()
    t0 = time.perf_counter()
    definition.rows(Qr, Kd, Vd, rows, cfg.scale, dOr=dOr)
    dt = time.perf_counter() - t0
    # scores, PV, dP, dQ: four length-(i+1) passes of 2*D flops per key, per head
    flops = float(sum(8.0 * cfg.D * (int(i) + 1) for i in rows)) * cfg.Hq
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": definition.threads(),
            "kind": "oracle",
            "sample": "row evaluator (O, LSE, Delta, dQ in fp64) on %d random query rows < %d of "
                      "the workload, all %d heads, %.1f s" % (n_rows, limit, cfg.Hq, dt)}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding or collectives); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2408_16978_amd import binding as B, inputs, runner

    if args.calibrate_mfma:
        torch.cuda.set_device(0)
        cal = {}
        for rep in range(2):  # the second pass is the one reported (clocks settled)
            for kind, name in enumerate(B.FPDT_CAL_KINDS):
                tf, ms = B.fpdt_calibrate_mfma(kind, 40000)
                cal[name] = {"tflops": tf, "frac_of_peak": tf / PEAK_BF16_TFLOPS, "ms": ms}
        print(json.dumps({"mfma_calibration": cal, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                          "note": "v_mfma_f32_32x32x16_bf16 on random operands of order one, one workgroup "
                                  "per compute unit; reg = register operands, lds1 = one LDS fragment per "
                                  "MFMA, lds2 = one per two MFMAs, softmax = 4 vector instructions per MFMA "
                                  "(fma, exp2, add, cvt_pk / max3), 1w / 2w = waves per SIMD"}))
        return
    cfg = inputs.CONFIGS[args.config]
    if args.chunk or args.seq or args.offload is not None:
        import dataclasses
        over = {}
        if args.chunk:
            over["chunk"] = args.chunk
        if args.seq:
            over["S"] = args.seq
        if args.offload is not None:
            over["kv_on_host"] = args.offload != "none"
            over["act_on_host"] = args.offload == "kv+act"
        cfg = dataclasses.replace(cfg, **over)
        cfg = dataclasses.replace(cfg, name="%s[S=%d,chunk=%d,offload=%s]" % (
            args.config, cfg.S, cfg.chunk,
            "kv+act" if cfg.act_on_host else "kv" if cfg.kv_on_host else "none"))
    torch.cuda.set_device(0)
    seed = 2024
    Q, K, V, dO = inputs.make_qkvdo(cfg.S, cfg.Hq, cfg.Hkv, cfg.D, cfg.dtype, seed, device="cuda")
    flags = (B.FPDT_KV_ON_HOST if cfg.kv_on_host else 0) | (B.FPDT_ACT_ON_HOST if cfg.act_on_host else 0)
    store_ds = cfg.store_ds if args.bwd is None else args.bwd == "stored-ds"
    if store_ds != cfg.store_ds:
        cfg = __import__("dataclasses").replace(cfg, store_ds=store_ds, name="%s[bwd=%s]" % (cfg.name, args.bwd))
    if store_ds:
        flags |= B.FPDT_BWD_STORE_DS
    if args.bwd_order is not None:
        flags |= B.FPDT_BWD_Q_OUTER if args.bwd_order == "q" else B.FPDT_BWD_KV_OUTER
        cfg = __import__("dataclasses").replace(cfg, name="%s[bwd=%s-outer]" % (cfg.name, args.bwd_order))
    mask = None
    pair_frac = 1.0  # kept share of the dense causal FLOPs
    if args.keep is not None:
        import numpy as np
        u = cfg.S // cfg.chunk
        mask = np.tril(np.random.default_rng(7).random((u, u)) < args.keep)
        np.fill_diagonal(mask, True)
        C = float(cfg.chunk)
        kept = (mask.sum() - u) * C * C + u * C * (C + 1) / 2
        pair_frac = kept / (cfg.S * (cfg.S + 1) / 2.0)
        cfg = __import__("dataclasses").replace(cfg, name="%s[keep=%g: %d of %d pairs]" % (
            cfg.name, args.keep, int(mask.sum()), u * (u + 1) // 2))
    bufs = runner.make_buffers(Q, K, V, dO, cfg.chunk, cfg.scale, flags, chunk_mask=mask)
    if cfg.kv_on_host:
        Kdev, Vdev = K, V
    del Q, dO
    torch.cuda.synchronize()

    # code-object load and first-launch costs are paid on a small problem of the same kernels
    if cfg.dtype == "bf16":
        w = inputs.make_qkvdo(1024, cfg.Hq, cfg.Hkv, cfg.D, "bf16", 1, device="cuda")
        wb = runner.make_buffers(*w, 256, cfg.scale, B.FPDT_PAIRWISE | (flags & B.FPDT_BWD_STORE_DS))
        runner.forward(wb)
        runner.backward(wb)
        torch.cuda.synchronize()
        del w, wb

    # Warm-up passes run the same kernels, chunk size, residency and copy pipeline on a PREFIX of
    # the workload (at most four chunks): a full pass of the default workload takes half a minute
    # and adds nothing that the prefix does not already warm (code objects, side streams, events,
    # pinned pages, clocks).  Workloads that take well under a second are warmed up in full.
    warm_S = cfg.S if cfg.S <= 262144 else 4 * cfg.chunk
    if warm_S == cfg.S:
        wbufs = bufs
    else:
        nc = warm_S // cfg.chunk
        dt = B.FPDT_DTYPE_BF16 if cfg.dtype == "bf16" else B.FPDT_DTYPE_F32
        fwd_flags = bufs.flags & ~(B.FPDT_BWD_KV_OUTER | B.FPDT_BWD_Q_OUTER | B.FPDT_BWD_STORE_DS)
        wbufs = runner.Buffers(
            Q=bufs.Q[:warm_S], K=bufs.K[:warm_S], V=bufs.V[:warm_S], dO=bufs.dO[:warm_S],
            O=bufs.O[:warm_S], dQ=bufs.dQ[:warm_S], dK=bufs.dK[:warm_S], dV=bufs.dV[:warm_S],
            LSE=torch.empty((cfg.Hq, warm_S), dtype=torch.float32, device=bufs.LSE.device,
                            pin_memory=bufs.LSE.is_pinned()),
            ws_fwd=B.alloc_workspace(warm_S, cfg.chunk, cfg.Hq, cfg.Hkv, cfg.D, dt, fwd_flags, False),
            ws_bwd=B.alloc_workspace(warm_S, cfg.chunk, cfg.Hq, cfg.Hkv, cfg.D, dt, bufs.flags, True),
            chunk=cfg.chunk, scale=cfg.scale, flags=bufs.flags,
            chunk_mask=mask[:nc, :nc].copy() if mask is not None else None)
    warm_done = 0
    tw = time.perf_counter()
    for _ in range(args.warmup):
        runner.forward(wbufs)
        runner.backward(wbufs)
        torch.cuda.synchronize()
        warm_done += 1
        if time.perf_counter() - tw > WARMUP_BUDGET_S:
            break
    if wbufs is not bufs:
        del wbufs
    torch.cuda.synchronize()

    B.fpdt_profile_enable(True)
    fwd_ms = bwd_ms = 0.0
    link = [0, 0]
    steps_done = 0
    t0 = time.perf_counter()
    while steps_done < args.steps:
        ta = time.perf_counter()
        runner.forward(bufs)
        torch.cuda.synchronize()
        tb = time.perf_counter()
        h, d = B.fpdt_last_link_bytes()
        link[0] += h
        link[1] += d
        runner.backward(bufs)
        torch.cuda.synchronize()
        tc = time.perf_counter()
        h, d = B.fpdt_last_link_bytes()
        link[0] += h
        link[1] += d
        fwd_ms += (tb - ta) * 1e3
        bwd_ms += (tc - tb) * 1e3
        steps_done += 1
        elapsed = tc - t0
        if elapsed + elapsed / steps_done > args.time_budget:  # the next pass would not fit
            break
    torch.cuda.synchronize()
    total_s = time.perf_counter() - t0
    B.fpdt_profile_enable(False)
    steps_requested, args.steps = args.steps, steps_done

    prof = {}
    for name, kind in (("fwd_sweep", B.FPDT_PROF_FWD), ("bwd_dkdv", B.FPDT_PROF_DKDV),
                       ("bwd_dq", B.FPDT_PROF_DQ), ("h2d", B.FPDT_PROF_H2D), ("d2h", B.FPDT_PROF_D2H)):
        ms, n = B.fpdt_profile_read(kind)
        prof[name] = {"total_ms": ms, "launches": n}

    ms_per_step = total_s * 1e3 / args.steps
    flops_step = cfg.flops_fwd_bwd() * pair_frac
    tflops = flops_step / (ms_per_step * 1e-3) / 1e12
    fwd_flops = cfg.flops_fwd() * pair_frac

    # dominant kernel: the one with the largest summed duration.  Algorithmic FLOPs of a
    # kernel = 2*D*Hq*S(S+1)/2 per GEMM it is defined by (forward 2, dK/dV 4, dQ 3, or 1 from stored dS).
    gemms = {"fwd_sweep": 2, "bwd_dkdv": 4, "bwd_dq": 1 if store_ds else 3}
    dom = max(gemms, key=lambda k: prof[k]["total_ms"])
    per_gemm = 2.0 * cfg.D * cfg.Hq * cfg.S * (cfg.S + 1) / 2.0 * pair_frac
    dom_flops = gemms[dom] * per_gemm * args.steps
    achieved = dom_flops / (prof[dom]["total_ms"] * 1e-3) / 1e12 if prof[dom]["total_ms"] > 0 else 0.0
    roofline = {"bound": "mfma", "kernel": dom, "achieved": achieved, "peak": PEAK_BF16_TFLOPS,
                "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS,
                "traffic": hbm_traffic_per_launch(cfg.name, dom),
                "avg_launch_ms": prof[dom]["total_ms"] / max(1, prof[dom]["launches"]),
                "launches": prof[dom]["launches"]}

    roofline_dq = None
    if store_ds and prof["bwd_dq"]["total_ms"] > 0:
        # the dQ kernel of the stored-dS backward reads every dS tile of the causal triangle once
        # (bf16, Hq heads): its algorithmic bytes; it is bound by HBM, not by the MFMA pipe
        ds_bytes = 2.0 * cfg.Hq * cfg.S * (cfg.S + 1) / 2.0 * pair_frac * args.steps
        gbps = ds_bytes / (prof["bwd_dq"]["total_ms"] * 1e-3) / 1e9
        roofline_dq = {"bound": "hbm", "kernel": "bwd_dq (from stored dS)", "achieved": gbps, "peak": 8000.0,
                       "unit": "GB/s", "frac": gbps / 8000.0,
                       "traffic": hbm_traffic_per_launch(cfg.name, "bwd_dq"),
                       "avg_launch_ms": prof["bwd_dq"]["total_ms"] / max(1, prof["bwd_dq"]["launches"]),
                       "launches": prof["bwd_dq"]["launches"]}

    out = {
        "metric": "chunked causal attn fwd+bwd TFLOPS",
        "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": warm_done,
        "steps_requested": steps_requested, "warmup_requested": args.warmup,
        "warmup_workload": "same kernels, chunk and residency on the first %d tokens" % warm_S,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": cfg.name, "S": cfg.S, "chunk": cfg.chunk, "Hq": cfg.Hq, "Hkv": cfg.Hkv,
                   "D": cfg.D, "kv_on_host": cfg.kv_on_host, "act_on_host": cfg.act_on_host,
                   "bwd": "stored-dS (5 executed GEMMs per chunk pair)" if store_ds else
                          "recompute (7 executed GEMMs per chunk pair)"},
        "frac_bf16_mfma_peak": tflops / PEAK_BF16_TFLOPS,
        "fwd_ms": fwd_ms / args.steps, "bwd_ms": bwd_ms / args.steps,
        "fwd_tflops": fwd_flops / (fwd_ms / args.steps * 1e-3) / 1e12,
        "bwd_tflops": 2.5 * fwd_flops / (bwd_ms / args.steps * 1e-3) / 1e12,
        "kernels": prof,
        "roofline": roofline,
    }
    if roofline_dq is not None:
        out["roofline_dq"] = roofline_dq
    if link[0] or link[1]:
        off = {"h2d_bytes_per_step": link[0] / args.steps, "d2h_bytes_per_step": link[1] / args.steps}
        if prof["h2d"]["total_ms"] > 0:
            off["h2d_GBps_while_busy"] = link[0] / (prof["h2d"]["total_ms"] * 1e-3) / 1e9
        if prof["d2h"]["total_ms"] > 0:
            off["d2h_GBps_while_busy"] = link[1] / (prof["d2h"]["total_ms"] * 1e-3) / 1e9
        off["h2d_GBps_needed"] = link[0] / total_s / 1e9
        out["offload"] = off
    if not args.no_link_probe:
        h64, d64 = link_probe(torch, 64 << 20)
        h1g, d1g = link_probe(torch, 1 << 30)
        out.setdefault("offload", {})["link_peak_GBps"] = {"h2d_64MiB": h64, "d2h_64MiB": d64,
                                                          "h2d_1GiB": h1g, "d2h_1GiB": d1g}
    if args.resident_compare and cfg.kv_on_host and not cfg.act_on_host:
        # same kernels, same pair order, K/V resident: the difference is the exposed copy time
        res_flags = B.FPDT_PAIRWISE | (flags & (B.FPDT_BWD_STORE_DS | B.FPDT_BWD_KV_OUTER | B.FPDT_BWD_Q_OUTER))
        del bufs.ws_bwd  # the resident run brings a backward workspace of its own
        b2 = runner.Buffers(Q=bufs.Q, K=Kdev, V=Vdev, dO=bufs.dO, O=bufs.O, LSE=bufs.LSE, dQ=bufs.dQ,
                            dK=torch.empty_like(Kdev), dV=torch.empty_like(Vdev),
                            ws_fwd=B.alloc_workspace(cfg.S, cfg.chunk, cfg.Hq, cfg.Hkv, cfg.D,
                                                     B.FPDT_DTYPE_BF16, B.FPDT_PAIRWISE, False),
                            ws_bwd=B.alloc_workspace(cfg.S, cfg.chunk, cfg.Hq, cfg.Hkv, cfg.D,
                                                     B.FPDT_DTYPE_BF16, res_flags, True),
                            chunk=cfg.chunk, scale=cfg.scale, flags=res_flags, chunk_mask=mask)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        runner.forward(b2)
        runner.backward(b2)
        torch.cuda.synchronize()
        res_ms = (time.perf_counter() - t1) * 1e3
        out["offload"]["resident_pairwise_ms"] = res_ms
        out["offload"]["exposed_copy_ms"] = ms_per_step - res_ms
    if args.calibrate_copy:
        a = torch.ones(1 << 28, dtype=torch.float32, device="cuda")  # 1 GiB
        b = torch.empty_like(a)
        torch.cuda.synchronize()
        torch.add(a, 0.0, out=b)  # one elementwise kernel: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del a, b
    if not args.no_cpu_baseline:
        src_k = Kdev if cfg.kv_on_host else bufs.K
        src_v = Vdev if cfg.kv_on_host else bufs.V
        out["cpu_baseline"] = cpu_baseline(torch, cfg, src_k, src_v, seed)
    out["wall_s"] = time.perf_counter() - T_START
    out["fits_in_driver_run"] = out["wall_s"] < 600.0
    print(json.dumps(out))


if __name__ == "__main__":
    main()
