#!/usr/bin/env python3
"""Benchmark of the sufficient-factor hot path on one MI355X.

A "step" is one pass of the whole path over one synthetic batch: SF compute
(forward contraction + softmax/label step) followed by reconstruction and
application of the summed rank-1 updates.  Default workload: the headline one,
multiclass logistic regression with J=325,000 classes, D=10,000 features,
B=1024, bf16 inputs, fp32 W and accumulation.  Inputs are resident in HBM before
the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# Published MI355X peaks used for the roofline fractions.
PEAK_HBM_GBS = 8000.0
PEAK_BF16_TFLOPS = 2500.0
PEAK_F32_TFLOPS = 157.3


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def kernel_sources_sha256():
    """Hash of the HIP sources the library is built from: the stamp that ties a counter profile to the kernels."""
    import hashlib
    csrc = os.path.join(ROOT, "paper_1409_5705_amd", "csrc")
    h = hashlib.sha256()
    for name in sorted(os.listdir(csrc)):
        if name.endswith((".hip", ".h", ".cpp")) and name != "peaks.hip":
            h.update(name.encode())
            h.update(open(os.path.join(csrc, name), "rb").read())
    return h.hexdigest()


def profile_traffic_bytes(profile="mlr_large_bf16_rocprofv3.md"):
    """Scaled FETCH_SIZE + WRITE_SIZE per launch, by kernel, from the committed rocprofv3 summary, and whether
    that summary was taken on the kernels of this tree (its `kernel_sources_sha256` line against the sources'
    hash): counters of other kernels are not quoted."""
    path = os.path.join(ROOT, "profiles", profile)
    out, stamp = {}, None
    try:
        for line in open(path):
            if line.startswith("traffic_bytes "):      # "traffic_bytes <kernel> <bytes>"
                _, name, val = line.split()
                out[name] = float(val)
            elif line.startswith("kernel_sources_sha256 "):
                stamp = line.split()[1]
    except OSError:
        pass
    current = stamp is not None and stamp == kernel_sources_sha256()
    return (out if current else {}), current


def cpu_baseline_mlr(cfg, X, y, W_rows):
    """The oracle, as it stands, on a bounded sample of the workload: the first Js classes of the
    benchmark's own W (softmax over those), all B samples, full D: SF compute + apply.  Scaled to the
    metric's unit by Js/J (both stages are linear in the number of classes)."""
    import numpy as np
    import oracle
    J, D, B = cfg["J"], cfg["D"], cfg["B"]
    Ws = W_rows
    Js = Ws.shape[0]
    ys = (y % Js).astype(np.int32)
    t0 = time.perf_counter()
    U, V = oracle.mlr_sf(Ws, X, ys)
    t1 = time.perf_counter()
    oracle.apply(Ws, U, V, cfg["eta"])
    t2 = time.perf_counter()
    dt = t2 - t0
    return {
        "value": (B / dt) * (Js / J),
        "unit": "updates/s",
        "cores": oracle.num_threads(),
        "kind": "oracle",
        "sample": "first %d of %d rows of the benchmark's W (softmax over those classes), all %d samples, D=%d; one step = SF compute "
                  "(%.1f s) + apply (%.1f s); rate scaled by %d/%d" % (Js, J, B, D, t1 - t0, t2 - t1, Js, J),
    }


def bench_fp32_workload(args):
    """Secondary bench lines: the fp32 parity configurations (MLR small, MLR with 7 peers' SF
    blocks, DML, sparse coding), one JSON line each.  A step is the whole path of that model."""
    import numpy as np
    import torch
    import oracle
    import sfb_synth as S
    import paper_1409_5705_amd as sfb

    name = args.workload
    cfg = S.CONFIGS[name]
    dev = torch.device("cuda", 0)
    ctx = sfb.Context(0)
    d = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    model = cfg["model"]
    if model == "mlr":
        J, D, B, eta = cfg["J"], cfg["D"], cfg["B"], cfg["eta"]
        P = cfg.get("peers", 0)
        N = B * (P + 1)
        W0 = S.normal_matrix(J, D, cfg["sigma"], seed=0)
        X, y = S.mlr_batch(J, D, B, seed=0, step=0)
        W, Xd, yd = d(W0), d(X), d(y)
        U = torch.empty((N, J), dtype=torch.float32, device=dev)
        V = torch.empty((N, D), dtype=torch.float32, device=dev)
        peers = [S.mlr_peer_sf(J, D, B, seed=0, step=0, peer=q) for q in range(P)]
        for q, (Uq, Vq) in enumerate(peers):
            U[B * (q + 1):B * (q + 2)] = d(Uq)
            V[B * (q + 1):B * (q + 2)] = d(Vq)

        def step():
            ctx.sfb_compute_sf(sfb.SFB_MLR, W, Xd, Y=yd, U=U[:B], V=V[:B])
            ctx.sfb_apply(W, U, V, eta)

        def oracle_step():
            Uo, Vo = oracle.mlr_sf(W0, X, y)
            oracle.apply(W0, np.concatenate([Uo] + [u for u, _ in peers]), np.concatenate([Vo] + [v for _, v in peers]), eta)
        flops = 2.0 * B * J * D + 2.0 * N * J * D
        desc = "%s: MLR fp32 J=%d D=%d local B=%d, N=%d rank-1 terms applied per step" % (name, J, D, B, N)
    elif model == "sdca":
        from oracle import sdca as osdca
        J, D, B, lam, Ntot, beta = cfg["J"], cfg["D"], cfg["B"], cfg["lam"], cfg["n_total"], cfg["beta"]
        P = cfg["peers"]
        N = B * (P + 1)
        W0 = S.normal_matrix(J, D, cfg["sigma"], seed=0)
        Z0 = (W0 * np.float32(lam)).astype(np.float32)
        X, y = S.mlr_batch(J, D, B, seed=0, step=0)
        P0 = S.sdca_dual_points(J, y, seed=0)
        W, Z, Xd = d(W0), d(Z0), d(X)
        Pd0 = d(P0)
        Pd = Pd0.clone()
        U = torch.empty((N, J), dtype=torch.float32, device=dev)
        V = torch.empty((N, D), dtype=torch.float32, device=dev)
        V[:B] = Xd
        # peers' factor blocks: dual steps have the statistics of MLR factors (rows summing to zero), scaled by beta
        peers = [S.mlr_peer_sf(J, D, B, seed=0, step=0, peer=q) for q in range(P)]
        for q, (Uq, Vq) in enumerate(peers):
            U[B * (q + 1):B * (q + 2)] = d(Uq) * beta
            V[B * (q + 1):B * (q + 2)] = d(Vq)

        def step():
            Pd.copy_(Pd0)                                     # every timed step starts from the same dual points
            ctx.sfb_sdca_mlr_sf(W, Xd, Pd, lam, Ntot, beta, U[:B])
            ctx.sfb_apply(Z, U, V, 1.0 / Ntot)
            ctx.sfb_dual_to_primal_l2(Z, W, lam)

        def oracle_step():
            dUo, _ = osdca.sdca_mlr_sf(W0, P0, X, lam, Ntot, beta)
            Zn = oracle.apply(Z0, np.concatenate([dUo] + [u * beta for u, _ in peers]),
                              np.concatenate([X] + [v for _, v in peers]), 1.0 / Ntot)
            osdca.dual_to_primal_l2(Zn, lam)
        flops = 2.0 * B * J * D + 2.0 * N * J * D
        desc = "%s: SDCA on l2-regularised MLR fp32 J=%d D=%d local B=%d, N=%d factor pairs applied to Z per step, W = Z/lambda" % (
            name, J, D, B, N)
    elif model == "dml":
        J, D, B, eta = cfg["K"], cfg["D"], cfg["B"], cfg["eta"]
        N = B
        W0 = S.normal_matrix(J, D, cfg["sigma"], seed=0)
        X, Y, sim = S.dml_batch(D, B, seed=0)
        W, Xd, Yd, simd = d(W0), d(X), d(Y), d(sim)
        U = torch.empty((B, J), dtype=torch.float32, device=dev)
        V = torch.empty((B, D), dtype=torch.float32, device=dev)
        na = torch.zeros((1,), dtype=torch.int32, device=dev)

        def step():
            ctx.sfb_compute_sf(sfb.SFB_DML, W, Xd, Y=Yd, sim=simd, U=U, V=V, n_active=na, margin=cfg["margin"])
            ctx.sfb_apply(W, U, V, eta)

        def oracle_step():
            Uo, Vo, _ = oracle.dml_sf(W0, X, Y, sim, margin=cfg["margin"])
            oracle.apply(W0, Uo, Vo, eta)
        flops = 4.0 * B * J * D
        desc = "%s: DML fp32 K=%d D=%d B=N=%d pairs (as stated: every hinge term inactive at this init)" % (name, J, D, B)
    else:
        J, D, B, eta = cfg["J"], cfg["D"], cfg["B"], cfg["eta"]
        N = B
        W0 = S.sc_dictionary(J, D, seed=0)
        X = S.sc_batch(D, B, seed=0)
        W, Xd = d(W0), d(X)
        U = torch.empty((B, J), dtype=torch.float32, device=dev)
        V = torch.empty((B, D), dtype=torch.float32, device=dev)

        def step():
            ctx.sfb_compute_sf(sfb.SFB_SC, W, Xd, U=U, V=V, lam=cfg["lam"], ista_iters=cfg["ista_iters"],
                               power_iters=cfg["power_iters"])
            ctx.sfb_apply(W, U, V, -eta)
            ctx.sfb_prox_rows(W, sfb.SFB_PROX_NORMALIZE)

        def oracle_step():
            Uo, Vo, _ = oracle.sc_sf(W0, X, cfg["lam"], cfg["ista_iters"], cfg["power_iters"])
            Wn = oracle.apply(W0, Uo, Vo, -eta)
            oracle.prox_rows(Wn, oracle.PROX_NORMALIZE)
        flops = (2 * cfg["ista_iters"] + 1) * 2.0 * B * J * D + 2.0 * B * J * D + cfg["power_iters"] * 4.0 * J * D
        desc = "%s: sparse coding fp32 J=%d D=%d B=N=%d, %d ISTA + %d power iterations, apply, prox" % (
            name, J, D, B, cfg["ista_iters"], cfg["power_iters"])

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ctx.sfb_profile_enable(True)
    ctx.sfb_profile_collect()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    prof = ctx.sfb_profile_collect()
    ctx.sfb_profile_enable(False)
    ms = (t1 - t0) * 1e3 / args.steps
    kernel_ms = {k: v[1] / args.steps for k, v in prof.items()}       # per step, all launches of a group
    gpu_ms = sum(kernel_ms.values())
    out = {
        "metric": "rank-1 SF updates applied/sec (SF compute + reconstruct/apply)",
        "value": N / (ms * 1e-3), "unit": "updates/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic", "config": {"workload": desc},
        "kernel_ms_per_step": kernel_ms, "gpu_busy_ms_per_step": gpu_ms,
        "roofline": {"kernel": "all fp32 MFMA contractions of a step", "bound": "mfma",
                     "achieved": flops / (gpu_ms * 1e-3) / 1e12, "peak": PEAK_F32_TFLOPS, "unit": "TFLOP/s",
                     "frac": flops / (gpu_ms * 1e-3) / 1e12 / PEAK_F32_TFLOPS, "traffic": None},
    }
    if args.measured_peaks is not None:
        out["measured_peaks"] = args.measured_peaks
    if args.graph:
        # the same step captured once into a HIP graph and replayed: removes the launch gaps of the
        # ~90 dependent kernels of a sparse-coding step (profiling events are off during capture)
        side = torch.cuda.Stream()
        with torch.cuda.stream(side):
            gctx = sfb.Context(0)
            ctx_eager = ctx
            ctx = gctx                      # step() resolves `ctx` at call time
            step()
            side.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                step()
        for _ in range(args.warmup):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        out["ms_per_step_graph_replay"] = (time.perf_counter() - t0) * 1e3 / args.steps
        ctx = ctx_eager
    if not args.no_cpu_baseline:
        t0 = time.perf_counter()
        oracle_step()
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": N / dt, "unit": "updates/s", "cores": oracle.num_threads(), "kind": "oracle",
                               "sample": "one whole step of this workload (%.2f s)" % dt}
    print(json.dumps(out), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="mlr_large_bf16")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB elementwise copy kernel (reference for HBM byte counters)")
    ap.add_argument("--layout", choices=["split", "fp32"], default="split",
                    help="mlr_large_bf16: how the library keeps W between steps: 'split' = the two 16-bit planes of "
                         "sfb_split_attach (same bits, no separate working copy), 'fp32' = the fp32 array plus a bf16 "
                         "working copy (sfb_shadow_attach)")
    ap.add_argument("--no-shadow", action="store_true",
                    help="do not attach a bf16 working copy of W (the forward then converts W on every call)")
    ap.add_argument("--graph", action="store_true",
                    help="fp32 workloads: also time the step replayed from a captured HIP graph")
    ap.add_argument("--peaks", action="store_true",
                    help="first run the stand-alone MFMA-only / HBM-streaming probe (paper_1409_5705_amd/sfb_peaks) "
                         "and report what this GPU sustains next to the published peaks")
    ap.add_argument("--no-other-layout", action="store_true",
                    help="mlr_large_bf16: skip the few extra steps in the fp32 + working-copy layout that are reported "
                         "beside the headline (ms_per_step_fp32_layout)")
    ap.add_argument("--zero-frac", type=float, default=None,
                    help="mlr_large_bf16: fraction of feature entries that are zero (default: the workload's 0.9); with "
                         "--csr, 0.995 is the tf-idf-like density at which sfb_mlr_sf_csr goes over the stored entries")
    ap.add_argument("--peers", type=int, default=0,
                    help="headline workload: also time sfb_apply on the local SF block plus this many peers' blocks "
                         "(N = (peers + 1) * B rows in one call: one GPU's share of a broadcast step); reported as "
                         "`apply_with_peers`, beside the headline, never as `value`")
    ap.add_argument("--csr", action="store_true",
                    help="mlr_large_bf16: hand the samples over as CSR rows (sfb_mlr_sf_csr / sfb_apply_csr)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (each GPU box has one GPU); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    measured_peaks = None
    if args.peaks:      # a child process, started before this one touches the GPU
        import subprocess
        exe = os.path.join(os.path.dirname(os.path.abspath(__file__)), "paper_1409_5705_amd", "sfb_peaks")
        if not os.path.exists(exe):
            print("bench: %s is not built (run __graft_entry__.build())" % exe, file=sys.stderr)
            sys.exit(2)
        r = subprocess.run([exe], capture_output=True, text=True, timeout=300)
        if r.returncode != 0:
            print("bench: sfb_peaks failed:\n" + r.stderr, file=sys.stderr)
            sys.exit(2)
        measured_peaks = json.loads(r.stdout.strip().splitlines()[-1])
        log("bench: measured peaks " + json.dumps(measured_peaks))
    args.measured_peaks = measured_peaks

    import numpy as np
    import torch
    import sfb_synth as S
    import paper_1409_5705_amd as sfb

    if args.workload in ("mlr_small", "mlr_peers", "dml", "sc", "sdca_peers"):
        bench_fp32_workload(args)
        return
    if args.workload != "mlr_large_bf16":
        print("unknown workload %r" % args.workload, file=sys.stderr)
        sys.exit(2)
    cfg = S.CONFIGS[args.workload]
    J, D, B, eta = cfg["J"], cfg["D"], cfg["B"], cfg["eta"]
    zero_frac = cfg["zero_frac"] if args.zero_frac is None else args.zero_frac
    dev = torch.device("cuda", 0)
    sfb.lib()

    log("bench: generating inputs (W %.1f GB on device)" % (J * D * 4 / 1e9))
    gen = torch.Generator(device=dev)
    gen.manual_seed(0)
    W = torch.randn((J, D), dtype=torch.float32, device=dev, generator=gen) * cfg["sigma"]
    n_batches = args.steps + args.warmup
    Xs, ys, X0, y0, nnzs = [], [], None, None, []
    for s in range(min(n_batches, 4)):                     # a few distinct batches, cycled
        X, y = S.mlr_batch(J, D, B, seed=0, step=s, zero_frac=zero_frac, bf16=True)
        if s == 0:
            X0, y0 = X, y
        nnzs.append(int(np.count_nonzero(X)))
        if args.csr:
            ip, ix, v = S.csr_from_dense(X)
            Xs.append((torch.from_numpy(ip).to(dev), torch.from_numpy(ix).to(dev),
                       torch.from_numpy(S.bf16_bits(v)).to(dev).view(torch.bfloat16)))
        else:
            Xs.append(torch.from_numpy(S.bf16_bits(X)).to(dev).view(torch.bfloat16))
        ys.append(torch.from_numpy(y).to(dev))
    nnz_mean = float(sum(nnzs)) / (len(nnzs) * B)
    U = torch.empty((B, J), dtype=torch.bfloat16, device=dev)
    ctx = sfb.Context(0)
    split = args.layout == "split" and not args.no_shadow
    if split:
        ctx.sfb_split_attach(W)      # W as two 16-bit planes (setup, like W itself): the planes are the parameters
    elif not args.no_shadow:
        ctx.sfb_shadow_attach(W)     # bf16 working copy of W, kept current by sfb_apply (setup, like W itself)

    def step(i):
        Xd, yd = Xs[i % len(Xs)], ys[i % len(ys)]
        if args.csr:
            ctx.sfb_mlr_sf_csr(W, Xd[0], Xd[1], Xd[2], yd, U)
            ctx.sfb_apply_csr(W, U, Xd[0], Xd[1], Xd[2], eta)
            return
        ctx.sfb_compute_sf(sfb.SFB_MLR, W, Xd, Y=yd, U=U)   # V = X
        ctx.sfb_apply(W, U, Xd, eta)

    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)     # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        torch.mul(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst
    log("bench: warmup")
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    ctx.sfb_profile_enable(True)
    ctx.sfb_profile_collect()
    torch.cuda.synchronize()
    log("bench: timing %d steps" % args.steps)
    # (one event per step boundary, recorded on the stream the library launches on: per-step durations)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    t0 = time.perf_counter()
    marks[0].record(ctx.stream)
    for i in range(args.steps):
        step(args.warmup + i)
        marks[i + 1].record(ctx.stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))
    prof = ctx.sfb_profile_collect()
    ctx.sfb_profile_enable(False)
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    if split:
        ctx.sfb_split_export(W)      # (outside the timed region: the fp32 array is only a snapshot in this layout)
        torch.cuda.synchronize()
    # The apply rewrites the bf16 image of W (high plane / working copy) four columns at a time and only where
    # its bits change.  Share of such groups in one more, untimed step, on a sample of rows: it sets the bytes
    # that step has to write.
    rows = slice(0, min(J, 4096))

    def bf16_image(Wrows):
        bits = Wrows.contiguous().view(torch.int32).to(torch.int64)
        return ((bits + 0x8000) >> 16) if split else Wrows.bfloat16().view(torch.int16).to(torch.int64)

    image_before = bf16_image(W[rows])
    step(args.warmup + args.steps)
    if split:
        ctx.sfb_split_export(W)
    torch.cuda.synchronize()
    rewritten = float((bf16_image(W[rows]) != image_before).view(-1, D // 4, 4).any(dim=2).float().mean()) \
        if not args.no_shadow else 0.0
    del image_before
    assert bool(torch.isfinite(W[:1024]).all())

    # per-kernel averages from the HIP events recorded on the library's stream
    kt = {k: v[1] / v[0] for k, v in prof.items()}          # ms per launch
    if "shadow_convert" in kt:                                # no working copy attached: conversion is part of forward
        kt["mlr_forward_bf16"] += kt["shadow_convert"]
    gather_ms = kt.get("csr_forward_gather")                 # CSR samples sparse enough for the route over stored entries
    fwd_ms = kt.get("mlr_forward_bf16", gather_ms if gather_ms is not None else float("nan"))
    app_ms = kt.get("apply_bf16", float("nan"))
    tr_ms = kt.get("apply_bf16_transpose", float("nan"))
    smx_ms = kt.get("mlr_softmax", float("nan"))
    gemm_flops = 2.0 * B * J * D                             # per GEMM stage
    # algorithmic HBM bytes per launch (the bf16 working copy of W counts: read by forward, written by apply)
    wb = 2 if not args.no_shadow else 4
    fwd_bytes = J * D * wb + B * D * 2 + B * J * 4           # W (copy / high plane) read once, X, logits written
    if split:      # both planes read, low plane written, high plane written where it changes, U^T, V^T read
        app_bytes = J * D * (4 + 2 + 2 * rewritten) + B * J * 2 + B * D * 2
    else:          # W read and written, bf16 copy written where it changes, U^T, V^T read
        app_bytes = J * D * (8 + (2 * rewritten if not args.no_shadow else 0)) + B * J * 2 + B * D * 2
    tr_bytes = 2 * (B * J * 2 + B * D * 2)                   # U, V read; U^T, V^T written
    smx_bytes = B * J * 4 + B * J * 2                        # logits read once, U written
    stages = {
        "forward_gemm": {"ms": fwd_ms, "tflops": gemm_flops / fwd_ms / 1e9,
                         "mfma_frac": gemm_flops / fwd_ms / 1e9 / PEAK_BF16_TFLOPS,
                         "hbm_gbs": fwd_bytes / fwd_ms / 1e6, "hbm_frac": fwd_bytes / fwd_ms / 1e6 / PEAK_HBM_GBS},
        "softmax": {"ms": smx_ms, "hbm_gbs": smx_bytes / smx_ms / 1e6,
                    "hbm_frac": smx_bytes / smx_ms / 1e6 / PEAK_HBM_GBS},
        "apply_transposes": {"ms": tr_ms, "hbm_gbs": tr_bytes / tr_ms / 1e6,
                             "hbm_frac": tr_bytes / tr_ms / 1e6 / PEAK_HBM_GBS},
        # zero fill + scatter of the aligned X and of V^T from the CSR rows, per step (0 for dense input)
        "csr_to_operand": {"ms": (prof.get("csr_to_operand", (0, 0.0))[1] + prof.get("fill", (0, 0.0))[1]) / args.steps},
        # forward over the stored entries of CSR samples (sfb_mlr_sf_csr's sparse route): HBM-bound, one pass over
        # the bf16 image of W, the logits written, the re-laid entries read; 0 when the dense product ran
        "forward_gather": ({"ms": gather_ms, "nnz_per_sample": nnz_mean,
                            "hbm_gbs": (J * D * 2 + B * J * 4 + 4 * nnz_mean * B) / gather_ms / 1e6,
                            "hbm_frac": (J * D * 2 + B * J * 4 + 4 * nnz_mean * B) / gather_ms / 1e6 / PEAK_HBM_GBS}
                           if gather_ms is not None else {"ms": 0.0}),
        "apply_gemm": {"ms": app_ms, "tflops": gemm_flops / app_ms / 1e9,
                       "mfma_frac": gemm_flops / app_ms / 1e9 / PEAK_BF16_TFLOPS,
                       "hbm_gbs": app_bytes / app_ms / 1e6, "hbm_frac": app_bytes / app_ms / 1e6 / PEAK_HBM_GBS},
    }
    if gather_ms is not None:
        stages["forward_gemm"] = {"ms": 0.0, "note": "the dense product did not run: see forward_gather"}
    # Roofline of the dominant kernel.  At this shape the forward contraction is
    # MFMA-bound (845 flop/B); the apply is bound by whichever roof its flops per
    # algorithmic byte put it under (ridge: 312 flop/B; 250 with the fp32 array,
    # 330 with the two planes when hardly any high half changes).
    # `traffic`: HBM-side bytes per launch of that kernel from the rocprofv3 --pmc
    # passes (FETCH_SIZE, WRITE_SIZE, scaled by the copy-kernel calibration) that
    # the committed summary under profiles/ records; null if it has no such line.
    traffic, traffic_current = profile_traffic_bytes()
    if fwd_ms >= app_ms:
        roof = {"kernel": "sf_gemm_kernel<0> (forward)", "bound": "mfma", "achieved": stages["forward_gemm"]["tflops"],
                "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": stages["forward_gemm"]["mfma_frac"],
                "traffic": traffic.get("sf_gemm_kernel<0>")}
    else:
        name = "sf_gemm_kernel<2> (apply on the two planes)" if split else "sf_gemm_kernel<1> (apply)"
        if gemm_flops / app_bytes > PEAK_BF16_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9):
            roof = {"kernel": name, "bound": "mfma", "achieved": stages["apply_gemm"]["tflops"],
                    "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": stages["apply_gemm"]["mfma_frac"]}
        else:
            roof = {"kernel": name, "bound": "hbm", "achieved": stages["apply_gemm"]["hbm_gbs"],
                    "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": stages["apply_gemm"]["hbm_frac"]}
        roof["traffic"] = traffic.get("sf_gemm_kernel<2>" if split else "sf_gemm_kernel<1>")
        roof["flop_per_algorithmic_byte"] = gemm_flops / app_bytes
        roof["algorithmic_bytes"] = app_bytes
        roof["bf16_image_groups_rewritten"] = rewritten
    roof["traffic_unit"] = "bytes per launch (rocprofv3 --pmc, separate run; see profiles/)" if traffic_current else \
        "null: the committed counter profile was taken on other kernel sources than this tree's"

    out = {
        "metric": "rank-1 SF updates applied/sec (SF compute + reconstruct/apply), MLR J=325k D=10k",
        "value": B / (ms_per_step * 1e-3),
        "unit": "updates/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "mlr_large_bf16: MLR J=325000 D=10000 B=N=1024, bf16 X/U/V, fp32 W and accumulate, "
                               "X ~ N(0,1) with %g%% zeros stored " % (100 * zero_frac) + ("as CSR rows" if args.csr else "dense") + ", eta=0.001; W kept as "
                               + ("two 16-bit planes (hi = bf16 operand of the forward, lo = the other half of the fp32 word)"
                                  if split else "an fp32 array plus a bf16 working copy"),
                   "J": J, "D": D, "B": B, "rank1_terms_per_step": B},
        "ms_per_step_events": {"median": per_step[len(per_step) // 2], "min": per_step[0], "max": per_step[-1]},
        "tflops_gemm_stages": 2 * gemm_flops / (ms_per_step * 1e-3) / 1e12,
        "mfma_frac_gemm_stages": (2 * gemm_flops / ((fwd_ms + app_ms) * 1e-3) / 1e12 / PEAK_BF16_TFLOPS if gather_ms is None
                                  else gemm_flops / (app_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS),
        "stages": stages,
        "roofline": roof,
    }
    if args.measured_peaks is not None:
        out["measured_peaks"] = args.measured_peaks
    if args.peers > 0 and not args.csr:
        # One GPU's share of a broadcast step with P = peers + 1 workers (Section 3: every worker applies the SF sets
        # of all workers): the local block and the peers' blocks in one sfb_apply call.  Peer factors by the input
        # recipe of the peer workloads (softmax of N(0,1) logits minus a uniform one-hot; samples like X), drawn on
        # the device because of their size.
        P1 = args.peers + 1
        g2 = torch.Generator(device=dev)
        g2.manual_seed(1)
        U_all = torch.empty((P1 * B, J), dtype=torch.bfloat16, device=dev)
        V_all = torch.empty((P1 * B, D), dtype=torch.bfloat16, device=dev)
        U_all[:B].copy_(U)
        V_all[:B].copy_(Xs[0])
        for q in range(1, P1):
            for r0 in range(0, B, 128):          # (in pieces: an fp32 block of logits is 1.3 GB)
                lg = torch.randn((128, J), dtype=torch.float32, device=dev, generator=g2)
                pr = torch.softmax(lg, dim=1)
                lab = torch.randint(0, J, (128,), device=dev, generator=g2)
                pr[torch.arange(128, device=dev), lab] -= 1.0
                U_all[q * B + r0:q * B + r0 + 128].copy_(pr)
            xv = torch.randn((B, D), dtype=torch.float32, device=dev, generator=g2)
            xv *= (torch.rand((B, D), device=dev, generator=g2) >= zero_frac)
            V_all[q * B:(q + 1) * B].copy_(xv)
        del lg, pr, xv
        for _ in range(2):
            ctx.sfb_apply(W, U_all, V_all, eta)
        torch.cuda.synchronize()
        ctx.sfb_profile_enable(True)
        ctx.sfb_profile_collect()
        reps = 3
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(ctx.stream)
        for _ in range(reps):
            ctx.sfb_apply(W, U_all, V_all, eta)
        e1.record(ctx.stream)
        torch.cuda.synchronize()
        prof2 = ctx.sfb_profile_collect()
        ctx.sfb_profile_enable(False)
        k2 = {k: v[1] / v[0] for k, v in prof2.items()}
        fl = 2.0 * P1 * B * J * D
        out["apply_with_peers"] = {
            "peers": args.peers, "N": P1 * B, "ms_per_call": e0.elapsed_time(e1) / reps,
            "transposes_ms": k2.get("apply_bf16_transpose"), "apply_gemm_ms": k2.get("apply_bf16"),
            "tflops": fl / k2["apply_bf16"] / 1e9, "mfma_frac": fl / k2["apply_bf16"] / 1e9 / PEAK_BF16_TFLOPS,
            "updates_per_s_apply_only": P1 * B / (e0.elapsed_time(e1) / reps * 1e-3)}
        del U_all, V_all
    if split and not args.no_other_layout:
        # the same steps with W kept as an fp32 array plus bf16 working copy (the library's other layout), untimed
        # set-up, a few timed steps: reported beside the headline, never as `value`
        ctx.sfb_split_detach()
        ctx.sfb_shadow_attach(W)
        for i in range(2):
            step(i)
        torch.cuda.synchronize()
        n2 = min(args.steps, 5)
        t0 = time.perf_counter()
        for i in range(n2):
            step(2 + i)
        torch.cuda.synchronize()
        out["ms_per_step_fp32_layout"] = (time.perf_counter() - t0) * 1e3 / n2
    if not args.no_cpu_baseline:
        log("bench: timing the CPU oracle on a bounded sample")
        out["cpu_baseline"] = cpu_baseline_mlr(cfg, X0, y0, W[:min(J, 32768)].cpu().numpy())
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
