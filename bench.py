#!/usr/bin/env python3
"""Benchmark: ms per linear layer pruned on one MI355X.

A "step" is one pass of the whole hot path over one synthetic layer: Hessian accumulation
over all calibration tokens, damped factorisation, and the column-block sweep (mask, per-row
solve, trailing update).  Default workload: the LLaMA-7B-shaped 4096 x 11008 layer (b = 11008
input channels), 262144 fp16 calibration tokens, 2:4 sparsity, block 128, damping 0.01.
Inputs are resident in HBM before the timed region starts.

Prints ONE JSON line: the metric (ms per layer) with its phases, a `roofline` object for the
dominant kernel (algorithmic flops per launch / measured launch time against the MI355X fp16
matrix-core peak, plus measured L2 <-> fabric bytes) and a `cpu_baseline` object (the float64
oracle timed on a bounded sample of the same workload on the host cores).
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

PEAK_MFMA_F16_TFLOPS = 2500.0   # MI355X dense fp16/bf16 matrix-core peak
PEAK_HBM_GBS = 8000.0

# Bytes that crossed the L2 <-> fabric boundary per launch of the dominant kernel
# (k_syrk16_dma), from two rocprofv3 --pmc runs (FETCH_SIZE, then WRITE_SIZE) of
# `bench.py --steps 1 --warmup 0 --no-cpu-baseline --copy-probe`, each scaled by what the same
# counter reads for the 1 GiB copy of --copy-probe (factors 2.0 and 1.0, i.e. the counters tick
# in 2 KiB and 1 KiB).  See profiles/k_syrk16_dma_4096x11008_traffic.md.  Key: (c, b, T, calls).
MEASURED_TRAFFIC_BYTES = {
    (4096, 11008, 262144, 1): 34231605 * 2 * 1024 + 1120862 * 1024,
}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--c", type=int, default=4096)
    ap.add_argument("--b", type=int, default=11008)
    ap.add_argument("--tokens", type=int, default=262144)
    ap.add_argument("--mode", default="nm", choices=["nm", "unstructured", "structured"])
    ap.add_argument("--n", type=int, default=2)
    ap.add_argument("--m", type=int, default=4)
    ap.add_argument("--sparsity", type=float, default=0.5)
    ap.add_argument("--block", type=int, default=128)
    ap.add_argument("--damping", type=float, default=0.01)
    ap.add_argument("--outlier-fraction", type=float, default=0.0,
                    help="alpha of the n:m algorithm: share of rows (largest loss) left dense")
    ap.add_argument("--rho", type=float, default=0.0,
                    help="correlated calibration channels (0 = independent, as configured)")
    ap.add_argument("--outlier-channels", action="store_true",
                    help="heavy-tailed activations: 0.5 %% of the channels scaled x20-100")
    ap.add_argument("--w-std", type=float, default=0.02)
    ap.add_argument("--chunks", type=int, default=1,
                    help="number of thanos_hessian_accumulate calls the tokens are split into")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--phases-only", action="store_true", help="skip the oracle, print phases")
    ap.add_argument("--copy-probe", action="store_true",
                    help="run one plain 1 GiB device copy first (reference for scaling the "
                         "FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    return ap.parse_args()


def make_inputs(args, torch):
    """Seeded synthetic layer on the device: W ~ N(0, w_std^2) fp16, X[t, j] = s_j * g, fp16
    (synth.make_layer_on_device; --rho / --outlier-channels select the correlated and the
    heavy-tailed variant of the recipe)."""
    from synth import LayerSpec, make_layer_on_device
    spec = LayerSpec("bench", c=args.c, b=args.b, tokens=args.tokens, dtype="f16", seed=0,
                     rho=getattr(args, "rho", 0.0), outliers=getattr(args, "outlier_channels", False),
                     w_std=getattr(args, "w_std", 0.02))
    return make_layer_on_device(spec, torch)


def cpu_baseline(args, W, X, torch):
    """The float64 oracle, as it stands, on a bounded sample of the same workload."""
    import numpy as np
    from oracle import thanos_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        threads = max((p.get("num_threads", 1) for p in threadpool_info()), default=1)
    except Exception:  # pragma: no cover
        threads = os.cpu_count() or 1
    tok_s = min(args.tokens, 32768)
    rows_s = min(args.c, 256)
    Xs = X[:tok_s].cpu().numpy()
    Ws = W[:rows_s].cpu().numpy()
    t0 = time.perf_counter()
    Hs = orc.hessian(Xs)
    t_h = time.perf_counter() - t0
    t0 = time.perf_counter()
    U = orc.inverse_factor(orc.damped(Hs, args.damping))
    t_f = time.perf_counter() - t0
    t0 = time.perf_counter()
    if args.mode == "structured":
        orc.prune_structured(Ws, Hs, args.sparsity, args.outlier_fraction, args.damping)
    else:
        orc.prune_fast(Ws, Hs, mode=args.mode, p=args.sparsity, n=args.n, m=args.m, B=args.block,
                       damp=args.damping, U=U,
                       alpha=args.outlier_fraction if args.mode == "nm" else 0)
    t_s = time.perf_counter() - t0
    est = t_h * (args.tokens / tok_s) + t_f + t_s * (args.c / rows_s)
    return {
        "value": est * 1e3, "unit": "ms per layer (extrapolated)", "cores": int(threads),
        "kind": "oracle",
        "sample": (f"hessian on {tok_s} of {args.tokens} tokens ({t_h:.2f}s, scaled by tokens) + "
                   f"full {args.b}x{args.b} factor ({t_f:.2f}s) + single-factorisation sweep of "
                   f"{rows_s} of {args.c} rows ({t_s:.2f}s, scaled by rows)"),
    }


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(the path is built and measured on a single MI355X)", file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2504_05346_amd as th
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    th.lib()

    W, X = make_inputs(args, torch)
    if args.copy_probe:
        src = torch.full((1 << 28,), 1.0, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)                       # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst
    c, b, T = args.c, args.b, args.tokens
    o = th.PruneOpts(mode={"nm": th.THANOS_NM, "unstructured": th.THANOS_UNSTRUCTURED,
                           "structured": th.THANOS_STRUCTURED}[args.mode],
                     sparsity=args.sparsity, n=args.n, m=args.m, block_size=args.block,
                     damping=args.damping, outlier_fraction=args.outlier_fraction)
    nbytes = th.thanos_prune_workspace_bytes(c, b, o)
    assert nbytes > 0
    ws = torch.empty((nbytes,), dtype=torch.uint8, device="cuda")
    H = torch.empty((b, b), dtype=torch.float32, device="cuda")
    Wo = torch.empty((c, b), dtype=torch.float32, device="cuda")
    M = torch.empty((c, b), dtype=torch.uint8, device="cuda")
    info = torch.zeros((1,), dtype=torch.int32, device="cuda")
    edges = [round(i * T / args.chunks) for i in range(args.chunks + 1)]

    ev = lambda: torch.cuda.Event(enable_timing=True)
    acc_ms, prune_ms = [], []

    def step(record):
        e0, e1, e2 = ev(), ev(), ev()
        H.zero_()
        e0.record()
        for a0, a1 in zip(edges[:-1], edges[1:]):
            th.thanos_hessian_accumulate(H, X[a0:a1])
        e1.record()
        th.thanos_prune_layer(W, H, o, Wo, None, M, ws, info)
        e2.record()
        if record is not None:
            record.append((e0, e1, e2))

    for _ in range(args.warmup):
        step(None)
    torch.cuda.synchronize()
    evs = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(evs)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    assert int(info.item()) == 0, f"numerical failure, info={int(info.item())}"
    for e0, e1, e2 in evs:
        acc_ms.append(e0.elapsed_time(e1))
        prune_ms.append(e1.elapsed_time(e2))
    ms_per_step = wall * 1e3 / args.steps
    syrk_ms = sum(acc_ms) / len(acc_ms) / args.chunks          # average launch duration
    flops_per_launch = (T / args.chunks) * b * (b + 1)         # lower-triangular Gram matrix
    achieved = flops_per_launch / (syrk_ms * 1e-3) / 1e12

    kept = int((M == 0).sum().item())
    workload = (f"{c}x{b} fp16 layer, {T} fp16 calibration tokens, "
                + (f"{args.n}:{args.m}" if args.mode == "nm" else f"{args.sparsity:g} {args.mode}")
                + f", block {args.block}, damping {args.damping:g}"
                + (f", outlier rows {args.outlier_fraction:g}" if args.outlier_fraction else ""))
    out = {
        "metric": "ms per linear layer pruned (4096x11008, 2:4); MFMA% / HBM GB/s per phase",
        "value": ms_per_step, "unit": "ms", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": False,
        "scaling": "weak", "vs_baseline": None, "dtype": "f16 in / f32 accumulate",
        "data": "synthetic", "config": {"workload": workload, "accumulate_calls": args.chunks},
        "phases_ms": {"hessian_accumulate": sum(acc_ms) / len(acc_ms),
                      "factor_and_sweep": sum(prune_ms) / len(prune_ms)},
        "kept_fraction": kept / (c * b),
        "roofline": {"kernel": "k_syrk16_dma (thanos_hessian_accumulate)", "bound": "mfma",
                     "achieved": achieved, "peak": PEAK_MFMA_F16_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / PEAK_MFMA_F16_TFLOPS,
                     "traffic": MEASURED_TRAFFIC_BYTES.get((c, b, T, args.chunks))},
    }
    if not (args.no_cpu_baseline or args.phases_only):
        out["cpu_baseline"] = cpu_baseline(args, W, X, torch)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
