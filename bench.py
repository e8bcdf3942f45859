#!/usr/bin/env python3
"""Benchmark: ms per linear layer pruned on one MI355X.

A "step" is one pass of the whole hot path over one synthetic layer: Hessian accumulation
over all calibration tokens, damped factorisation, and the column-block sweep (mask, per-row
solve, trailing update).  Default workload: the LLaMA-7B-shaped 4096 x 11008 layer (b = 11008
input channels), 262144 fp16 calibration tokens, 2:4 sparsity, block 128, damping 0.01.
Inputs are resident in HBM before the timed region starts.

Prints ONE JSON line:
  * the metric (ms per layer, wall clock over the timed steps) with `phases_ms`: the accumulate
    call timed with events inside the timed region, and factor / mask / solve / update from ONE
    diagnostic call after the timed region in which the library runs its kernels one after the
    other and times the phases itself (in the timed region those phases overlap on helper
    streams, so their sum exceeds `factor_and_sweep_overlapped`);
  * `roofline`: the dominant kernel (the SYRK of the accumulate call) against the fp16
    matrix-core peak, with the L2 <-> fabric bytes of a tracked rocprofv3 summary;
  * `rooflines`: one entry per phase (algorithmic flops and bytes / phase time);
  * `extra`: the second workload of the target, the same layer at 50 % unstructured sparsity,
    timed the same way in the same run (only when the default workload is run);
  * `measured_peaks`: the accumulate kernel on an all-zero matrix of the same shape, and what this
    GPU sustains in a loop of nothing but fp16 MFMAs (smooth and
    random operands, with the shader clock it runs at) and in a plain HBM copy;
  * `cpu_baseline`: the float64 oracle timed on a bounded sample on the host cores.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_MFMA_F16_TFLOPS = 2500.0   # MI355X dense fp16/bf16 matrix-core peak
PEAK_MFMA_F32_TFLOPS = 157.3    # fp32 matrix-core peak (= fp32 vector peak)
PEAK_HBM_GBS = 8000.0

# L2 <-> fabric bytes per launch of the dominant kernel come from a tracked rocprofv3 --pmc
# summary (FETCH_SIZE and WRITE_SIZE runs, scaled by a 1 GiB copy); the file carries one
# machine-readable line per measured shape:  traffic_bytes_per_launch[c=..,b=..,T=..,calls=..] = N
TRAFFIC_PROFILE = "profiles/k_syrk16_dma_4096x11008_traffic.md"


def measured_traffic(c, b, T, calls):
    try:
        text = open(os.path.join(ROOT, TRAFFIC_PROFILE)).read()
    except OSError:
        return None
    m = re.search(rf"traffic_bytes_per_launch\[c={c},b={b},T={T},calls={calls}\]\s*=\s*(\d+)", text)
    return int(m.group(1)) if m else None


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
    ap.add_argument("--no-extra", action="store_true",
                    help="do not time the 50 %% unstructured workload next to the default one")
    ap.add_argument("--phases-only", action="store_true", help="skip the oracle, print phases")
    ap.add_argument("--no-measured-peaks", action="store_true",
                    help="skip the measured ceilings of this GPU (MFMA-only loop with its shader "
                         "clock on smooth and on random operands, HBM copy; ~0.1 s)")
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


def workload_name(args, mode):
    c, b, T = args.c, args.b, args.tokens
    return (f"{c}x{b} fp16 layer, {T} fp16 calibration tokens, "
            + (f"{args.n}:{args.m}" if mode == "nm" else f"{args.sparsity:g} {mode}")
            + f", block {args.block}, damping {args.damping:g}"
            + (f", outlier rows {args.outlier_fraction:g}" if args.outlier_fraction else "")
            + (f", rho {args.rho:g}" if args.rho else "")
            + (", outlier channels" if args.outlier_channels else ""))


def phase_rooflines(args, mode, ph, M, torch):
    """Algorithmic work of each phase / its time in the diagnostic (serialised) call."""
    c, b, B = args.c, args.b, args.block
    starts = list(range(0, b, B))
    resid = sum(b - j1 for j1 in starts)                       # sum over blocks of (b - j1)
    out = []

    def entry(phase, bound, work, unit, peak, ms, **kw):
        ach = work / (ms * 1e-3) / (1e12 if unit == "TFLOP/s" else 1e9) if ms > 0 else None
        e = {"phase": phase, "bound": bound, "achieved": ach, "peak": peak, "unit": unit,
             "frac": (ach / peak) if ach else None, "ms": ms}
        e.update(kw)
        out.append(e)

    entry("factor", "mfma", (2.0 / 3.0) * b ** 3, "TFLOP/s", PEAK_MFMA_F32_TFLOPS, ph["factor"],
          note="fp32 products (Cholesky b^3/3 + triangular inverse b^3/3) against the fp32 "
               "matrix-core peak; computed as 6 bf16 MFMAs per product")
    upd_flops = 2.0 * c * sum(min(B, b - j1) * (b - j1) for j1 in starts)
    upd_bytes = 2.0 * 4.0 * c * resid
    entry("update", "mfma", upd_flops, "TFLOP/s", PEAK_MFMA_F32_TFLOPS, ph["update"],
          note="rank-B update W[:, j1:] -= Lambda P_k, fp32 products as 6 bf16 MFMAs")
    entry("update", "hbm", upd_bytes, "GB/s", PEAK_HBM_GBS, ph["update"],
          note="read + write of every residual fp32 weight once per block")
    if out[-2]["frac"] is not None:
        binds = "mfma" if out[-2]["frac"] >= out[-1]["frac"] else "hbm"
        out[-2]["binds"] = out[-1]["binds"] = binds
    if mode == "unstructured":
        entry("mask", "hbm", 4.0 * c * resid, "GB/s", PEAK_HBM_GBS, ph["mask"],
              note="whole selection chain of a block (all its launches) over one algorithmic "
                   "read of the residual fp32 weights per block")
    else:
        out.append({"phase": "mask", "bound": "hbm", "achieved": None, "peak": PEAK_HBM_GBS,
                    "unit": "GB/s", "frac": None, "ms": 0.0,
                    "note": "n:m: the per-group choice is made inside the solve kernel on the "
                            "block's own c x B weights (2 MB per block): no pass of its own"})
    # per-row systems: s unknowns per (row, block) from the mask itself
    nblk = len(starts)
    pad = nblk * B - b
    Mp = torch.nn.functional.pad(M, (0, pad)) if pad else M
    s = Mp.view(c, nblk, B).sum(dim=2, dtype=torch.float64)
    flops = float((s ** 3 / 3.0 + 2.0 * s ** 2 + 2.0 * s * B).sum().item())
    systems = int((s > 0).sum().item())
    ms = ph["solve"]
    entry("solve", "alu", flops, "TFLOP/s", PEAK_MFMA_F32_TFLOPS, ms,
          systems_per_s=(systems / (ms * 1e-3)) if ms > 0 else None, systems=systems,
          mean_unknowns=float(s.sum().item()) / max(systems, 1),
          note="s^3/3 + 2 s^2 + 2 s B fp32 flops per system against the fp32 vector peak; the "
               "honest bound is instruction issue / latency of the dependent eliminations")
    entry("solve", "hbm", 9.0 * c * b, "GB/s", PEAK_HBM_GBS, ms,
          note="block weights read, multipliers and mask bytes written: 9 bytes per weight")
    return out


def run_workload(args, mode, W, X, torch, th, with_traffic):
    c, b, T = args.c, args.b, args.tokens
    o = th.PruneOpts(mode={"nm": th.THANOS_NM, "unstructured": th.THANOS_UNSTRUCTURED,
                           "structured": th.THANOS_STRUCTURED}[mode],
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
    acc_ms = [e0.elapsed_time(e1) for e0, e1, _ in evs]
    prune_ms = [e1.elapsed_time(e2) for _, e1, e2 in evs]
    ms_per_step = wall * 1e3 / args.steps
    acc = sum(acc_ms) / len(acc_ms)
    syrk_ms = acc / args.chunks                                # average launch duration
    flops_per_launch = (T / args.chunks) * b * (b + 1)         # lower-triangular Gram matrix
    achieved = flops_per_launch / (syrk_ms * 1e-3) / 1e12
    kept = int((M == 0).sum().item())

    res = {
        "workload": workload_name(args, mode), "ms_per_step": ms_per_step,
        "kept_fraction": kept / (c * b),
        "phases_ms": {"hessian_accumulate": acc,
                      "factor_and_sweep_overlapped": sum(prune_ms) / len(prune_ms)},
        "roofline": {"kernel": "k_syrk16_dma (thanos_hessian_accumulate)", "bound": "mfma",
                     "achieved": achieved, "peak": PEAK_MFMA_F16_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / PEAK_MFMA_F16_TFLOPS,
                     "traffic": measured_traffic(c, b, T, args.chunks) if with_traffic else None,
                     "traffic_source": TRAFFIC_PROFILE if with_traffic else None},
    }
    if mode != "structured":
        # one diagnostic call: kernels serialised on one stream, phases timed by the library
        phase_buf = (ctypes.c_float * len(th.THANOS_PHASES))()
        o.phase_ms_out = ctypes.addressof(phase_buf)
        th.thanos_prune_layer(W, H, o, Wo, None, M, ws, info)
        torch.cuda.synchronize()
        o.phase_ms_out = None
        assert int(info.item()) == 0
        ph = {name: float(phase_buf[i]) for i, name in enumerate(th.THANOS_PHASES)}
        res["phases_ms"].update({k: ph[k] for k in ("prep", "factor", "mask", "solve", "update",
                                                    "finalise")})
        res["phases_ms"]["note"] = ("prep .. finalise: one diagnostic call with the kernels "
                                    "serialised on one stream; in the timed steps they overlap")
        res["rooflines"] = ([dict(res["roofline"], phase="hessian_accumulate", ms=acc)]
                            + phase_rooflines(args, mode, ph, M, torch))
    return res


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

    main_res = run_workload(args, args.mode, W, X, torch, th, with_traffic=True)
    out = {
        "metric": "ms per linear layer pruned (4096x11008, 2:4); MFMA% / HBM GB/s per phase",
        "value": main_res["ms_per_step"], "unit": "ms", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": main_res["ms_per_step"], "higher_is_better": False,
        "scaling": "weak", "vs_baseline": None,
        "dtype": ("f16 in / f32 accumulate (Hessian); factor, block rows and trailing update: "
                  "f32 storage, products as 3-way split bf16 on the matrix cores (6 bf16 MFMAs "
                  "per fp32 product); per-row solves f32"),
        "data": "synthetic",
        "config": {"workload": main_res["workload"], "accumulate_calls": args.chunks},
        "phases_ms": main_res["phases_ms"], "kept_fraction": main_res["kept_fraction"],
        "roofline": main_res["roofline"],
    }
    if "rooflines" in main_res:
        out["rooflines"] = main_res["rooflines"]
    default_workload = (args.mode == "nm" and (args.n, args.m) == (2, 4)
                        and not args.outlier_fraction)
    if default_workload and not args.no_extra:
        # the second half of the target: the same layer at 50 % unstructured sparsity (Alg. 1)
        x = run_workload(args, "unstructured", W, X, torch, th, with_traffic=False)
        out["extra"] = [{"metric": "ms per linear layer pruned", "value": x["ms_per_step"],
                         "unit": "ms", "steps": args.steps, "warmup": args.warmup,
                         "config": {"workload": x["workload"], "accumulate_calls": args.chunks},
                         "phases_ms": x["phases_ms"], "kept_fraction": x["kept_fraction"],
                         "rooflines": x.get("rooflines")}]
    if not args.no_measured_peaks:
        # what this chip sustains, next to the data-sheet peaks the fractions are quoted against:
        # its matrix cores are clocked down under load, and more so when the operands toggle
        from paper_2504_05346_amd import peak_probe
        mp = peak_probe.measure(torch)
        out["measured_peaks"] = mp
        ceil = [m["tflops"] for m in mp["mfma_f16"]
                if m["operands"] == "random" and m["run"] == "sustained"]
        if ceil:
            out["roofline"]["frac_of_measured_mfma_only_rate"] = out["roofline"]["achieved"] / ceil[0]
        # the accumulate call of this workload once more on an all-zero calibration matrix of the
        # same shape: same kernel, instructions, addresses and traffic, operands that do not
        # toggle.  What it gains over the timed rate is what the power limit takes on real data.
        Xz = torch.zeros_like(X)
        Hz = torch.zeros((args.b, args.b), dtype=torch.float32, device="cuda")
        best = None
        for _ in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            th.thanos_hessian_accumulate(Hz, Xz)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1)
            best = ms if best is None else min(best, ms)
        del Xz, Hz
        tf = args.tokens * args.b * (args.b + 1) / best / 1e9
        mp["accumulate_same_kernel_on_zeros"] = {
            "ms": best, "tflops": tf, "frac_of_peak": tf / out["roofline"]["peak"],
            "note": "one call over all tokens; compare roofline.achieved (same kernel on the workload's data)"}
    if not (args.no_cpu_baseline or args.phases_only):
        out["cpu_baseline"] = cpu_baseline(args, W, X, torch)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
