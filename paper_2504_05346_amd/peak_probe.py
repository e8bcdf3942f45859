"""Measured ceilings of the GPU (matrix-core fp16 rate of an MFMA-only loop with the shader
clock it runs at, HBM copy bandwidth), from libthanos_probe.so.

    python -m paper_2504_05346_amd.peak_probe               # prints one JSON object
    python -m paper_2504_05346_amd.peak_probe --syrk-data   # adds: the Hessian kernel by operand data

bench.py adds the first object to its line as `measured_peaks`.  The numbers put the roofline
fractions (quoted against the data-sheet peaks) next to what the chip sustains.  `--syrk-data`
times the library's own accumulate call (same kernel, same instruction stream, same traffic) on
calibration matrices that differ only in their values: the difference is what the power limit
takes.
"""
from __future__ import annotations

import ctypes
import json
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
lib_path = os.path.join(_HERE, "libthanos_probe.so")


def measure(torch, mfma_ms: float = 20.0) -> dict:
    if not os.path.exists(lib_path):
        raise RuntimeError(f"{lib_path} not found: build it with `python -m paper_2504_05346_amd.build`")
    L = ctypes.CDLL(lib_path)
    vp, dp = ctypes.c_void_p, ctypes.POINTER(ctypes.c_double)
    L.thanos_probe_mfma_f16.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, vp, dp, dp, dp, vp]
    L.thanos_probe_copy.argtypes = [vp, vp, ctypes.c_int64, ctypes.c_int, dp, dp, vp]
    stream = int(torch.cuda.current_stream().cuda_stream)
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    wgs = cus                                   # one workgroup of 8 wavefronts per compute unit
    scratch = torch.zeros((16 * wgs + 64,), dtype=torch.uint8, device="cuda")
    ms, tf, clk = ctypes.c_double(), ctypes.c_double(), ctypes.c_double()
    out = {"compute_units": cus, "mfma_f16": []}
    # 32 cycles per MFMA at ~2 GHz: iterations for a short and for a long (sustained) run
    for operands in ("smooth", "random"):
        for label, target_ms in (("short", 1.0), ("sustained", mfma_ms)):
            iters = max(64, int(target_ms * 1e-3 * 1.6e9 / (2 * 8 * 32)))
            rc = L.thanos_probe_mfma_f16(wgs, iters, 1 if operands == "random" else 0,
                                         scratch.data_ptr(), ctypes.byref(ms), ctypes.byref(tf),
                                         ctypes.byref(clk), stream)
            if rc != 0:
                raise RuntimeError(f"probe failed: HIP error {rc}")
            out["mfma_f16"].append({"operands": operands, "run": label, "ms": ms.value,
                                    "tflops": tf.value, "shader_clock_ghz": clk.value})
    n = 1 << 30
    src = torch.ones((n,), dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    gbs = ctypes.c_double()
    rc = L.thanos_probe_copy(src.data_ptr(), dst.data_ptr(), n, 5, ctypes.byref(ms),
                             ctypes.byref(gbs), stream)
    if rc != 0:
        raise RuntimeError(f"copy probe failed: HIP error {rc}")
    out["hbm_copy"] = {"bytes": n, "ms": ms.value, "gbs_read_plus_write": gbs.value}
    return out


def syrk_by_data(torch, b: int = 11008, tokens: int = 262144, reps: int = 3) -> list:
    """thanos_hessian_accumulate on [tokens, b] fp16 matrices of different content."""
    from .binding import thanos_hessian_accumulate
    X = torch.empty((tokens, b), dtype=torch.float16, device="cuda")
    H = torch.zeros((b, b), dtype=torch.float32, device="cuda")
    chunk = 16384

    def fill(kind):
        g = torch.Generator(device="cuda")
        g.manual_seed(0)
        if kind == "zeros":
            X.zero_()
        elif kind == "ones":
            X.fill_(1.0)
        elif kind == "column-constant":      # random across channels, the same for every token
            X[:] = torch.randn((1, b), generator=g, device="cuda").half()
        else:
            for t0 in range(0, tokens, chunk):
                n = min(chunk, tokens - t0)
                if kind == "bernoulli{0,1}":
                    X[t0:t0 + n] = torch.randint(0, 2, (n, b), generator=g, device="cuda").half()
                else:                        # "normal"
                    X[t0:t0 + n] = torch.randn((n, b), generator=g, device="cuda",
                                               dtype=torch.float32).half()

    out = []
    for kind in ("normal", "zeros", "ones", "bernoulli{0,1}", "column-constant", "normal"):
        fill(kind)
        torch.cuda.synchronize()
        best = None
        for _ in range(reps):
            H.zero_()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            thanos_hessian_accumulate(H, X)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1)
            best = ms if best is None else min(best, ms)
        out.append({"data": kind, "ms": best, "tflops": tokens * b * (b + 1) / best / 1e9})
    return out


if __name__ == "__main__":
    import sys
    import torch
    assert torch.cuda.is_available(), "needs a GPU"
    res = measure(torch)
    if "--syrk-data" in sys.argv[1:]:
        res["syrk_by_data"] = syrk_by_data(torch)
    print(json.dumps(res))
