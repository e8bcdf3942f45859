"""Measured ceilings of the GPU (matrix-core fp16 rate of an MFMA-only loop with the shader
clock it runs at, HBM copy bandwidth), from libthanos_probe.so.

    python -m paper_2504_05346_amd.peak_probe          # prints one JSON object

bench.py --measured-peaks adds the same object to its line.  The numbers put the roofline
fractions (quoted against the data-sheet peaks) next to what the chip sustains.
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


if __name__ == "__main__":
    import torch
    assert torch.cuda.is_available(), "needs a GPU"
    print(json.dumps(measure(torch)))
