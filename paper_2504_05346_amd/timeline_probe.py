"""Where the time of a block update goes: timestamps taken inside `k_update` and inside the
tile product it runs, from libthanos_timeline.so (the product's sources compiled with
-DTHANOS_TIMELINE, see csrc/timeline.h; built by `python -m paper_2504_05346_amd.build`).

    python -m paper_2504_05346_amd.timeline_probe        # prints one JSON object

Two launches of the 4096 x 11008 layer are recorded, both with 1472 workgroups:
  * 50 % unstructured, B = 128: the update of block 40 (K = 128, all columns right of it);
  * 2:4, B = 128: the far update of the fifth super-block (K = 1024).
Times in microseconds, medians over the workgroups.  The instrumented kernels are a few per
cent slower than the product's (one extra wait in front of the row pass, the stores of the
timestamps).
"""
from __future__ import annotations

import ctypes
import json
import os
import types

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
lib_path = os.path.join(_HERE, "libthanos_timeline.so")
SLOTS, WGS = 80, 4096


def _run(torch, th, L, W, H, opts, grid):
    c, b = W.shape
    ws = torch.zeros((th.thanos_prune_workspace_bytes(c, b, opts),), dtype=torch.uint8, device="cuda")
    Wo = torch.empty((c, b), dtype=torch.float32, device="cuda")
    M = torch.empty((c, b), dtype=torch.uint8, device="cuda")
    info = torch.zeros((1,), dtype=torch.int32, device="cuda")
    assert L.thanos_timeline_select(0) == 0
    th.thanos_prune_layer(W, H, opts, Wo, None, M, ws, info)      # warm-up, nothing recorded
    torch.cuda.synchronize()
    assert L.thanos_timeline_clear() == 0 and L.thanos_timeline_select(grid) == 0
    th.thanos_prune_layer(W, H, opts, Wo, None, M, ws, info)
    torch.cuda.synchronize()
    assert int(info.item()) == 0
    buf = np.zeros(WGS * SLOTS, dtype=np.uint64)
    assert L.thanos_timeline_read(buf.ctypes.data, buf.nbytes) == 0
    ts = buf.reshape(WGS, SLOTS).astype(np.int64)
    ts = ts[ts[:, 0] > 0]
    return (ts - ts[:, 0].min()) / 100.0       # 100 MHz wall clock -> microseconds


def _med(a):
    return float(np.median(a))


def measure(torch) -> dict:
    if not os.path.exists(lib_path):
        raise RuntimeError(f"{lib_path} not found: build it with `python -m paper_2504_05346_amd.build`")
    from . import binding as bd
    import paper_2504_05346_amd as th
    assert bd._lib is None, "run in a fresh process: the binding must load the timeline build"
    bd.lib_path = lib_path
    L = bd.lib()
    L.thanos_timeline_select.argtypes = [ctypes.c_int]
    L.thanos_timeline_read.argtypes = [ctypes.c_void_p, ctypes.c_size_t]
    from synth import LayerSpec, make_layer_on_device
    c, b, B = 4096, 11008, 128
    W, X = make_layer_on_device(LayerSpec("timeline", c=c, b=b, tokens=32768, dtype="f16", seed=0), torch)
    H = torch.zeros((b, b), dtype=torch.float32, device="cuda")
    th.thanos_hessian_accumulate(H, X)
    del X
    grid = 8 * 4 * ((b - 5120) // 128)          # 32 row tiles in 8 bands of 4, 46 column tiles
    out = {"layer": f"{c}x{b}", "workgroups_of_the_recorded_launch": grid}

    us = _run(torch, th, L, W, H, th.PruneOpts(mode=th.THANOS_UNSTRUCTURED, sparsity=0.5,
                                               block_size=B, damping=0.01), grid)
    d = np.diff(us[:, :6], axis=1)
    out["unstructured_update_of_block_40"] = {
        "workgroups": int(len(us)), "launch_span_us": float(us[:, 5].max()),
        "per_workgroup_us": {"product_K128": _med(d[:, 0]), "stage_tile_in_lds": _med(d[:, 1]),
                             "wait_for_old_tile_values": _med(d[:, 2]),
                             "row_pass_and_stores": _med(d[:, 3]),
                             "window_counts_and_lists": _med(d[:, 4]),
                             "total": _med(us[:, 5] - us[:, 0])},
        "start_of_the_three_rounds_us": [float(x) for x in np.percentile(us[:, 0], [10, 50, 90])]}

    us = _run(torch, th, L, W, H, th.PruneOpts(mode=th.THANOS_NM, n=2, m=4, block_size=B,
                                               damping=0.01), grid)
    its = 17
    p0, p1 = us[:, 8:8 + 4 * its:4], us[:, 9:9 + 4 * its:4]
    c0, c1 = us[:, 10:10 + 4 * its:4], us[:, 11:11 + 4 * its:4]
    nxt = us[:, 12:12 + 4 * its:4]
    sl = slice(2, its - 1)
    out["nm_far_update_K1024"] = {
        "workgroups": int(len(us)), "launch_span_us": float(us[:, 5].max()),
        "per_slab_of_32_k_us": {"producer_fill_split_store_request": _med((p1 - p0)[:, sl]),
                                "barrier_to_multiply": _med((c0 - p1)[:, sl]),
                                "multiply_48_mfma_per_wavefront": _med((c1 - c0)[:, sl]),
                                "barrier_to_next_fill": _med((nxt[:, :-1] - c1[:, :-1])[:, sl]),
                                "slab_period": _med(np.diff(p0, axis=1)[:, sl])},
        "per_workgroup_us": {"product_K1024": _med(us[:, 1] - us[:, 0]),
                             "total": _med(us[:, 5] - us[:, 0])}}
    return out


if __name__ == "__main__":
    import torch
    assert torch.cuda.is_available(), "needs a GPU"
    print(json.dumps(measure(torch)))
