"""Layers that read the same input share the Hessian, hence the damped factor.

The q/k/v projections of an attention block, or the gate/up projections of an MLP, are pruned
against the same calibration input X (paper, Alg. 1: H depends on X only).  `prune_layer_set`
accumulates H once, factors it once and runs one sweep per weight matrix with `factor_in`
(include/thanos.h).  Sequencing and allocation only: every step runs in the library's kernels.
"""
from typing import Iterable, List, Sequence, Tuple

import torch

from .binding import (PruneOpts, thanos_factor, thanos_factor_workspace_bytes,
                      thanos_hessian_accumulate, thanos_prune_layer,
                      thanos_prune_workspace_bytes)


def prune_layer_set(weights: Sequence[torch.Tensor], x_chunks: Iterable[torch.Tensor], *, mode: int,
                    sparsity: float = 0.0, n: int = 0, m: int = 0, block_size: int = 128,
                    damping: float = 0.01, outlier_fraction: float = 0.0, cast: bool = False,
                    stream=None) -> Tuple[List[dict], torch.Tensor]:
    """Prune every matrix of `weights` (each c_i x b, same b, on the GPU) against the input given
    as token-major chunks [n_tok, b].  Returns ([{"W": fp32, "W_cast": dtype of the input or
    None, "mask": uint8, "info": int32[1]}, ...], H).  `info` follows thanos_prune_layer; the
    caller synchronises before reading it."""
    if not weights:
        raise ValueError("no weight matrix given")
    b = weights[0].shape[1]
    dev = weights[0].device
    H = torch.zeros((b, b), dtype=torch.float32, device=dev)
    for xc in x_chunks:
        thanos_hessian_accumulate(H, xc, 1.0, stream)
    U = torch.empty((b, b), dtype=torch.float32, device=dev)
    xnorm2 = torch.empty((b,), dtype=torch.float32, device=dev)
    finfo = torch.zeros((1,), dtype=torch.int32, device=dev)
    fws = torch.empty((thanos_factor_workspace_bytes(b),), dtype=torch.uint8, device=dev)
    thanos_factor(H, damping, U, xnorm2, fws, finfo, stream)
    del fws
    out = []
    ws = None
    for W in weights:
        c = W.shape[0]
        assert W.shape[1] == b and W.device == dev
        o = PruneOpts(mode=mode, sparsity=float(sparsity), n=n, m=m, block_size=block_size,
                      damping=damping, outlier_fraction=float(outlier_fraction))
        o.factor_in, o.xnorm2_in = U.data_ptr(), xnorm2.data_ptr()
        need = thanos_prune_workspace_bytes(c, b, o)
        if need == 0:
            raise ValueError("options rejected by thanos_prune_workspace_bytes")
        if ws is None or ws.numel() < need:
            ws = torch.empty((need,), dtype=torch.uint8, device=dev)
        res = {"W": torch.empty((c, b), dtype=torch.float32, device=dev),
               "W_cast": torch.empty((c, b), dtype=W.dtype, device=dev) if cast else None,
               "mask": torch.empty((c, b), dtype=torch.uint8, device=dev),
               "info": torch.zeros((1,), dtype=torch.int32, device=dev)}
        # a failed factorisation shows in finfo; the sweeps then run on a meaningless factor
        thanos_prune_layer(W, H, o, res["W"], res["W_cast"], res["mask"], ws, res["info"], stream)
        out.append(res)
    return out, H
