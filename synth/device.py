"""The recipe of synth.inputs, drawn on the GPU with a seeded torch generator.

For layers whose calibration set is too large to draw on the host in reasonable time
(262144 tokens x 11008 channels = 2.9e9 Gaussians).  Same distributions as synth.inputs, other
random streams: whoever needs the values on the host downloads them from the returned tensors,
so that both sides of a comparison read identical numbers.  Channel scales and the mixing matrix
come from synth.inputs (host, Philox) and are uploaded.

No pruning arithmetic lives in this module.
"""
from __future__ import annotations

import numpy as np

from .inputs import LayerSpec, channel_scales, _mixing


def make_layer_on_device(spec: LayerSpec, torch, device="cuda", chunk_tokens: int = 8192):
    """(W [c, b], X [T, b]) as fp16 tensors on `device`.

    W ~ N(0, w_std^2); X[t, j] = s_j * g[t, j] with g ~ N(0, 1) (rho = 0) or
    g = sqrt(1 - rho^2) e + rho (z A^T), z ~ N(0, I_k), A in R^{b x k} with unit rows (rho > 0).
    """
    assert spec.dtype == "f16"
    gen = torch.Generator(device=device)
    gen.manual_seed(1234 + spec.seed)
    W = (torch.randn((spec.c, spec.b), generator=gen, device=device, dtype=torch.float32)
         * spec.w_std).to(torch.float16)
    s = torch.from_numpy(channel_scales(spec)).to(device=device, dtype=torch.float32)
    A = None
    if spec.rho > 0:
        A = torch.from_numpy(_mixing(spec).astype(np.float32)).to(device)
    X = torch.empty((spec.tokens, spec.b), dtype=torch.float16, device=device)
    for t0 in range(0, spec.tokens, chunk_tokens):
        n = min(chunk_tokens, spec.tokens - t0)
        g = torch.randn((n, spec.b), generator=gen, device=device, dtype=torch.float32)
        if A is not None:
            z = torch.randn((n, spec.k_mix), generator=gen, device=device, dtype=torch.float32)
            g = g * float(np.sqrt(1.0 - spec.rho ** 2)) + float(spec.rho) * (z @ A.T)
        X[t0:t0 + n] = (g * s).to(torch.float16)
    torch.cuda.synchronize()
    return W, X
