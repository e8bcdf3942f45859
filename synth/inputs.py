"""Seeded synthetic layers: weights W [c, b] and calibration activations X [T, b].

Stand-ins for the OPT / LLaMA linear layers and the calibration activations
the method is evaluated on: only shapes and rough statistics are modelled.

Recipe
------
* W[i, j] ~ N(0, w_std^2), stored in the layer's dtype (fp16 or fp32).
* X is token-major, X[t, j] = s_j * g[t, j] with g ~ N(0, 1) and a per-channel
  scale s_j ~ LogNormal(0, 0.5).  With ``outliers=True`` 0.5 % of the channels
  get an extra factor U(20, 100) (heavy-tailed activations).
* ``rho > 0`` gives the correlated variant
  g = sqrt(1 - rho^2) * e + rho * (z @ A^T), e ~ N(0, I_b), z ~ N(0, I_k),
  A in R^{b x k} with unit-norm rows, so that the Gram matrix is far from
  diagonal and the weight update of the pruning method is not negligible.

All streams are counter-based (numpy Philox) and keyed by
(seed, tensor id, chunk index): a chunk of X can be regenerated on its own,
and the host oracle and the GPU path read bit-identical arrays.

No pruning arithmetic lives in this module.
"""
from __future__ import annotations

import dataclasses
from typing import Iterator, Tuple

import numpy as np

_TENSOR_W = 1
_TENSOR_SCALE = 2
_TENSOR_MIX = 3
_TENSOR_X = 4
_TENSOR_OUTLIER = 5


@dataclasses.dataclass(frozen=True)
class LayerSpec:
    """One linear layer to prune and its calibration set."""

    name: str
    c: int                  # output rows of W
    b: int                  # input columns of W == channels of X
    tokens: int             # T, calibration tokens
    dtype: str              # "f16" | "f32" (storage type of W and X)
    w_std: float = 0.02
    outliers: bool = False  # heavy-tailed channel scales
    rho: float = 0.0        # 0: independent channels, >0: correlated variant
    k_mix: int = 32         # rank of the correlated component
    seed: int = 0

    def replace(self, **kw) -> "LayerSpec":
        return dataclasses.replace(self, **kw)


def _np_dtype(dtype: str):
    return {"f16": np.float16, "f32": np.float32}[dtype]


def _rng(seed: int, tensor: int, chunk: int = 0) -> np.random.Generator:
    # Philox takes a 2-word key here; (seed, tensor id) fill it, and the chunk
    # index offsets the counter space through a jump, so chunks are independent.
    bitgen = np.random.Philox(key=[np.uint64(seed), np.uint64(tensor)])
    if chunk:
        bitgen = bitgen.jumped(chunk)
    return np.random.Generator(bitgen)


def channel_scales(spec: LayerSpec) -> np.ndarray:
    """Per-channel activation scale s_j (float64, length b)."""
    s = np.exp(0.5 * _rng(spec.seed, _TENSOR_SCALE).standard_normal(spec.b))
    if spec.outliers:
        g = _rng(spec.seed, _TENSOR_OUTLIER)
        n_out = max(1, int(round(0.005 * spec.b)))
        idx = g.choice(spec.b, size=n_out, replace=False)
        s[idx] *= g.uniform(20.0, 100.0, size=n_out)
        # keep 6 sigma inside the fp16 range
        s = np.minimum(s, 65504.0 / 6.0)
    return s


def _mixing(spec: LayerSpec) -> np.ndarray:
    a = _rng(spec.seed, _TENSOR_MIX).standard_normal((spec.b, spec.k_mix))
    a /= np.linalg.norm(a, axis=1, keepdims=True)
    return a


def make_weight(spec: LayerSpec) -> np.ndarray:
    """W [c, b] in the layer's storage dtype."""
    w = _rng(spec.seed, _TENSOR_W).standard_normal((spec.c, spec.b), dtype=np.float32)
    w *= np.float32(spec.w_std)
    return w.astype(_np_dtype(spec.dtype))


def iter_calibration_chunks(spec: LayerSpec, chunk_tokens: int = 8192
                            ) -> Iterator[Tuple[int, np.ndarray]]:
    """Yield (first token index, X chunk [n, b]) in the layer's storage dtype."""
    s = channel_scales(spec).astype(np.float32)
    a = _mixing(spec).astype(np.float32) if spec.rho > 0 else None
    t0 = 0
    chunk = 0
    while t0 < spec.tokens:
        n = min(chunk_tokens, spec.tokens - t0)
        g = _rng(spec.seed, _TENSOR_X, chunk + 1)
        e = g.standard_normal((n, spec.b), dtype=np.float32)
        if a is not None:
            z = g.standard_normal((n, spec.k_mix), dtype=np.float32)
            e *= np.float32(np.sqrt(1.0 - spec.rho ** 2))
            e += np.float32(spec.rho) * (z @ a.T)
        e *= s[None, :]
        yield t0, e.astype(_np_dtype(spec.dtype))
        t0 += n
        chunk += 1


def make_calibration(spec: LayerSpec, chunk_tokens: int = 8192) -> np.ndarray:
    """Whole X [T, b]; only for sizes that fit host memory comfortably."""
    out = np.empty((spec.tokens, spec.b), dtype=_np_dtype(spec.dtype))
    for t0, x in iter_calibration_chunks(spec, chunk_tokens):
        out[t0:t0 + x.shape[0]] = x
    return out


# Layer sets of the benchmark configurations.  Index = configuration number.
CONFIGS = {
    1: dict(tokens=2048, dtype="f32", w_std=0.02, outliers=False,
            layers=[("512x512", 512, 512)],
            prune=dict(mode="unstructured", sparsity=0.5, block=128)),
    2: dict(tokens=262144, dtype="f16", w_std=0.02, outliers=False,
            layers=[("768x768", 768, 768), ("3072x768", 3072, 768), ("768x3072", 768, 3072)],
            prune=dict(mode="unstructured", sparsity=0.5, block=128)),
    3: dict(tokens=262144, dtype="f16", w_std=0.02, outliers=False,
            layers=[("4096x4096", 4096, 4096), ("11008x4096", 11008, 4096),
                    ("4096x11008", 4096, 11008)],
            prune=dict(mode="nm", n=2, m=4, block=128)),
    4: dict(tokens=262144, dtype="f16", w_std=0.02, outliers=True,
            layers=[("5120x5120", 5120, 5120), ("13824x5120", 13824, 5120),
                    ("5120x13824", 5120, 13824)],
            prune=dict(mode="nm", n=4, m=8, block=128)),
    5: dict(tokens=262144, dtype="f16", w_std=0.015, outliers=True,
            layers=[("8192x8192", 8192, 8192), ("28672x8192", 28672, 8192),
                    ("8192x28672", 8192, 28672)],
            prune=dict(mode="unstructured", sparsity=0.6, block=256)),
}


def layer_spec(config: int, layer: str, *, rho: float = 0.0, seed: int = 0,
               tokens: int | None = None) -> LayerSpec:
    """LayerSpec of a named layer of a benchmark configuration."""
    cfg = CONFIGS[config]
    for name, c, b in cfg["layers"]:
        if name == layer:
            return LayerSpec(name=f"cfg{config}/{name}", c=c, b=b,
                             tokens=cfg["tokens"] if tokens is None else tokens,
                             dtype=cfg["dtype"], w_std=cfg["w_std"],
                             outliers=cfg["outliers"], rho=rho, seed=seed)
    raise KeyError(f"no layer {layer!r} in config {config}")
