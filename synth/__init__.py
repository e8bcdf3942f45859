"""Seeded synthetic inputs (weights, calibration activations) for layer pruning.

This package holds input generators only: no pruning arithmetic lives here.
It is the one module that both the CPU oracle's tests and the GPU path's
tests / benchmark import, so that both sides consume bit-identical inputs.
"""
from .inputs import (  # noqa: F401
    LayerSpec,
    CONFIGS,
    channel_scales,
    make_weight,
    iter_calibration_chunks,
    make_calibration,
    layer_spec,
)
from .device import make_layer_on_device  # noqa: F401,E402
