"""Thin Python binding of libthanos (HIP, gfx950): argument marshalling only.

Every step of the pruning path runs inside the library's kernels; PyTorch is used
for device memory and streams.  There is no CPU fallback: if the shared library
is missing or a GPU is absent, calls raise.
"""
from .binding import (  # noqa: F401
    lib,
    lib_path,
    ThanosError,
    PruneOpts,
    THANOS_F32, THANOS_F16, THANOS_BF16,
    THANOS_UNSTRUCTURED, THANOS_NM, THANOS_STRUCTURED, THANOS_PHASES,
    thanos_hessian_accumulate,
    thanos_factor,
    thanos_factor_workspace_bytes,
    thanos_prune_layer,
    thanos_prune_layer_noalloc,
    THANOS_NOALLOC_SCRATCH_BYTES,
    thanos_prune_workspace_bytes,
    thanos_status_string,
)
from .layer_set import prune_layer_set  # noqa: F401,E402
