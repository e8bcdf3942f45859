"""ctypes binding of the C ABI declared in include/thanos.h.

The functions here have the names and argument order of the C entry points and do
nothing but marshal arguments: tensors become raw device pointers, the current
torch stream becomes the hipStream_t.  Output tensors and workspaces are torch
tensors the caller (or the small helpers below) allocates.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch  # noqa: F401  (imported first so that the HIP runtime torch ships is the one in use)

THANOS_F32, THANOS_F16, THANOS_BF16 = 0, 1, 2
THANOS_UNSTRUCTURED, THANOS_NM, THANOS_STRUCTURED = 0, 1, 2
THANOS_PHASES = ("prep", "factor", "mask", "solve", "update", "finalise")

_HERE = os.path.dirname(os.path.abspath(__file__))
lib_path = os.path.join(_HERE, "libthanos.so")


class ThanosError(RuntimeError):
    pass


class PruneOpts(ctypes.Structure):
    """Mirror of thanos_prune_opts."""
    _fields_ = [
        ("mode", ctypes.c_int32),
        ("sparsity", ctypes.c_double),
        ("n", ctypes.c_int32),
        ("m", ctypes.c_int32),
        ("block_size", ctypes.c_int32),
        ("damping", ctypes.c_float),
        ("mask_in", ctypes.c_void_p),
        ("factor_in", ctypes.c_void_p),
        ("xnorm2_in", ctypes.c_void_p),
        ("outlier_fraction", ctypes.c_double),
        ("threshold_out", ctypes.c_void_p),
        ("phase_ms_out", ctypes.c_void_p),
    ]


_lib = None


def lib() -> ctypes.CDLL:
    """Load libthanos.so (built by paper_2504_05346_amd.build); raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(lib_path):
        raise ThanosError(
            f"{lib_path} not found: build it with `python -m paper_2504_05346_amd.build` "
            "(there is no CPU fallback)")
    L = ctypes.CDLL(lib_path)
    vp, i64, f32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_float, ctypes.c_size_t
    L.thanos_status_string.restype = ctypes.c_char_p
    L.thanos_status_string.argtypes = [ctypes.c_int]
    L.thanos_hessian_accumulate.restype = ctypes.c_int
    L.thanos_hessian_accumulate.argtypes = [vp, i64, vp, ctypes.c_int, i64, i64, f32, vp]
    L.thanos_factor_workspace_bytes.restype = sz
    L.thanos_factor_workspace_bytes.argtypes = [i64]
    L.thanos_factor.restype = ctypes.c_int
    L.thanos_factor.argtypes = [vp, i64, f32, vp, vp, vp, sz, vp, vp]
    L.thanos_prune_workspace_bytes.restype = sz
    L.thanos_prune_workspace_bytes.argtypes = [i64, i64, ctypes.POINTER(PruneOpts)]
    L.thanos_prune_layer.restype = ctypes.c_int
    L.thanos_prune_layer.argtypes = [vp, ctypes.c_int, i64, i64, vp, ctypes.POINTER(PruneOpts),
                                     vp, vp, vp, vp, sz, vp, vp]
    L.thanos_prune_layer_noalloc.restype = ctypes.c_int
    L.thanos_prune_layer_noalloc.argtypes = [vp, ctypes.c_int, i64, i64, vp,
                                             ctypes.POINTER(PruneOpts), vp, vp, vp, vp, vp]
    _lib = L
    return L


def thanos_status_string(status: int) -> str:
    return lib().thanos_status_string(int(status)).decode()


def _check(status: int, what: str) -> None:
    if status != 0:
        raise ThanosError(f"{what}: {thanos_status_string(status)} (status {status})")


def _dtype_code(t: torch.Tensor) -> int:
    return {torch.float32: THANOS_F32, torch.float16: THANOS_F16,
            torch.bfloat16: THANOS_BF16}[t.dtype]


def _stream(stream) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise ThanosError("device tensor expected")
    return t.data_ptr()


def thanos_hessian_accumulate(H: torch.Tensor, Xc: torch.Tensor, alpha: float = 1.0,
                              stream=None) -> None:
    """H (b x b fp32, lower triangle) += alpha * Xc^T Xc, Xc token-major [n_tok, b]."""
    b = H.shape[0]
    assert H.dtype == torch.float32 and H.is_contiguous() and H.shape == (b, b)
    assert Xc.dim() == 2 and Xc.shape[1] == b and Xc.stride(1) == 1
    st = lib().thanos_hessian_accumulate(_ptr(H), b, _ptr(Xc), _dtype_code(Xc), Xc.shape[0],
                                         Xc.stride(0) if Xc.shape[0] > 1 else b, float(alpha),
                                         _stream(stream))
    _check(st, "thanos_hessian_accumulate")


def thanos_factor_workspace_bytes(b: int) -> int:
    return int(lib().thanos_factor_workspace_bytes(b))


def thanos_factor(H: torch.Tensor, damping: float, U: torch.Tensor, xnorm2: torch.Tensor,
                  ws: torch.Tensor, info: torch.Tensor, stream=None) -> None:
    """U (upper) with inv(H + damping*mean(diag H) I) = U^T U; xnorm2 = diag(H)."""
    b = H.shape[0]
    assert H.dtype == torch.float32 and H.is_contiguous()
    assert U.dtype == torch.float32 and U.is_contiguous() and U.shape == (b, b)
    assert xnorm2.dtype == torch.float32 and xnorm2.numel() == b
    assert info.dtype == torch.int32
    st = lib().thanos_factor(_ptr(H), b, float(damping), _ptr(U), _ptr(xnorm2), _ptr(ws),
                             ws.numel() * ws.element_size(), _ptr(info), _stream(stream))
    _check(st, "thanos_factor")


def thanos_prune_workspace_bytes(c: int, b: int, opts: PruneOpts) -> int:
    return int(lib().thanos_prune_workspace_bytes(c, b, ctypes.byref(opts)))


def thanos_prune_layer(W_in: torch.Tensor, H: Optional[torch.Tensor], opts: PruneOpts,
                       W_out: torch.Tensor, W_out_cast: Optional[torch.Tensor],
                       mask_out: torch.Tensor, ws: torch.Tensor, info: torch.Tensor,
                       stream=None) -> None:
    """Block sweep on W_in (c x b); writes W_out (fp32), optional cast copy, mask (uint8)."""
    c, b = W_in.shape
    assert W_in.is_contiguous() and W_out.is_contiguous() and mask_out.is_contiguous()
    assert W_out.dtype == torch.float32 and W_out.shape == (c, b)
    assert mask_out.dtype == torch.uint8 and mask_out.shape == (c, b)
    if W_out_cast is not None:
        assert W_out_cast.dtype == W_in.dtype and W_out_cast.shape == (c, b)
    st = lib().thanos_prune_layer(_ptr(W_in), _dtype_code(W_in), c, b, _ptr(H),
                                  ctypes.byref(opts), _ptr(W_out), _ptr(W_out_cast),
                                  _ptr(mask_out), _ptr(ws), ws.numel() * ws.element_size(),
                                  _ptr(info), _stream(stream))
    _check(st, "thanos_prune_layer")


THANOS_NOALLOC_SCRATCH_BYTES = 64 << 20


def thanos_prune_layer_noalloc(W_in: torch.Tensor, H: Optional[torch.Tensor], opts: PruneOpts,
                               W_out: torch.Tensor, W_out_cast: Optional[torch.Tensor],
                               mask_out: torch.Tensor, info: torch.Tensor, stream=None) -> None:
    """thanos_prune_layer with the library's static device workspace (no ws argument)."""
    c, b = W_in.shape
    assert W_in.is_contiguous() and W_out.is_contiguous() and mask_out.is_contiguous()
    assert W_out.dtype == torch.float32 and W_out.shape == (c, b)
    assert mask_out.dtype == torch.uint8 and mask_out.shape == (c, b)
    if W_out_cast is not None:
        assert W_out_cast.dtype == W_in.dtype and W_out_cast.shape == (c, b)
    st = lib().thanos_prune_layer_noalloc(_ptr(W_in), _dtype_code(W_in), c, b, _ptr(H),
                                          ctypes.byref(opts), _ptr(W_out), _ptr(W_out_cast),
                                          _ptr(mask_out), _ptr(info), _stream(stream))
    _check(st, "thanos_prune_layer_noalloc")
