"""Helpers shared by the GPU parity tests (allocation and marshalling only)."""
import numpy as np
import torch

import paper_2504_05346_amd as th


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def gpu_hessian(X: np.ndarray, chunks=1, alpha=1.0, ldx=None) -> np.ndarray:
    """Lower triangle of sum-of-chunks Gram matrix from the library; upper part mirrored."""
    T, b = X.shape
    H = torch.zeros((b, b), dtype=torch.float32, device="cuda")
    if X.dtype == np.float16 or X.dtype == np.float32:
        Xd = dev(X)
    else:
        raise TypeError(X.dtype)
    if ldx is not None:
        buf = torch.zeros((T, ldx), dtype=Xd.dtype, device="cuda")
        buf[:, :b] = Xd
        Xd = buf[:, :b]
    edges = np.linspace(0, T, chunks + 1).astype(int)
    for a0, a1 in zip(edges[:-1], edges[1:]):
        th.thanos_hessian_accumulate(H, Xd[a0:a1], alpha)
    torch.cuda.synchronize()
    Hn = H.cpu().numpy().astype(np.float64)
    return np.tril(Hn) + np.tril(Hn, -1).T


def gpu_factor(H32: np.ndarray, damping: float):
    b = H32.shape[0]
    Hd = dev(H32.astype(np.float32))
    U = torch.empty((b, b), dtype=torch.float32, device="cuda")
    xn2 = torch.empty((b,), dtype=torch.float32, device="cuda")
    ws = torch.empty((th.thanos_factor_workspace_bytes(b),), dtype=torch.uint8, device="cuda")
    info = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    th.thanos_factor(Hd, damping, U, xn2, ws, info)
    torch.cuda.synchronize()
    return U.cpu().numpy(), xn2.cpu().numpy(), int(info.item())


def gpu_prune(W: np.ndarray, H32: np.ndarray, *, mode: str, p=0.0, n=0, m=0, B=128, damp=0.01,
              mask_in=None, cast=False, U=None, xnorm2=None, alpha=0.0, tau=False):
    """Run thanos_prune_layer; returns (W_hat fp32, mask uint8, info[, W_cast][, tau per block])."""
    c, b = W.shape
    Wd = dev(W)
    Hd = dev(H32.astype(np.float32)) if H32 is not None else None
    keep = []
    o = th.PruneOpts(mode={"unstructured": th.THANOS_UNSTRUCTURED, "nm": th.THANOS_NM,
                           "structured": th.THANOS_STRUCTURED}[mode],
                     sparsity=float(p), n=n, m=m, block_size=B, damping=damp,
                     outlier_fraction=float(alpha))
    if mask_in is not None:
        md = dev(mask_in.astype(np.uint8))
        keep.append(md)
        o.mask_in = md.data_ptr()
    if U is not None:
        Ud, xd = dev(U.astype(np.float32)), dev(xnorm2.astype(np.float32))
        keep += [Ud, xd]
        o.factor_in, o.xnorm2_in = Ud.data_ptr(), xd.data_ptr()
    tau_d = None
    if tau:
        tau_d = torch.full(((b + B - 1) // B,), -2.0, dtype=torch.float32, device="cuda")
        o.threshold_out = tau_d.data_ptr()
    nbytes = th.thanos_prune_workspace_bytes(c, b, o)
    assert nbytes > 0, "options rejected"
    ws = torch.empty((nbytes,), dtype=torch.uint8, device="cuda")
    Wo = torch.empty((c, b), dtype=torch.float32, device="cuda")
    Wc = torch.empty((c, b), dtype=Wd.dtype, device="cuda") if cast else None
    M = torch.empty((c, b), dtype=torch.uint8, device="cuda")
    info = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    th.thanos_prune_layer(Wd, Hd, o, Wo, Wc, M, ws, info)
    torch.cuda.synchronize()
    out = (Wo.cpu().numpy(), M.cpu().numpy(), int(info.item()))
    if cast:
        out = out + (Wc.cpu().numpy(),)
    if tau:
        out = out + (tau_d.cpu().numpy(),)
    return out
