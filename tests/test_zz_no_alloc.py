"""thanos_prune_layer_noalloc (static device workspace, single stream, no allocation) against
thanos_prune_layer on the same inputs: two calls in a row, the second on a smaller layer, so
that the second call finds the first call's contents in the shared array.

Both entry points run the same kernels on the same numbers; the only difference is the order in
which the wide updates and the chain of short kernels are interleaved, which changes no value.
Bar: masks identical, W_hat bit-identical (asserted as such; the documented bar of 1e-3 relative
Frobenius error is checked as well so that a failure says how far off the result is).
"""
import ctypes

import numpy as np
import pytest

from synth import LayerSpec, make_weight, make_calibration

pytestmark = pytest.mark.gpu


def _inputs(c, b, T, seed):
    import torch
    import paper_2504_05346_amd as th
    spec = LayerSpec("na", c=c, b=b, tokens=T, dtype="f16", rho=0.7, k_mix=16, seed=seed)
    W = torch.from_numpy(make_weight(spec)).cuda()
    X = torch.from_numpy(make_calibration(spec)).cuda()
    H = torch.zeros((b, b), dtype=torch.float32, device="cuda")
    th.thanos_hessian_accumulate(H, X)
    torch.cuda.synchronize()
    return W, H


def _opts(mode, B):
    import paper_2504_05346_amd as th
    if mode == "nm":
        return th.PruneOpts(mode=th.THANOS_NM, sparsity=0.0, n=2, m=4, block_size=B, damping=0.01)
    if mode == "nm_outliers":
        return th.PruneOpts(mode=th.THANOS_NM, sparsity=0.0, n=4, m=8, block_size=B, damping=0.01,
                            outlier_fraction=0.1)
    if mode == "structured":
        return th.PruneOpts(mode=th.THANOS_STRUCTURED, sparsity=0.3, n=0, m=0, block_size=B,
                            damping=0.01, outlier_fraction=0.1)
    return th.PruneOpts(mode=th.THANOS_UNSTRUCTURED, sparsity=0.5, n=0, m=0, block_size=B,
                        damping=0.01)


def _run_both(W, H, o):
    import torch
    import paper_2504_05346_amd as th
    c, b = W.shape
    out = []
    for noalloc in (False, True):
        Wo = torch.empty((c, b), dtype=torch.float32, device="cuda")
        Wc = torch.empty((c, b), dtype=W.dtype, device="cuda")
        M = torch.empty((c, b), dtype=torch.uint8, device="cuda")
        info = torch.full((1,), -7, dtype=torch.int32, device="cuda")
        if noalloc:
            th.thanos_prune_layer_noalloc(W, H, o, Wo, Wc, M, info)
        else:
            ws = torch.empty((th.thanos_prune_workspace_bytes(c, b, o),), dtype=torch.uint8,
                             device="cuda")
            th.thanos_prune_layer(W, H, o, Wo, Wc, M, ws, info)
        torch.cuda.synchronize()
        assert int(info.item()) == 0
        out.append((Wo.cpu().numpy(), Wc.cpu().numpy(), M.cpu().numpy()))
    return out


@pytest.mark.parametrize("mode,B", [("nm", 128), ("unstructured", 128), ("nm_outliers", 64),
                                    ("structured", 128)])
def test_noalloc_matches_prune_layer_twice(mode, B):
    # first call: 1152 columns = 9 blocks of 128 (two super-blocks for n:m); second call smaller
    # (ragged: 200 rows, 392 columns), which leaves most of the first call's workspace in place
    for k, (c, b, T, seed) in enumerate([(384, 1152, 2304, 11), (200, 392, 1024, 12)]):
        print(f"noalloc {mode} B={B} call {k}: {c}x{b}", flush=True)
        W, H = _inputs(c, b, T, seed)
        (Wa, Wca, Ma), (Wb, Wcb, Mb) = _run_both(W, H, _opts(mode, B))
        np.testing.assert_array_equal(Ma, Mb)
        assert np.linalg.norm(Wa.astype(np.float64) - Wb) <= 1e-3 * np.linalg.norm(Wa)
        np.testing.assert_array_equal(Wa, Wb)
        np.testing.assert_array_equal(Wca, Wcb)
        assert Ma.sum() > 0 and np.all(Wb[Mb == 1] == 0.0)


def test_noalloc_rejects_what_does_not_fit():
    import torch
    import paper_2504_05346_amd as th
    L = th.lib()
    c, b = 4096, 4096
    o = _opts("nm", 128)
    assert th.thanos_prune_workspace_bytes(c, b, o) > th.THANOS_NOALLOC_SCRATCH_BYTES
    W = torch.zeros((8, 8), dtype=torch.float16, device="cuda")   # never touched: rejected first
    H = torch.zeros((8, 8), dtype=torch.float32, device="cuda")
    Wo = torch.zeros((8, 8), dtype=torch.float32, device="cuda")
    M = torch.zeros((8, 8), dtype=torch.uint8, device="cuda")
    info = torch.zeros((1,), dtype=torch.int32, device="cuda")
    st = L.thanos_prune_layer_noalloc(W.data_ptr(), th.THANOS_F16, c, b, H.data_ptr(),
                                      ctypes.byref(o), Wo.data_ptr(), None, M.data_ptr(),
                                      info.data_ptr(), None)
    assert st == 6 and "scratch" in th.thanos_status_string(st)
    with pytest.raises(th.ThanosError):
        th.thanos_prune_layer_noalloc(torch.zeros((c, b), dtype=torch.float16, device="cuda"),
                                      torch.zeros((b, b), dtype=torch.float32, device="cuda"), o,
                                      torch.zeros((c, b), dtype=torch.float32, device="cuda"), None,
                                      torch.zeros((c, b), dtype=torch.uint8, device="cuda"), info)
