"""One layer of each of the other benchmark configurations at its own size (262144 calibration
tokens), GPU against the oracle:
  * configuration 2: 768 x 768 and 3072 x 768, 50 % unstructured, B = 128 -- small enough for the
    LITERAL oracle (residual Hessian re-inverted at every block) on the whole layer;
  * configuration 4: 5120 x 5120, 4:8, heavy-tailed activations, B = 128 -- sampled rows;
  * configuration 5: 8192 x 8192, 60 % unstructured, B = 256, N(0, 0.015^2) weights, outlier
    channels -- sampled rows against the per-block thresholds the GPU reports.
Each on the configured (independent) channels and on the correlated variant.  Also the two
"next" variants at a benchmark size: 4:8 with outlier rows (5120 x 5120) and structured pruning
(Alg. 2, 4096 x 4096).
"""
import types

import numpy as np
import pytest

from oracle import thanos_oracle as orc
from synth import LayerSpec, make_layer_on_device
from tests.fullsize_util import sample_rows, check_nm_rows, check_unstructured_rows, per_row_checks

pytestmark = pytest.mark.gpu

T, DAMP = 262144, 0.01


def _device_layer(c, b, rho, outliers=False, w_std=0.02, seed=3):
    import torch
    import paper_2504_05346_amd as th
    spec = LayerSpec("cfg", c=c, b=b, tokens=T, dtype="f16", rho=rho, outliers=outliers,
                     w_std=w_std, seed=seed)
    W, X = make_layer_on_device(spec, torch)
    H = torch.zeros((b, b), dtype=torch.float32, device="cuda")
    th.thanos_hessian_accumulate(H, X)
    torch.cuda.synchronize()
    return W, X, H


def _sym64(H):
    Hl = H.cpu().numpy().astype(np.float64)
    return np.tril(Hl) + np.tril(Hl, -1).T


def _prune(W, H, mode, block, p=0.5, n=0, m=0, alpha=0.0):
    import torch
    import paper_2504_05346_amd as th
    c, b = W.shape
    tau = torch.full(((b + block - 1) // block,), -2.0, dtype=torch.float32, device="cuda")
    o = th.PruneOpts(mode=th.THANOS_NM if mode == "nm" else th.THANOS_UNSTRUCTURED, sparsity=p,
                     n=n, m=m, block_size=block, damping=DAMP, outlier_fraction=alpha)
    if mode != "nm":
        o.threshold_out = tau.data_ptr()
    ws = torch.empty((th.thanos_prune_workspace_bytes(c, b, o),), dtype=torch.uint8, device="cuda")
    Wo = torch.empty((c, b), dtype=torch.float32, device="cuda")
    M = torch.empty((c, b), dtype=torch.uint8, device="cuda")
    info = torch.zeros((1,), dtype=torch.int32, device="cuda")
    th.thanos_prune_layer(W, H, o, Wo, None, M, ws, info)
    torch.cuda.synchronize()
    assert int(info.item()) == 0
    return Wo, M, tau.cpu().numpy()


@pytest.mark.parametrize("c,b", [(768, 768), (3072, 768)])
@pytest.mark.parametrize("rho", [0.0, 0.7])
def test_cfg2_whole_layer_against_the_literal_oracle(c, b, rho):
    print(f"configuration 2: {c}x{b}, rho={rho}", flush=True)
    W, X, H = _device_layer(c, b, rho)
    # the Hessian of all 262144 tokens against the float64 Gram matrix of the same fp16 values
    Href = orc.hessian(X.cpu().numpy())
    Hg = _sym64(H)
    assert np.linalg.norm(Hg - Href) <= 1e-5 * np.linalg.norm(Href)
    del X
    Wo, M, tau = _prune(W, H, "unstructured", 128)
    Wg, Mg = Wo.cpu().numpy().astype(np.float64), M.cpu().numpy()
    Wh = W.cpu().numpy()
    r = orc.num_to_remove(0.5, c, b)
    assert int(Mg.sum()) == r and np.all(Wg[Mg == 1] == 0.0)
    # literal Alg. 1 on the whole layer, on the Hessian the GPU built (both sides then decide on
    # the same numbers in the first block)
    Wl, Ml, margins = orc.prune_unstructured(Wh, Hg, 0.5, 128, DAMP, return_margins=True)
    ndiff = int((Mg != Ml).sum())
    print(f"  masks differ at {ndiff} of {c * b} positions; oracle margins per block "
          f"{np.array2string(margins, precision=1)}", flush=True)
    # fp16 weights: equal metrics inside a column are common in the first block and are ranked
    # identically on both sides; later blocks can differ at near-ties only
    np.testing.assert_array_equal(Mg[:, :128], Ml[:, :128])
    assert ndiff <= max(4, 2e-5 * c * b)
    check_unstructured_rows(Wh, Hg, orc.inverse_factor(orc.damped(Hg, DAMP)), Wg, Mg, tau, 0.5,
                            128, DAMP, f"cfg2 {c}x{b} rho={rho}")
    if ndiff == 0:
        assert np.linalg.norm(Wg - Wl) <= 1e-3 * np.linalg.norm(Wl)
    eo = orc.reconstruction_error(Wh, Wl, Hg)
    eg = orc.reconstruction_error(Wh, Wg, Hg)
    assert abs(eg - eo) <= 0.01 * eo
    Wm, _ = orc.magnitude_prune(Wh, p=0.5)
    assert eg <= orc.reconstruction_error(Wh, Wm, Hg)


@pytest.mark.parametrize("rho", [0.0, 0.7])
def test_cfg4_5120_heavy_tailed_4of8(rho):
    c = b = 5120
    print(f"configuration 4: {c}x{b} 4:8, heavy-tailed, rho={rho}", flush=True)
    W, X, H = _device_layer(c, b, rho, outliers=True)
    del X
    Wo, M, _ = _prune(W, H, "nm", 128, n=4, m=8)
    assert bool((M.view(c, b // 8, 8).sum(dim=2) == 4).all())
    assert float(Wo[M == 1].abs().max()) == 0.0
    Hg = _sym64(H)
    U = orc.inverse_factor(orc.damped(Hg, DAMP))
    rows = sample_rows(c, 64, seed=4)
    check_nm_rows(W[rows.tolist()].cpu().numpy(), Hg, U,
                  Wo[rows.tolist()].cpu().numpy().astype(np.float64),
                  M[rows.tolist()].cpu().numpy(), 4, 8, 128, DAMP, f"cfg4 5120x5120 4:8 rho={rho}")


def test_cfg4_5120_4of8_with_outlier_rows():
    """The n:m algorithm with outlier rows (App. G.4.4, alpha = 0.1) at the size of configuration
    4: the ceil(alpha c) rows of largest loss h_i = ||W_i X||^2 stay untouched, the others are
    pruned 4:8 as before."""
    c = b = 5120
    alpha = 0.1
    print(f"configuration 4: {c}x{b} 4:8 with {alpha} outlier rows", flush=True)
    W, X, H = _device_layer(c, b, 0.7, outliers=True)
    del X
    Wo, M, _ = _prune(W, H, "nm", 128, n=4, m=8, alpha=alpha)
    Hg = _sym64(H)
    Wh = W.cpu().numpy()
    Mg = M.cpu().numpy()
    n_out = orc.num_outlier_rows(alpha, c)
    kept_g = ~Mg.any(axis=1)                       # rows the GPU left alone
    assert int(kept_g.sum()) == n_out == 512
    # the same rows as the oracle's ranking of the row losses, unless the cut is a near-tie
    h = orc.row_losses(Wh, Hg)
    pruned_o = orc.pruned_rows(Wh, Hg, alpha)
    hs = np.sort(h)
    gap = (hs[c - n_out] - hs[c - n_out - 1]) / hs[c - n_out]
    print(f"  row-loss gap at the cut {gap:.2e}", flush=True)
    if gap > 1e-5:
        np.testing.assert_array_equal(kept_g, ~pruned_o)
    else:                                          # either side of a near-tie is acceptable
        wrong = np.flatnonzero(kept_g != ~pruned_o)
        assert len(wrong) <= 2 and np.all(np.abs(h[wrong] - hs[c - n_out]) <= 1e-5 * hs[c - n_out])
    # untouched rows: bit-identical to the input, nothing masked
    kept_idx = np.flatnonzero(kept_g)
    np.testing.assert_array_equal(Wo[kept_idx.tolist()].cpu().numpy(),
                                  Wh[kept_idx].astype(np.float32))
    # pruned rows: 4 of every 8, exact zeros, sampled rows against the oracle
    pr = np.flatnonzero(~kept_g)
    assert bool((M[pr.tolist()].view(len(pr), b // 8, 8).sum(dim=2) == 4).all())
    assert float(Wo[M == 1].abs().max()) == 0.0
    U = orc.inverse_factor(orc.damped(Hg, DAMP))
    rows = pr[sample_rows(len(pr), 48, seed=6)]
    check_nm_rows(Wh[rows], Hg, U, Wo[rows.tolist()].cpu().numpy().astype(np.float64), Mg[rows],
                  4, 8, 128, DAMP, "cfg4 5120x5120 4:8 alpha=0.1")


@pytest.mark.parametrize("rho", [0.0, 0.7])
def test_cfg5_8192_block256_60pct(rho):
    c = b = 8192
    print(f"configuration 5: {c}x{b} 60 % unstructured, B = 256, rho={rho}", flush=True)
    W, X, H = _device_layer(c, b, rho, outliers=True, w_std=0.015)
    del X
    Wo, M, tau = _prune(W, H, "unstructured", 256, p=0.6)
    assert int(M.sum().item()) == orc.num_to_remove(0.6, c, b)
    assert float(Wo[M == 1].abs().max()) == 0.0
    Hg = _sym64(H)
    U = orc.inverse_factor(orc.damped(Hg, DAMP))
    rows = sample_rows(c, 48, seed=5)
    check_unstructured_rows(W[rows.tolist()].cpu().numpy(), Hg, U,
                            Wo[rows.tolist()].cpu().numpy().astype(np.float64),
                            M[rows.tolist()].cpu().numpy(), tau, 0.6, 256, DAMP,
                            f"cfg5 8192x8192 60 % B=256 rho={rho}")


def test_structured_4096_with_outlier_rows():
    """Alg. 2 (structured pruning with outlier rows) on a 4096 x 4096 layer with 262144
    calibration tokens: p = 0.3, alpha = 0.1, i.e. s = ceil(p b / (1 - alpha)) = 1366 columns
    leave the 3686 rows of smallest loss, in one shot."""
    import torch
    import paper_2504_05346_amd as th
    c = b = 4096
    p, alpha = 0.3, 0.1
    print(f"structured {c}x{b}, p={p}, alpha={alpha}", flush=True)
    W, X, H = _device_layer(c, b, 0.7, seed=8)
    del X
    o = th.PruneOpts(mode=th.THANOS_STRUCTURED, sparsity=p, damping=DAMP, outlier_fraction=alpha)
    ws = torch.empty((th.thanos_prune_workspace_bytes(c, b, o),), dtype=torch.uint8, device="cuda")
    Wo = torch.empty((c, b), dtype=torch.float32, device="cuda")
    M = torch.empty((c, b), dtype=torch.uint8, device="cuda")
    info = torch.zeros((1,), dtype=torch.int32, device="cuda")
    th.thanos_prune_layer(W, H, o, Wo, None, M, ws, info)
    torch.cuda.synchronize()
    assert int(info.item()) == 0
    Hg = _sym64(H)
    Wh = W.cpu().numpy()
    Wg, Mg = Wo.cpu().numpy().astype(np.float64), M.cpu().numpy()
    s_cols = orc.num_columns_to_remove(p, alpha, b)
    n_out = orc.num_outlier_rows(alpha, c)
    assert s_cols == 1366 and n_out == 410
    # gaps of the oracle's two rankings at their cuts
    rows_o = orc.pruned_rows(Wh, Hg, alpha)
    hs = np.sort(orc.row_losses(Wh, Hg))
    vs = np.sort(orc.column_losses(Wh.astype(np.float64), np.diag(Hg), rows_o))
    gap_r = (hs[c - n_out] - hs[c - n_out - 1]) / hs[c - n_out]
    gap_c = (vs[s_cols] - vs[s_cols - 1]) / vs[s_cols]
    print(f"  gaps at the cuts: rows {gap_r:.2e}, columns {gap_c:.2e}", flush=True)
    Wt, Mt = orc.prune_structured(Wh, Hg, p, alpha, DAMP)
    assert int(Mg.sum()) == int(Mt.sum()) == s_cols * (c - n_out)
    assert np.all(Wg[Mg == 1] == 0.0)
    if not np.array_equal(Mg, Mt):
        assert min(gap_r, gap_c) < 1e-5, "structured masks differ without a near-tie at a cut"
        pytest.skip("near-tie at a cut of the structured ranking: W_hat not compared")
    np.testing.assert_array_equal(Wg[~rows_o], Wh[~rows_o].astype(np.float64))
    assert np.linalg.norm(Wg - Wt) <= 1e-3 * np.linalg.norm(Wt)
    eo = orc.reconstruction_error(Wh, Wt, Hg)
    eg = orc.reconstruction_error(Wh, Wg, Hg)
    assert abs(eg - eo) <= 0.01 * eo
