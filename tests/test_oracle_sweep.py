"""Pins for the block sweeps of the CPU oracle (no GPU needed)."""
import numpy as np
import pytest

from oracle import thanos_oracle as orc
from synth import LayerSpec, make_weight, make_calibration


def _layer(seed=0, c=24, b=48, T=256, rho=0.7, dtype="f32"):
    spec = LayerSpec("t", c=c, b=b, tokens=T, dtype=dtype, rho=rho, k_mix=8, seed=seed)
    W = make_weight(spec)
    X = make_calibration(spec)
    return W, X, orc.hessian(X)


# ------------------------------------------------------------------ counts
@pytest.mark.parametrize("p,B", [(0.5, 16), (0.6, 16), (0.3, 20), (0.5, 48), (0.5, 100), (0.37, 1)])
def test_unstructured_counts_and_zeros(p, B):
    W, X, H = _layer(1)
    Wh, M = orc.prune_unstructured(W, H, p, B, 0.01)
    c, b = W.shape
    assert int(M.sum()) == int(np.floor(round(p * c * b, 9)))
    assert np.all(Wh[M == 1] == 0.0)
    assert np.all(Wh[M == 0] != 0.0)


@pytest.mark.parametrize("n,m,B", [(2, 4, 16), (4, 8, 16), (1, 4, 8), (2, 4, 48), (2, 4, 20)])
def test_nm_pattern(n, m, B):
    W, X, H = _layer(2)
    Wh, M = orc.prune_nm(W, H, n, m, B, 0.01)
    c, b = W.shape
    assert np.all(M.reshape(c, b // m, m).sum(axis=2) == n)
    assert np.all(Wh[M == 1] == 0.0)


# ------------------------------------------------------------------ special cases
@pytest.mark.parametrize("B", [8, 16, 48, 13])
def test_diagonal_hessian_reduces_to_global_metric_mask(B):
    # With a diagonal Hessian no surviving weight moves, so the block schedule of the
    # global residual mask must reproduce one global psi over the whole layer.
    g = np.random.default_rng(3)
    W = g.standard_normal((10, 48))
    H = np.diag(g.uniform(0.5, 4.0, 48))
    Wh, M = orc.prune_unstructured(W, H, 0.5, B, 0.01)
    M_ref = orc.psi(W, np.diag(H), 240)
    np.testing.assert_array_equal(M, M_ref)
    np.testing.assert_allclose(Wh, W * (1 - M_ref), rtol=0, atol=1e-15)


def test_one_block_is_optimal_reconstruction_for_its_mask():
    # B >= b: a single joint solve per row; the result must be the least-squares optimum
    # over the kept weights for the mask it chose (brute force with lstsq on the
    # damping-augmented X), and cannot be worse than zeroing the same mask.
    W, X, H = _layer(4, c=6, b=20, T=120)
    damp = 0.05
    Wh, M = orc.prune_unstructured(W, H, 0.5, 64, damp)
    lam = damp * np.mean(np.diag(H))
    Xaug = np.vstack([X.astype(np.float64), np.sqrt(lam) * np.eye(20)])
    for i in range(6):
        keep = np.flatnonzero(M[i] == 0)
        target = Xaug @ W[i].astype(np.float64)
        sol, *_ = np.linalg.lstsq(Xaug[:, keep], target, rcond=None)
        np.testing.assert_allclose(Wh[i, keep], sol, rtol=1e-7, atol=1e-10)
    Hd = orc.damped(H, damp)
    assert orc.reconstruction_error(W, Wh, Hd) <= orc.reconstruction_error(W, W * (1 - M), Hd)


def test_block_size_one_is_sequential_obs_with_rank_one_downdates():
    # B = 1: each step removes at most one weight per row with the single-weight OBS
    # rule, and the residual inverse can be reached by the classical elimination
    # Hinv' = (Hinv - Hinv[:,0] Hinv[0,:] / Hinv[0,0])[1:,1:] instead of re-inverting.
    W, X, H = _layer(5, c=8, b=12, T=80)
    n, m = 2, 4
    Wh, M = orc.prune_nm(W, H, n, m, 4, 0.01)          # masks decided per block of 4
    # replay the same mask column by column on a B=1 sweep driven by mask_in
    Wseq = W.astype(np.float64).copy()
    Hinv = np.linalg.inv(orc.damped(H, 0.01))
    W1, M1 = orc.prune_fast(W, H, mode="nm", n=n, m=m, B=1, damp=0.01, mask_in=M)
    for j in range(12):
        for i in range(8):
            if M[i, j]:
                Wseq[i, j:] -= (Wseq[i, j] / Hinv[0, 0]) * Hinv[0, :]
                Wseq[i, j] = 0.0
        Hinv = (Hinv - np.outer(Hinv[:, 0], Hinv[0, :]) / Hinv[0, 0])[1:, 1:]
    np.testing.assert_array_equal(M1, M)
    np.testing.assert_allclose(W1, Wseq, rtol=1e-8, atol=1e-12)


def test_columns_left_of_a_block_are_frozen_and_blocks_see_updated_weights():
    W, X, H = _layer(6, c=8, b=32, T=200)
    Wh, M = orc.prune_nm(W, H, 2, 4, 8, 0.01)
    # n:m decisions of the first block do not depend on later columns of W ...
    W2 = W.copy()
    W2[:, 8:] *= 3.0
    Wh2, M2 = orc.prune_nm(W2, H, 2, 4, 8, 0.01)
    np.testing.assert_array_equal(M[:, :8], M2[:, :8])
    np.testing.assert_allclose(Wh[:, :8], Wh2[:, :8], rtol=1e-12)
    # ... and the second block is decided on the UPDATED weights: its mask differs from
    # the mask of the untouched input somewhere on strongly correlated data.
    M_static = orc.nm_mask(W, np.diag(H), 2, 4)
    assert np.any(M[:, 8:] != M_static[:, 8:])


# ------------------------------------------------------------------ invariances
def test_hessian_scale_invariance():
    W, X, H = _layer(7)
    a = orc.prune_unstructured(W, H, 0.5, 16, 0.01, metric_dtype=np.float64)
    b_ = orc.prune_unstructured(W, 2.0 * H, 0.5, 16, 0.01, metric_dtype=np.float64)
    np.testing.assert_array_equal(a[1], b_[1])
    np.testing.assert_allclose(a[0], b_[0], rtol=1e-9, atol=1e-14)


def test_nm_rows_are_independent():
    W, X, H = _layer(8)
    perm = np.random.default_rng(0).permutation(W.shape[0])
    Wh, M = orc.prune_nm(W, H, 2, 4, 16, 0.01)
    Whp, Mp = orc.prune_nm(W[perm], H, 2, 4, 16, 0.01)
    np.testing.assert_array_equal(Mp, M[perm])
    np.testing.assert_allclose(Whp, Wh[perm], rtol=1e-12)


# ------------------------------------------------------------------ end to end
@pytest.mark.parametrize("mode", ["unstructured", "nm24", "nm48"])
def test_not_worse_than_magnitude_pruning(mode):
    W, X, H = _layer(9, c=48, b=128, T=1024, rho=0.7)
    if mode == "unstructured":
        Wh, M = orc.prune_unstructured(W, H, 0.5, 32, 0.01)
        Wm, _ = orc.magnitude_prune(W, p=0.5)
    else:
        n, m = (2, 4) if mode == "nm24" else (4, 8)
        Wh, M = orc.prune_nm(W, H, n, m, 32, 0.01)
        Wm, _ = orc.magnitude_prune(W, n=n, m=m)
    assert orc.reconstruction_error(W, Wh, H) <= orc.reconstruction_error(W, Wm, H)


# ------------------------------------------------------------------ literal == single factorisation
@pytest.mark.parametrize("c,b,B", [(32, 96, 32), (16, 200, 64), (40, 256, 128)])
def test_fast_equals_literal(c, b, B):
    W, X, H = _layer(10, c=c, b=b, T=4 * b)
    Wl, Ml = orc.prune_unstructured(W, H, 0.5, B, 0.01)
    Wf, Mf = orc.prune_fast(W, H, mode="unstructured", p=0.5, B=B, damp=0.01)
    np.testing.assert_array_equal(Mf, Ml)
    assert np.linalg.norm(Wf - Wl) <= 1e-10 * np.linalg.norm(Wl)
    Wl, Ml = orc.prune_nm(W, H, 2, 4, B, 0.01)
    Wf, Mf = orc.prune_fast(W, H, mode="nm", n=2, m=4, B=B, damp=0.01)
    np.testing.assert_array_equal(Mf, Ml)
    assert np.linalg.norm(Wf - Wl) <= 1e-10 * np.linalg.norm(Wl)


def test_margins_reported():
    W, X, H = _layer(11)
    _, _, mg = orc.prune_unstructured(W, H, 0.5, 16, 0.01, return_margins=True)
    assert mg.shape == (3,) and np.all(mg >= 0)
    _, _, mg = orc.prune_nm(W, H, 2, 4, 16, 0.01, return_margins=True)
    assert mg.shape == (24, 12) and np.all(mg >= 0)
