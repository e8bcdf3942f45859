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


def test_unstructured_later_blocks_rank_the_updated_weights_with_the_reduced_budget():
    """Alg. 1: the global residual mask of block j+1 is psi_X of the weights AFTER block j's row
    updates, with r reduced by ||M||_F^2 of block j.  Replayed by hand for the second and third
    block (psi, one inverse of the residual Hessian and row_update per row, nothing else)."""
    W, X, H = _layer(6, c=8, b=32, T=200)
    p, B, damp = 0.5, 8, 0.01
    Wh, M = orc.prune_unstructured(W, H, p, B, damp)
    xn2 = np.diag(H)
    Hd = orc.damped(H, damp)
    Wcur = W.astype(np.float64).copy()
    r = (8 * 32) // 2
    differs_from_static = False
    for j1 in (0, 8, 16):
        Mb = orc.psi(Wcur[:, j1:], xn2[j1:], r)[:, :B]
        np.testing.assert_array_equal(M[:, j1:j1 + B], Mb)
        if j1 > 0:
            # the same budget on the INPUT weights gives another mask: the ranking did see the updates
            Mstatic = orc.psi(W[:, j1:].astype(np.float64), xn2[j1:], r)[:, :B]
            differs_from_static |= bool(np.any(Mstatic != Mb))
        Hinv = np.linalg.inv(Hd[j1:, j1:])
        for i in range(8):
            Wcur[i, j1:] = orc.row_update(Wcur[i, j1:], Hinv, orc.phi(Mb[i]))
        r -= int(Mb.sum())
        np.testing.assert_allclose(Wh[:, j1:j1 + B], Wcur[:, j1:j1 + B], rtol=1e-12, atol=0)
    assert differs_from_static
    # and a budget that was not reduced would overshoot: the count is exact
    assert int(M.sum()) == (8 * 32) // 2


# ------------------------------------------------------------------ decision margins
def test_global_margin_by_hand():
    """Relative gap between the r-th and (r+1)-th smallest metric of a residual, on a 3 x 8
    example small enough to sort by eye: metric = |W| * sqrt(4) = 2 |W|."""
    W = np.array([[1, -2, 3, -4, 5, -6, 7, -8],
                  [9, 10, -11, 12, 13, -14, 15, 16],
                  [-17, 18, 19, 20, -21, 22, 23, -24]], dtype=np.float64)
    xn2 = np.full(8, 4.0)
    for dt in (np.float32, np.float64):
        # sorted metrics 2, 4, ..., 48: the 5th is 10, the 6th is 12
        assert orc._global_margin(W, xn2, 5, dt) == pytest.approx((12 - 10) / 12, rel=1e-6)
        assert orc._global_margin(W, xn2, 23, dt) == pytest.approx((48 - 46) / 48, rel=1e-6)
        assert orc._global_margin(W, xn2, 0, dt) == float("inf")     # nothing selected
        assert orc._global_margin(W, xn2, 24, dt) == float("inf")    # everything selected
        Wt = W.copy()
        Wt[1, 0] = -5.0                       # planted tie at the cut: 2, 4, 6, 8, 10 | 10, 12
        assert orc._global_margin(Wt, xn2, 5, dt) == 0.0
        assert orc._global_margin(Wt, xn2, 4, dt) == pytest.approx((10 - 8) / 10, rel=1e-6)
        Wg = W.copy()
        Wg[0, 5] = 100.0                      # planted gap: 2, ..., 10 | 14, ... (12 is gone)
        assert orc._global_margin(Wg, xn2, 5, dt) == pytest.approx((14 - 10) / 14, rel=1e-6)
    # the sweep reports the margin of the decision it takes: block 0 on the input weights
    _, _, mg = orc.prune_unstructured(W, np.diag(xn2), 5 / 24, 4, 0.0, return_margins=True)
    assert mg[0] == pytest.approx(1 / 6, rel=1e-6)


def test_group_margins_by_hand():
    """Per row and group of m: relative gap between the n-th and (n+1)-th smallest metric."""
    W = np.array([[1, -2, 3, -4, 8, 6, -7, 5],
                  [3, 1, 1, 2, 1, 2, -2, 3],
                  [10, 0, 0, 20, 1, 1, 1, 1]], dtype=np.float64)
    xn2 = np.full(8, 4.0)
    for dt in (np.float32, np.float64):
        g = orc._group_margins(W, xn2, 2, 4, dt)
        assert g.shape == (3, 2)
        want = np.array([[(6 - 4) / 6, (14 - 12) / 14],      # 2,4|6,8 ; 10,12|14,16
                         [(4 - 2) / 4, 0.0],                 # 2,2|4,6 ; 2,4|4,6: tie at the cut
                         [1.0, 0.0]])                        # 0,0|20,40 ; all equal
        np.testing.assert_allclose(g, want, rtol=1e-6, atol=0)
        g1 = orc._group_margins(W, xn2, 1, 4, dt)
        np.testing.assert_allclose(g1[0], [(4 - 2) / 4, (12 - 10) / 12], rtol=1e-6)
        assert g1[1, 0] == 0.0 and g1[2, 0] == 0.0            # 2|2 ; 0|0 -> tiny denominator, gap 0
    # a decision flips exactly when a perturbation exceeds the margin: scale the 2nd smallest
    # of group (0, 0) past the 3rd and the n:m mask changes, just below it and it does not
    base = orc.nm_mask(W[:1, :4], xn2[:4], 2, 4)
    below, above = W[:1, :4].copy(), W[:1, :4].copy()
    below[0, 1] *= 1 + 0.9 * 0.5              # 4 -> 5.8 < 6: margin relative to the kept value is
    above[0, 1] *= 1 + 1.1 * 0.5              # (6-4)/6, i.e. 0.5 relative to the removed one
    np.testing.assert_array_equal(orc.nm_mask(below, xn2[:4], 2, 4), base)
    assert np.any(orc.nm_mask(above, xn2[:4], 2, 4) != base)


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
