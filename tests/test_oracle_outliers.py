"""Pins of the oracle's outlier-row step (n:m algorithm of App. G.4.4 with alpha > 0,
Sec. 4.7 "Outlier rows").  CPU only."""
import numpy as np
import pytest

from oracle import thanos_oracle as orc
from synth import LayerSpec, make_calibration, make_weight


def _layer(c=24, b=32, tokens=96, seed=3):
    spec = LayerSpec("t", c=c, b=b, tokens=tokens, dtype="f32", rho=0.7, k_mix=8, seed=seed)
    W = make_weight(spec).astype(np.float64)
    # spread the row norms so that the row losses are well separated
    W *= np.linspace(0.5, 2.0, c)[np.random.default_rng(seed).permutation(c)][:, None]
    X = make_calibration(spec).astype(np.float64)
    return W, X, orc.hessian(X)


def test_row_loss_is_the_output_energy_of_the_row():
    # h_i = ||W_i X||_2^2 with X in R^{b x a}: here X is token-major, so W_i X = X_tm W_i^T
    W, X, H = _layer()
    direct = np.array([np.sum((X @ W[i]) ** 2) for i in range(W.shape[0])])
    np.testing.assert_allclose(orc.row_losses(W, H), direct, rtol=1e-12)


@pytest.mark.parametrize("alpha,c,expect", [(0.1, 1000, 100), (0.1, 4096, 410), (0.5, 7, 4),
                                            (0.0, 5, 0), (0.25, 8, 2), (0.3, 10, 3)])
def test_number_of_outlier_rows_is_the_ceiling(alpha, c, expect):
    assert orc.num_outlier_rows(alpha, c) == expect


def test_outlier_rows_are_the_largest_losses_and_stay_untouched():
    W, X, H = _layer()
    c, b = W.shape
    alpha = 0.3
    n_out = orc.num_outlier_rows(alpha, c)           # ceil(7.2) = 8
    assert n_out == 8
    Wh, M = orc.prune_nm(W, H, 2, 4, 16, 0.01, alpha=alpha)
    h = np.array([np.sum((X @ W[i]) ** 2) for i in range(c)])
    outl = set(np.argsort(h)[-n_out:].tolist())      # brute force: the n_out largest
    for i in range(c):
        if i in outl:
            assert np.array_equal(Wh[i], W[i]) and M[i].sum() == 0
        else:
            assert np.all(M[i].reshape(-1, 4).sum(axis=1) == 2)
            assert np.all(Wh[i][M[i] == 1] == 0.0)
    # total sparsity = n/m * (c - ceil(alpha c)) / c
    assert M.sum() == (c - n_out) * b // 2


def test_pruned_rows_do_not_depend_on_the_outlier_rows():
    # rows are independent in the n:m algorithm: the pruned rows come out exactly as if the
    # outlier rows were not there
    W, X, H = _layer(seed=5)
    rows = orc.pruned_rows(W, H, 0.25)
    Wh, M = orc.prune_nm(W, H, 2, 4, 16, 0.01, alpha=0.25)
    Ws, Ms = orc.prune_nm(W[rows], H, 2, 4, 16, 0.01)
    np.testing.assert_array_equal(M[rows], Ms)
    np.testing.assert_allclose(Wh[rows], Ws, rtol=0, atol=0)


def test_alpha_zero_is_the_plain_algorithm_and_single_factor_sweep_agrees():
    W, X, H = _layer(seed=7)
    W0, M0 = orc.prune_nm(W, H, 2, 4, 16, 0.01)
    W1, M1 = orc.prune_nm(W, H, 2, 4, 16, 0.01, alpha=0)
    assert np.array_equal(M0, M1) and np.array_equal(W0, W1)
    Wn, Mn = orc.prune_nm(W, H, 4, 8, 16, 0.01, alpha=0.2)
    Wf, Mf = orc.prune_fast(W, H, mode="nm", n=4, m=8, B=16, damp=0.01, alpha=0.2)
    assert np.array_equal(Mn, Mf)
    np.testing.assert_allclose(Wf, Wn, rtol=0, atol=1e-10 * np.abs(Wn).max())


def test_ties_in_the_row_loss_go_by_row_index():
    W, X, H = _layer(c=6, b=8, tokens=40)
    W[4] = W[1]                                      # equal losses
    W[5] = 10 * W[0]                                 # clearly the largest
    rows = orc.pruned_rows(W, H, 0.3)                # 2 outliers
    h = orc.row_losses(W, H)
    assert not rows[5]
    # the second outlier is the larger of the remaining rows; among equal losses the later row
    rest = [i for i in range(5)]
    top = max(rest, key=lambda i: (h[i], i))
    assert not rows[top] and rows.sum() == 4
