"""Pins of the oracle's structured pruning (Alg. 2, Sec. 4.7).  CPU only."""
import numpy as np
import pytest

from oracle import thanos_oracle as orc
from synth import LayerSpec, make_calibration, make_weight


def _layer(c=20, b=24, tokens=80, seed=2):
    spec = LayerSpec("t", c=c, b=b, tokens=tokens, dtype="f32", rho=0.7, k_mix=8, seed=seed)
    W = make_weight(spec).astype(np.float64)
    rng = np.random.default_rng(seed)
    W *= np.linspace(0.5, 2.0, c)[rng.permutation(c)][:, None]   # separated row losses
    W *= np.linspace(0.6, 1.8, b)[rng.permutation(b)][None, :]   # separated column losses
    X = make_calibration(spec).astype(np.float64)
    return W, X, orc.hessian(X)


@pytest.mark.parametrize("p,alpha,b,expect", [(0.5, 0.0, 100, 50), (0.5, 0.1, 100, 56),
                                              (0.3, 0.1, 768, 256), (0.25, 0.5, 8, 4),
                                              (0.0, 0.2, 10, 0)])
def test_number_of_removed_columns(p, alpha, b, expect):
    assert orc.num_columns_to_remove(p, alpha, b) == expect


def test_column_loss_is_the_energy_of_the_rank_one_terms():
    # v_j = || W_{R,j} (outer) X_j ||_F^2 with X_j the j-th row of X (b x a): here X is
    # token-major, X_j = X[:, j]
    W, X, H = _layer()
    rows = orc.pruned_rows(W, H, 0.2)
    v = orc.column_losses(W, np.diag(H), rows)
    for j in (0, 5, 23):
        direct = np.linalg.norm(np.outer(W[rows, j], X[:, j]), "fro") ** 2
        assert abs(v[j] - direct) <= 1e-12 * direct


def test_structure_of_the_result():
    W, X, H = _layer()
    c, b = W.shape
    p, alpha = 0.4, 0.2
    s = orc.num_columns_to_remove(p, alpha, b)            # ceil(9.6 / 0.8) = 12
    assert s == 12
    Wh, M = orc.prune_structured(W, H, p, alpha, 0.01)
    rows = orc.pruned_rows(W, H, alpha)
    assert rows.sum() == c - 4
    # outlier rows untouched; in the other rows exactly the same s columns are removed
    assert np.array_equal(Wh[~rows], W[~rows]) and M[~rows].sum() == 0
    Q = np.flatnonzero(M[rows][0])
    assert len(Q) == s and np.all(M[rows] == M[rows][0])
    assert np.all(Wh[np.ix_(rows, Q)] == 0.0)
    # Q = the s smallest column losses (brute force from X)
    v = np.array([np.sum(np.outer(W[rows, j], X[:, j]) ** 2) for j in range(b)])
    assert set(Q.tolist()) == set(np.argsort(v)[:s].tolist())
    # overall sparsity reaches p
    assert M.sum() / (c * b) >= p - 1e-12


def test_update_is_the_constrained_least_squares_optimum():
    # for the chosen columns Q the update of every pruned row minimises ||(w_hat - w) X||^2 +
    # damping subject to w_hat[Q] = 0: delta_K = w_Q Hd[Q,K] Hd[K,K]^{-1} on the kept columns K
    W, X, H = _layer(seed=4)
    Wh, M = orc.prune_structured(W, H, 0.5, 0.0, 0.01)
    Hd = orc.damped(H, 0.01)
    Q = np.flatnonzero(M[0])
    K = np.setdiff1d(np.arange(W.shape[1]), Q)
    for i in (0, 7, 19):
        dK = W[i, Q] @ Hd[np.ix_(Q, K)] @ np.linalg.inv(Hd[np.ix_(K, K)])
        np.testing.assert_allclose(Wh[i, K] - W[i, K], dK, rtol=1e-8, atol=1e-12)
        # KKT: gradient of the quadratic vanishes on the kept columns
        d = Wh[i] - W[i]
        assert np.max(np.abs((d @ Hd)[K])) <= 1e-9 * np.max(np.abs(d @ Hd))


def test_equals_the_generic_row_update_with_one_block():
    # Alg. 2 is the row update of Sec. 4.1 with the same q for every row and the inverse of
    # the full Hessian: one block that spans the whole matrix, mask forced
    W, X, H = _layer(seed=6)
    Wh, M = orc.prune_structured(W, H, 0.3, 0.1, 0.01)
    Wf, Mf = orc.prune_fast(W, H, mode="unstructured", p=0.0, B=W.shape[1], damp=0.01, mask_in=M)
    assert np.array_equal(M, Mf)
    np.testing.assert_allclose(Wf, Wh, rtol=0, atol=1e-10 * np.abs(Wh).max())


def test_column_permutation_commutes():
    W, X, H = _layer(seed=8)
    perm = np.random.default_rng(0).permutation(W.shape[1])
    Wh, M = orc.prune_structured(W, H, 0.4, 0.1, 0.01)
    Wp, Mp = orc.prune_structured(W[:, perm], H[np.ix_(perm, perm)], 0.4, 0.1, 0.01)
    assert np.array_equal(Mp, M[:, perm])
    np.testing.assert_allclose(Wp, Wh[:, perm], rtol=0, atol=1e-10 * np.abs(Wh).max())


def test_not_worse_than_dropping_the_columns_without_update():
    W, X, H = _layer(seed=9)
    Wh, M = orc.prune_structured(W, H, 0.5, 0.0, 0.01)
    plain = W * (1 - M)
    assert orc.reconstruction_error(W, Wh, H) <= orc.reconstruction_error(W, plain, H)
