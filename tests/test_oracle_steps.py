"""Pins for the step-level functions of the CPU oracle (no GPU needed).

Each test checks the oracle against something other than itself: values the
paper prints, a closed form, a brute-force least-squares solution, a library
routine reached by a different route, or an invariant of the mathematics.
"""
import json
import os

import numpy as np
import pytest

from oracle import thanos_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rng(seed):
    return np.random.default_rng(seed)


def _spd_problem(seed, b, T=None, damp=0.01):
    """Correlated token-major X [T, b], its Gram matrix, damped copy."""
    g = _rng(seed)
    T = T or 4 * b
    X = g.standard_normal((T, b)) @ (np.eye(b) + 0.3 * g.standard_normal((b, b)))
    H = X.T @ X
    return X, H, orc.damped(H, damp)


# ---------------------------------------------------------------- paper examples
def test_psi_paper_example():
    ex = json.load(open(os.path.join(GOLDEN, "psi_example.json")))
    W = np.array(ex["W"], dtype=np.float64)
    Xcs = np.array(ex["X_channels_by_samples"], dtype=np.float64)   # b x a as in the paper
    H = orc.hessian(Xcs.T)                                          # oracle takes token-major
    xn2 = np.diag(H)
    np.testing.assert_array_equal(orc.metric(W, xn2, np.float64), np.array(ex["metric"], float))
    np.testing.assert_array_equal(orc.metric(W, xn2, np.float32), np.array(ex["metric"], np.float32))
    for r in (1, 2, 4):
        np.testing.assert_array_equal(orc.psi(W, xn2, r), np.array(ex[f"psi_{r}"], np.uint8))
    assert orc.psi(W, xn2, 0).sum() == 0
    assert orc.psi(W, xn2, 6).sum() == 6


def test_phi_paper_example():
    ex = json.load(open(os.path.join(GOLDEN, "phi_example.json")))
    for case in ex["cases"]:
        np.testing.assert_array_equal(orc.phi(np.array(case["x"])) + 1, case["phi_one_based"])


# ---------------------------------------------------------------- Hessian
def test_hessian_is_gram_matrix_bruteforce():
    g = _rng(0)
    X = g.standard_normal((37, 5)).astype(np.float16)       # exact conversion to float64
    H = orc.hessian(X, chunk=8)                              # several ragged chunks
    ref = np.zeros((5, 5))
    for t in range(37):
        for i in range(5):
            for j in range(5):
                ref[i, j] += float(X[t, i]) * float(X[t, j])
    np.testing.assert_allclose(H, ref, rtol=1e-14, atol=0)
    np.testing.assert_array_equal(H, H.T)
    assert np.all(np.linalg.eigvalsh(H) > -1e-9)
    np.testing.assert_allclose(np.diag(H), (X.astype(np.float64) ** 2).sum(0), rtol=1e-14)


def test_metric_is_loss_of_plain_removal():
    # App. G.3: removing W_kq with no compensation costs w_q^2 ||X_q:||^2 = ||delta X||^2
    g = _rng(1)
    X = g.standard_normal((50, 7))
    H = orc.hessian(X)
    W = g.standard_normal((3, 7))
    mu = orc.metric(W, np.diag(H), np.float64)
    for k in range(3):
        for q in range(7):
            d = np.zeros(7)
            d[q] = -W[k, q]
            np.testing.assert_allclose(mu[k, q] ** 2, np.sum((d @ X.T) ** 2), rtol=1e-12)


def test_damped():
    H = np.diag([1.0, 2.0, 3.0]) + 0.1
    Hd = orc.damped(H, 0.5)
    lam = 0.5 * np.mean([1.1, 2.1, 3.1])
    np.testing.assert_allclose(Hd, H + lam * np.eye(3), rtol=1e-15)
    assert H[0, 0] == 1.1    # input not modified


def test_num_to_remove_exact():
    assert orc.num_to_remove(0.6, 2, 5) == 6          # float 0.6*10 = 5.999999...
    assert orc.num_to_remove(0.5, 3, 3) == 4
    assert orc.num_to_remove(0.6, 8192, 8192) == 40265318
    assert orc.num_to_remove(0.0, 10, 10) == 0


# ---------------------------------------------------------------- row update
def test_row_update_single_weight_is_closed_form_obs():
    # eq. (OBS solution): Delta = -(w_q / Hinv_qq) Hinv_q:
    _, _, Hd = _spd_problem(2, 9)
    Hinv = np.linalg.inv(Hd)
    w = _rng(3).standard_normal(9)
    for q in (0, 4, 8):
        got = orc.row_update(w, Hinv, np.array([q]))
        want = w - (w[q] / Hinv[q, q]) * Hinv[q, :]
        want[q] = 0.0
        np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-14)
        # loss of the removal, S = w_q^2 / (2 Hinv_qq)
        d = got - w
        np.testing.assert_allclose(0.5 * d @ Hd @ d, 0.5 * w[q] ** 2 / Hinv[q, q], rtol=1e-10)


@pytest.mark.parametrize("seed,b,s", [(5, 12, 1), (6, 12, 4), (7, 16, 9), (8, 10, 10)])
def test_row_update_is_constrained_least_squares(seed, b, s):
    # The update must minimise ||delta X_aug||^2 subject to delta_q = -w_q, where
    # X_aug stacks X and sqrt(lambda) I (so that X_aug^T X_aug is the damped Hessian).
    g = _rng(seed)
    X, H, Hd = _spd_problem(seed, b)
    lam = Hd[0, 0] - H[0, 0]
    Xaug = np.vstack([X, np.sqrt(lam) * np.eye(b)])
    w = g.standard_normal(b)
    q = np.sort(g.choice(b, size=s, replace=False))
    keep = np.setdiff1d(np.arange(b), q)
    got = orc.row_update(w, np.linalg.inv(Hd), q)
    delta = got - w
    np.testing.assert_array_equal(got[q], 0.0)
    if len(keep):
        # brute force: least squares over the free coordinates
        rhs = Xaug[:, q] @ w[q]
        d_keep, *_ = np.linalg.lstsq(Xaug[:, keep], rhs, rcond=None)
        np.testing.assert_allclose(delta[keep], d_keep, rtol=1e-8, atol=1e-10)
        # KKT: gradient vanishes on the free coordinates
        grad = Hd @ delta
        assert np.max(np.abs(grad[keep])) <= 1e-9 * np.max(np.abs(grad))
    # loss identity: 1/2 delta Hd delta^T = 1/2 u Rhat^{-1} u^T
    Hinv = np.linalg.inv(Hd)
    u = w[q]
    np.testing.assert_allclose(0.5 * delta @ Hd @ delta,
                               0.5 * u @ np.linalg.solve(Hinv[np.ix_(q, q)], u), rtol=1e-9)


def test_row_update_beats_any_feasible_perturbation():
    g = _rng(11)
    _, _, Hd = _spd_problem(11, 14)
    w = g.standard_normal(14)
    q = np.array([1, 5, 6, 12])
    best = orc.row_update(w, np.linalg.inv(Hd), q) - w
    f_best = best @ Hd @ best
    for _ in range(50):
        d = best + 0.1 * g.standard_normal(14)
        d[q] = -w[q]
        assert d @ Hd @ d >= f_best


def test_row_update_empty_and_uses_rows_of_inverse():
    _, _, Hd = _spd_problem(12, 6)
    Hinv = np.linalg.inv(Hd)
    w = np.arange(6, dtype=float) + 1
    np.testing.assert_array_equal(orc.row_update(w, Hinv, np.array([], dtype=int)), w)
    # a non-symmetric "Hinv" exposes a transposed R (rows, not columns, are gathered)
    A = Hinv + np.triu(np.ones((6, 6)), 1) * 0.01
    q = np.array([2, 3])
    got = orc.row_update(w, A, q)
    R = A[q, :]
    lam = w[q] @ np.linalg.inv(R[:, q])
    want = w - lam @ R
    want[q] = 0
    np.testing.assert_allclose(got, want, rtol=1e-12)


# ---------------------------------------------------------------- n:m mask
def test_nm_mask_bruteforce():
    g = _rng(13)
    W = g.standard_normal((5, 16))
    xn2 = g.uniform(0.5, 2.0, 16)
    for n, m in ((2, 4), (4, 8), (1, 4), (3, 4)):
        M = orc.nm_mask(W, xn2, n, m, np.float64)
        mu = np.abs(W) * np.sqrt(xn2)
        for i in range(5):
            for g0 in range(0, 16, m):
                grp = mu[i, g0:g0 + m]
                want = np.zeros(m, np.uint8)
                want[sorted(range(m), key=lambda k: (grp[k], k))[:n]] = 1
                np.testing.assert_array_equal(M[i, g0:g0 + m], want)


def test_tie_break_is_row_major():
    W = np.ones((2, 4))
    xn2 = np.ones(4)
    np.testing.assert_array_equal(orc.psi(W, xn2, 5), [[1, 1, 1, 1], [1, 0, 0, 0]])
    np.testing.assert_array_equal(orc.nm_mask(W, xn2, 2, 4), [[1, 1, 0, 0], [1, 1, 0, 0]])


def test_inverse_factor_gives_every_residual_inverse():
    _, _, Hd = _spd_problem(14, 24)
    U = orc.inverse_factor(Hd)
    assert np.allclose(U, np.triu(U))
    for j in (0, 1, 7, 16, 23):
        np.testing.assert_allclose(U[j:, j:].T @ U[j:, j:], np.linalg.inv(Hd[j:, j:]),
                                   rtol=1e-8, atol=1e-12)


def test_reconstruction_error_definition():
    g = _rng(15)
    X = g.standard_normal((40, 6))
    W = g.standard_normal((3, 6))
    Wh = W + 0.1 * g.standard_normal((3, 6))
    np.testing.assert_allclose(orc.reconstruction_error(W, Wh, orc.hessian(X)),
                               np.sum(((Wh - W) @ X.T) ** 2), rtol=1e-12)


def test_magnitude_prune():
    W = np.array([[0.1, -3.0, 0.2, 4.0], [-0.05, 1.0, -2.0, 0.3]])
    Wh, M = orc.magnitude_prune(W, p=0.5)
    np.testing.assert_array_equal(M, [[1, 0, 1, 0], [1, 0, 0, 1]])
    np.testing.assert_array_equal(Wh, W * (1 - M))
    Wh, M = orc.magnitude_prune(W, n=2, m=4)
    np.testing.assert_array_equal(M, [[1, 0, 1, 0], [1, 0, 0, 1]])
