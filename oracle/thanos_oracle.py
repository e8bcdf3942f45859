"""CPU oracle for Thanos block-wise pruning of one linear layer.

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow float64
numpy implementation written from the paper, used to check the GPU library and
as the timed CPU baseline.  It shares no code with the GPU path and must not be
imported by it.

Notation (paper, "Formulation of the problem" and the notation table):
  W in R^{c x b}   weights (c output rows, b input columns)
  X                calibration input; here token-major, X[t, j], T tokens
  H                Hessian of the row-wise objective, proportional to X^T X
  M in {0,1}^{c x b}, M_ij = 1 means W_ij is removed
  B                block size, p sparsity ratio, r weights still to remove

What is followed
  * Hessian:                Alg. 1 step "H <- 2XX^T" (here the Gram matrix of the
                            token-major X; a positive scale of H changes nothing).
  * Metric and psi_X:       Sec. 4.2 / eq. (psi): |W_ij| * ||X_j:||_2, mask of the
                            r smallest.
  * phi:                    Sec. 4.5 / eq. (phi): ascending indices of the ones.
  * R, R_hat, u, update:    Sec. 4.1, eqs. (R), (R_hat), (u) and
                            Delta = -u R_hat^{-1} R.
  * Unstructured sweep:     Alg. 1 (global residual mask, local block mask,
                            r <- r - ||M||_F^2, residual Hessian re-inverted per block).
  * n:m sweep:              the n:m algorithm of App. G.4.4; alpha > 0 (outlier rows,
                            Sec. 4.7 "Outlier rows"): row losses h_i = ||W_i X||^2, the
                            ceil(alpha*c) rows with the largest loss are not pruned.
  * Structured pruning:     Alg. 2 (Sec. 4.7): s = ceil(p*b/(1-alpha)) whole columns, chosen by
                            the column loss v_j of the non-outlier rows, removed from those
                            rows in one shot with the full inverse Hessian.
  * Magnitude pruning:      Sec. 3.1 / App. F.1 (comparator for the sanity bound).

Readings taken where the paper is silent or inconsistent (each is listed in the
design notes of the repository as well):
  * r = floor(p*c*b), evaluated exactly on the decimal value of p.
  * blocks are the half-open column ranges [jB, min(b, (j+1)B)), j = 0..ceil(b/B)-1.
  * after a block, "H" is the trailing principal sub-matrix of the damped
    Hessian and "H^{-1}" its inverse (not a sub-block of the full inverse).
  * damping: H_d = H + damp * mean(diag H) * I, once, on the full matrix.
  * the metric uses ||X_j||^2 = diag(H) before damping and the CURRENT weights.
  * ties: ascending (metric, row, column); the ranking is done on the metric
    rounded to float32 (the precision in which the GPU path takes the same
    decision), computed as fl32(|fl32(W)|) * fl32(sqrt(fl32(diag H))).
  * n:m: per row and per group of m consecutive columns, the n smallest-metric
    weights are removed (n = number of zeros per group).
  * outlier rows: their number is ceil(alpha*c) (the text), hence c - ceil(alpha*c) rows
    are pruned (the listing's loop bound ceil(c(1-alpha)) differs when alpha*c is not an
    integer); rows are ranked by ascending (h_i, i) and the last ones are the outliers;
    alpha is evaluated exactly on its decimal value; the row loss uses the undamped H.
  * removed weights are set to exactly 0.

parity status: every function below is pinned by tests/test_oracle_*.py
(worked examples printed in the paper, closed-form single-weight OBS, brute-force
constrained least squares, exact counts, special cases, invariances).  The
end-to-end value of (W_hat, M) on large layers has no independent pin beyond
those step-level ones and the literal == single-factorisation identity.
"""
from __future__ import annotations

import math
from fractions import Fraction
from typing import Optional, Tuple

import numpy as np
import scipy.linalg as sla


# --------------------------------------------------------------------------
# Hessian
# --------------------------------------------------------------------------
def hessian(X: np.ndarray, chunk: int = 16384) -> np.ndarray:
    """Gram matrix sum_t X[t,:]^T X[t,:] in float64 (Alg. 1, "H <- 2XX^T", unscaled).

    X is token-major [T, b] of any float dtype; it is converted exactly.
    """
    T, b = X.shape
    H = np.zeros((b, b), dtype=np.float64)
    for t0 in range(0, T, chunk):
        x = np.asarray(X[t0:t0 + chunk], dtype=np.float64)
        H += x.T @ x
    return H


def damped(H: np.ndarray, damp: float) -> np.ndarray:
    """H_d = H + damp * mean(diag H) * I."""
    Hd = np.array(H, dtype=np.float64, copy=True)
    lam = float(damp) * float(np.mean(np.diag(H)))
    Hd[np.diag_indices_from(Hd)] += lam
    return Hd


# --------------------------------------------------------------------------
# Metric, psi, phi
# --------------------------------------------------------------------------
def metric(W: np.ndarray, xnorm2: np.ndarray, dtype=np.float32) -> np.ndarray:
    """Pruning metric |W_ij| * ||X_j:||_2 (Sec. 4.2), ||X_j:||^2 given as xnorm2.

    With dtype=float32 every operand is rounded to float32 first and the
    product is a float32 product; with float64 it is the plain formula.
    """
    w = np.abs(np.asarray(W).astype(dtype))
    sx = np.sqrt(np.asarray(xnorm2).astype(dtype))
    return (w * sx[None, :]).astype(dtype)


def psi(W: np.ndarray, xnorm2: np.ndarray, r: int, dtype=np.float32) -> np.ndarray:
    """psi_X(W, r): mask (uint8) of the r entries with the smallest metric.

    Ties are broken by ascending (row, column).
    """
    mu = metric(W, xnorm2, dtype)
    M = np.zeros(mu.shape, dtype=np.uint8)
    if r <= 0:
        return M
    order = np.argsort(mu, axis=None, kind="stable")  # row-major flat index breaks ties
    M.flat[order[:r]] = 1
    return M


def phi(x: np.ndarray) -> np.ndarray:
    """phi(x): ascending 0-based indices of the non-zero entries of a 0/1 vector.

    (The paper prints 1-based indices; add 1 to compare with its examples.)
    """
    return np.flatnonzero(np.asarray(x))


def nm_mask(Wblk: np.ndarray, xnorm2_blk: np.ndarray, n: int, m: int,
            dtype=np.float32) -> np.ndarray:
    """n:m mask of a block of columns: in every row and every group of m
    consecutive columns the n smallest-metric weights are marked (App. G.4.4)."""
    c, width = Wblk.shape
    if width % m:
        raise ValueError("block width must be a multiple of m")
    mu = metric(Wblk, xnorm2_blk, dtype).reshape(c, width // m, m)
    order = np.argsort(mu, axis=2, kind="stable")
    M = np.zeros((c, width // m, m), dtype=np.uint8)
    np.put_along_axis(M, order[:, :, :n], 1, axis=2)
    return M.reshape(c, width)


# --------------------------------------------------------------------------
# Row update (Sec. 4.1)
# --------------------------------------------------------------------------
def row_update(w: np.ndarray, Hinv: np.ndarray, q: np.ndarray) -> np.ndarray:
    """Return w + Delta with Delta = -u R_hat^{-1} R  (eqs. (R), (R_hat), (u)).

    w: current row over the residual columns; Hinv: inverse of the residual
    (damped) Hessian; q: ascending indices to remove.  Entries q of the result
    are set to exactly zero.
    """
    w = np.array(w, dtype=np.float64, copy=True)
    if len(q) == 0:
        return w
    R = Hinv[q, :]            # s x (b - j1)
    Rhat = R[:, q]            # s x s
    u = w[q]                  # 1 x s
    lam = np.linalg.solve(Rhat.T, u)   # lam Rhat = u
    w -= lam @ R
    w[q] = 0.0
    return w


def num_to_remove(p, c: int, b: int) -> int:
    """r = floor(p*c*b), exact on the decimal value of p."""
    return int(Fraction(str(p)) * c * b // 1)


# --------------------------------------------------------------------------
# Literal sweeps: residual Hessian re-inverted at every block
# --------------------------------------------------------------------------
def _blocks(b: int, B: int):
    j1 = 0
    while j1 < b:
        yield j1, min(b, j1 + B)
        j1 += B


def prune_unstructured(W: np.ndarray, H: np.ndarray, p, B: int, damp: float,
                       metric_dtype=np.float32,
                       return_margins: bool = False):
    """Alg. 1 (unstructured).  Returns (W_hat float64, M uint8[, margins]).

    margins[j] = relative gap between the largest removed and the smallest kept
    metric of the global residual selection of block j (inf if nothing or
    everything was selected) -- used by tests to recognise near-ties.
    """
    W = np.array(W, dtype=np.float64, copy=True)
    c, b = W.shape
    xn2 = np.diag(H).astype(np.float64)
    Hd = damped(H, damp)
    M_full = np.zeros((c, b), dtype=np.uint8)
    r = num_to_remove(p, c, b)
    margins = []
    for j1, j2 in _blocks(b, B):
        Hinv = np.linalg.inv(Hd[j1:, j1:])
        Mhat = psi(W[:, j1:], xn2[j1:], r, metric_dtype)
        if return_margins:
            margins.append(_global_margin(W[:, j1:], xn2[j1:], r, metric_dtype))
        M = Mhat[:, :j2 - j1]
        r -= int(M.sum())
        for i in range(c):
            q = phi(M[i])
            if len(q):
                W[i, j1:] = row_update(W[i, j1:], Hinv, q)
        M_full[:, j1:j2] = M
    if return_margins:
        return W, M_full, np.array(margins)
    return W, M_full


def row_losses(W: np.ndarray, H: np.ndarray) -> np.ndarray:
    """h_i = ||W_i X||_2^2 = W_i H W_i^T (Sec. 4.7, eq. (row outlier loss)), H = X^T X."""
    W = np.asarray(W, dtype=np.float64)
    return np.einsum("ij,ij->i", W @ np.asarray(H, dtype=np.float64), W)


def num_outlier_rows(alpha, c: int) -> int:
    """ceil(alpha*c), evaluated exactly on the decimal value of alpha."""
    a = Fraction(str(alpha)) if not isinstance(alpha, Fraction) else alpha
    if not (0 <= a < 1):
        raise ValueError("alpha must be in [0, 1)")
    return int(math.ceil(a * c))


def pruned_rows(W: np.ndarray, H: np.ndarray, alpha, dtype=np.float64) -> np.ndarray:
    """Boolean vector: True for the rows that are pruned, False for the ceil(alpha*c) outlier
    rows (largest row loss; ascending (h, row) order, the rows permutation of App. G.4.3
    without moving anything).  `dtype` is the precision in which the ranking is taken."""
    c = W.shape[0]
    n_out = num_outlier_rows(alpha, c)
    h = row_losses(W, H).astype(dtype)
    order = np.lexsort((np.arange(c), h))        # ascending h, ties by row index
    keep = np.ones(c, dtype=bool)
    if n_out:
        keep[order[c - n_out:]] = False
    return keep


def prune_nm(W: np.ndarray, H: np.ndarray, n: int, m: int, B: int, damp: float,
             metric_dtype=np.float32,
             return_margins: bool = False, alpha=0, rows: Optional[np.ndarray] = None):
    """n:m algorithm of App. G.4.4.  Returns (W_hat, M[, margins]).

    alpha > 0: the outlier rows (see pruned_rows) are skipped: no mask, no update.
    `rows` (boolean, c) overrides the choice of pruned rows.

    margins has one entry per (row, group): relative gap between the n-th and
    the (n+1)-th smallest metric of the group at the time it was decided.
    """
    W = np.array(W, dtype=np.float64, copy=True)
    c, b = W.shape
    if b % m or B % m:
        raise ValueError("m must divide both b and B")
    xn2 = np.diag(H).astype(np.float64)
    Hd = damped(H, damp)
    if rows is None:
        rows = pruned_rows(W, H, alpha)
    M_full = np.zeros((c, b), dtype=np.uint8)
    margins = np.zeros((c, b // m))
    for j1, j2 in _blocks(b, B):
        Hinv = np.linalg.inv(Hd[j1:, j1:])
        M = nm_mask(W[:, j1:j2], xn2[j1:j2], n, m, metric_dtype)
        M[~rows] = 0
        if return_margins:
            margins[:, j1 // m:j2 // m] = _group_margins(W[:, j1:j2], xn2[j1:j2], n, m,
                                                         metric_dtype)
            margins[~rows, j1 // m:j2 // m] = np.inf   # nothing is decided in outlier rows
        for i in range(c):
            q = phi(M[i])
            W[i, j1:] = row_update(W[i, j1:], Hinv, q)
        M_full[:, j1:j2] = M
    if return_margins:
        return W, M_full, margins
    return W, M_full


def _global_margin(Wres, xn2res, r, dtype) -> float:
    mu = np.sort(metric(Wres, xn2res, dtype), axis=None).astype(np.float64)
    if r <= 0 or r >= mu.size:
        return float("inf")
    lo, hi = mu[r - 1], mu[r]
    return float((hi - lo) / max(hi, np.finfo(np.float64).tiny))


def _group_margins(Wblk, xn2blk, n, m, dtype) -> np.ndarray:
    c, width = Wblk.shape
    mu = np.sort(metric(Wblk, xn2blk, dtype).reshape(c, width // m, m), axis=2).astype(np.float64)
    lo, hi = mu[:, :, n - 1], mu[:, :, n]
    return (hi - lo) / np.maximum(hi, np.finfo(np.float64).tiny)


# --------------------------------------------------------------------------
# Structured pruning (Alg. 2)
# --------------------------------------------------------------------------
def num_columns_to_remove(p, alpha, b: int) -> int:
    """s = ceil(p*b / (1 - alpha)), evaluated exactly on the decimal values of p and alpha."""
    pf = Fraction(str(p)) if not isinstance(p, Fraction) else p
    af = Fraction(str(alpha)) if not isinstance(alpha, Fraction) else alpha
    if not (0 <= pf < 1 and 0 <= af < 1):
        raise ValueError("p and alpha must be in [0, 1)")
    return int(math.ceil(pf * b / (1 - af)))


def column_losses(W: np.ndarray, xnorm2: np.ndarray, rows: np.ndarray) -> np.ndarray:
    """v_j = ||W_{rows, j} (outer) X_j||_F^2 = (sum_{i in rows} W_ij^2) * ||X_j||^2 (Sec. 4.7,
    eq. (column loss)); `rows` = the rows that are pruned (outlier rows do not count)."""
    W = np.asarray(W, dtype=np.float64)
    return (W[rows] ** 2).sum(axis=0) * np.asarray(xnorm2, dtype=np.float64)


def prune_structured(W: np.ndarray, H: np.ndarray, p, alpha, damp: float,
                     dtype=np.float64):
    """Alg. 2.  Returns (W_hat, M).  No matrix is physically permuted: Q W P of the listing
    only serves to address the pruned rows (all but the ceil(alpha*c) of largest loss h_i) and
    the removed columns (the s of smallest loss v_j, ascending (v, j)).  The update is
    eq. (structured solution), Delta = -W_{:,Q} (Hinv[Q,Q])^{-1} Hinv[Q,:], with Hinv the
    inverse of the damped Hessian.  `dtype` is the precision in which both rankings are taken.
    """
    W = np.array(W, dtype=np.float64, copy=True)
    c, b = W.shape
    s = num_columns_to_remove(p, alpha, b)
    if s > b:
        raise ValueError("p / (1 - alpha) must not exceed 1")
    rows = pruned_rows(W, H, alpha, dtype)
    v = column_losses(W, np.diag(H), rows).astype(dtype)
    Q = np.sort(np.lexsort((np.arange(b), v))[:s])
    M = np.zeros((c, b), dtype=np.uint8)
    if s == 0 or not rows.any():
        return W, M
    Hinv = np.linalg.inv(damped(H, damp))
    lam = np.linalg.solve(Hinv[np.ix_(Q, Q)].T, W[np.ix_(rows, Q)].T).T   # W_Q (Hinv_QQ)^-1
    W[rows] -= lam @ Hinv[Q, :]
    W[np.ix_(rows, Q)] = 0.0
    M[np.ix_(rows, Q)] = 1
    return W, M


# --------------------------------------------------------------------------
# Single-factorisation sweeps (same result, used for large shapes / timing)
# --------------------------------------------------------------------------
def inverse_factor(Hd: np.ndarray) -> np.ndarray:
    """Upper-triangular U with Hd^{-1} = U^T U.

    Then inv(Hd[j:, j:]) = U[j:, j:]^T U[j:, j:] for every j, which is the
    matrix Alg. 1 re-computes after each block ("H <- 2(XX^T)_{j2:b, j2:b}").
    tests/test_oracle_steps.py (test_inverse_factor_gives_every_residual_inverse) checks that
    identity against np.linalg.inv of every trailing sub-matrix.
    """
    Hinv = sla.cho_solve(sla.cho_factor(Hd, lower=True), np.eye(Hd.shape[0]))
    Hinv = 0.5 * (Hinv + Hinv.T)
    return sla.cholesky(Hinv, lower=False)


def prune_fast(W: np.ndarray, H: np.ndarray, *, mode: str, p=None, n: int = 0, m: int = 0,
               B: int, damp: float, metric_dtype=np.float32,
               mask_in: Optional[np.ndarray] = None,
               U: Optional[np.ndarray] = None, alpha=0,
               rows: Optional[np.ndarray] = None,
               on_block=None) -> Tuple[np.ndarray, np.ndarray]:
    """Same sweeps as prune_unstructured / prune_nm, but every residual inverse is
    read off one factor U (see inverse_factor).  mask_in (c x b) forces the mask.

    on_block(j1, j2, W_current), if given, is called at the start of every block, before its
    mask is chosen, with the weights as they stand (read-only view for tests that check the
    decisions of a block against the weights the block actually saw); it changes nothing.
    """
    W = np.array(W, dtype=np.float64, copy=True)
    c, b = W.shape
    xn2 = np.diag(H).astype(np.float64)
    if U is None:
        U = inverse_factor(damped(H, damp))
    if rows is None:
        rows = pruned_rows(W, H, alpha) if mode == "nm" else np.ones(c, dtype=bool)
    M_full = np.zeros((c, b), dtype=np.uint8)
    r = num_to_remove(p, c, b) if mode == "unstructured" else 0
    for j1, j2 in _blocks(b, B):
        Ubb = U[j1:j2, j1:j2]
        Rows = Ubb.T @ U[j1:j2, j1:]          # first (j2-j1) rows of the residual inverse
        if on_block is not None:
            on_block(j1, j2, W)
        if mask_in is not None:
            M = np.asarray(mask_in[:, j1:j2], dtype=np.uint8)
        elif mode == "unstructured":
            M = psi(W[:, j1:], xn2[j1:], r, metric_dtype)[:, :j2 - j1]
            r -= int(M.sum())
        elif mode == "nm":
            M = nm_mask(W[:, j1:j2], xn2[j1:j2], n, m, metric_dtype)
            M[~rows] = 0
        else:
            raise ValueError(mode)
        G = Rows[:, :j2 - j1]
        for i in range(c):
            q = np.flatnonzero(M[i])
            if len(q) == 0:
                continue
            lam = np.linalg.solve(G[np.ix_(q, q)].T, W[i, j1 + q])
            W[i, j1:] -= lam @ Rows[q, :]
            W[i, j1 + q] = 0.0
        M_full[:, j1:j2] = M
    return W, M_full


# --------------------------------------------------------------------------
# Comparator and error measure
# --------------------------------------------------------------------------
def magnitude_prune(W: np.ndarray, *, p=None, n: int = 0, m: int = 0):
    """Magnitude pruning (Sec. 3.1): remove the smallest |W_ij|, no update.

    Unstructured: the floor(p*c*b) smallest over the layer; n:m: the n smallest
    of every group of m consecutive weights of a row.
    """
    W = np.array(W, dtype=np.float64, copy=True)
    c, b = W.shape
    ones = np.ones(b)
    if p is not None:
        M = psi(W, ones, num_to_remove(p, c, b), np.float64)
    else:
        M = nm_mask(W, ones, n, m, np.float64)
    W[M == 1] = 0.0
    return W, M


def reconstruction_error(W: np.ndarray, W_hat: np.ndarray, H: np.ndarray) -> float:
    """||(W_hat - W) X||_F^2 = tr(D H D^T), D = W_hat - W, H the undamped Gram matrix."""
    D = np.asarray(W_hat, dtype=np.float64) - np.asarray(W, dtype=np.float64)
    return float(np.einsum("ij,ij->", D @ H, D))
