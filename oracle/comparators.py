"""CPU comparators for the reconstruction-error tables: Wanda and SparseGPT as the paper
describes them (Sec. 3.3, 3.4; App. F.3, F.4).  TEST INFRASTRUCTURE, float64 numpy, not
imported by the GPU path.

  * Wanda: metric |W_ij| * ||X_j||_2 (the OBD metric with a diagonal Hessian), compared inside
    every output row; the smallest are removed, nothing is updated.
  * SparseGPT: columns are visited left to right.  Whenever the column index is a multiple of
    the mask block size Bs, the mask of the next Bs columns is chosen from the saliency
    w^2 / [Hinv]_qq of the CURRENT weights (unstructured: the share p of the c x Bs panel with
    the smallest saliency; n:m: Bs = m, per row the n smallest).  A masked weight of column j
    is removed with the single-weight OBS update of its row,
    w[j:] -= w_j / Hinv_jj * Hinv[j, j:], after which column j leaves the problem: Hinv becomes
    the inverse of the Hessian without row and column j (rank-one down-date).
"""
from __future__ import annotations

import numpy as np

from . import thanos_oracle as orc


def wanda_prune(W: np.ndarray, H: np.ndarray, *, p=None, n: int = 0, m: int = 0):
    W = np.array(W, dtype=np.float64, copy=True)
    c, b = W.shape
    mu = np.abs(W) * np.sqrt(np.diag(H))[None, :]
    M = np.zeros((c, b), dtype=np.uint8)
    if p is not None:
        k = orc.num_to_remove(p, 1, b)                 # per output row
        order = np.argsort(mu, axis=1, kind="stable")
        np.put_along_axis(M, order[:, :k], 1, axis=1)
    else:
        g = mu.reshape(c, b // m, m)
        order = np.argsort(g, axis=2, kind="stable")
        Mg = np.zeros_like(g, dtype=np.uint8)
        np.put_along_axis(Mg, order[:, :, :n], 1, axis=2)
        M = Mg.reshape(c, b)
    W[M == 1] = 0.0
    return W, M


def sparsegpt_prune(W: np.ndarray, H: np.ndarray, *, p=None, n: int = 0, m: int = 0,
                    Bs: int = 128, damp: float = 0.01):
    W = np.array(W, dtype=np.float64, copy=True)
    c, b = W.shape
    if p is None:
        Bs = m
    Hinv = np.linalg.inv(orc.damped(H, damp))          # inverse of the trailing Hessian
    M = np.zeros((c, b), dtype=np.uint8)
    for j in range(b):
        if j % Bs == 0:
            w = min(Bs, b - j)
            sal = W[:, j:j + w] ** 2 / np.diag(Hinv)[None, :w]
            if p is not None:
                k = orc.num_to_remove(p, c, w)
                idx = np.argsort(sal, axis=None, kind="stable")[:k]
                blk = np.zeros(c * w, dtype=np.uint8)
                blk[idx] = 1
                M[:, j:j + w] = blk.reshape(c, w)
            else:
                order = np.argsort(sal, axis=1, kind="stable")
                blk = np.zeros((c, w), dtype=np.uint8)
                np.put_along_axis(blk, order[:, :n], 1, axis=1)
                M[:, j:j + w] = blk
        rows = np.flatnonzero(M[:, j])
        if len(rows):
            W[rows, j:] -= np.outer(W[rows, j] / Hinv[0, 0], Hinv[0, :])
            W[rows, j] = 0.0
        # column j leaves the problem
        Hinv = Hinv[1:, 1:] - np.outer(Hinv[1:, 0], Hinv[0, 1:]) / Hinv[0, 0]
    return W, M
