"""Pins of the comparator oracles (Wanda, SparseGPT as the paper describes them).  CPU only."""
import numpy as np

from oracle import comparators as cmp
from oracle import thanos_oracle as orc
from synth import LayerSpec, make_calibration, make_weight


def _layer(c=12, b=16, tokens=64, seed=1):
    spec = LayerSpec("t", c=c, b=b, tokens=tokens, dtype="f32", rho=0.7, k_mix=8, seed=seed)
    return make_weight(spec).astype(np.float64), orc.hessian(make_calibration(spec))


def test_wanda_removes_the_smallest_metric_of_every_row_and_updates_nothing():
    W, H = _layer()
    Wh, M = cmp.wanda_prune(W, H, p=0.5)
    mu = orc.metric(W, np.diag(H), np.float64)
    for i in range(W.shape[0]):
        assert M[i].sum() == 8
        assert mu[i][M[i] == 1].max() <= mu[i][M[i] == 0].min()
    assert np.array_equal(Wh, W * (1 - M))
    Wn, Mn = cmp.wanda_prune(W, H, n=2, m=4)
    assert np.all(Mn.reshape(12, 4, 4).sum(axis=2) == 2)
    # with one group per row it is the paper's psi applied row by row
    for i in range(W.shape[0]):
        assert np.array_equal(orc.psi(W[i:i + 1], np.diag(H), 8, np.float64)[0], M[i])


def test_sparsegpt_single_weight_is_the_obs_update():
    # c = 1, one weight to remove in the first mask block: closed form of Sec. 3.2
    W, H = _layer(c=1, b=5)
    Hd = orc.damped(H, 0.01)
    Hinv = np.linalg.inv(Hd)
    Wh, M = cmp.sparsegpt_prune(W, H, p=0.2, Bs=5, damp=0.01)
    q = int(np.flatnonzero(M[0])[0])
    sal = W[0] ** 2 / np.diag(Hinv)
    assert q == int(np.argmin(sal))
    if q == 0:   # removed in the first step: the full inverse applies
        expect = W[0] - W[0, 0] / Hinv[0, 0] * Hinv[0]
        np.testing.assert_allclose(Wh[0], expect, atol=1e-12)
    assert Wh[0, q] == 0.0


def test_sparsegpt_is_sequential_obs_on_the_trailing_problem_and_never_beats_the_optimum():
    W, H = _layer(seed=3)
    Wh, M = cmp.sparsegpt_prune(W, H, p=0.5, Bs=8, damp=0.01)
    assert M.sum() == 12 * 16 // 2 and np.all(Wh[M == 1] == 0.0)
    Wn, Mn = cmp.sparsegpt_prune(W, H, n=2, m=4, damp=0.01)
    assert np.all(Mn.reshape(12, 4, 4).sum(axis=2) == 2)
    # for ITS OWN mask the one-shot constrained least squares (Thanos update with one block
    # over the whole row) is optimal for the damped objective
    Hd = orc.damped(H, 0.01)
    Wopt, _ = orc.prune_fast(W, H, mode="unstructured", p=0.0, B=16, damp=0.01, mask_in=M)
    obj = lambda Wx: float(np.einsum("ij,ij->", (Wx - W) @ Hd, Wx - W))
    assert obj(Wopt) <= obj(Wh) * (1 + 1e-9)
    # the first column's removals are exact OBS steps with the full inverse
    Hinv = np.linalg.inv(Hd)
    rows = np.flatnonzero(M[:, 0])
    if len(rows):
        W1 = W.copy()
        W1[rows] -= np.outer(W[rows, 0] / Hinv[0, 0], Hinv[0])
        # later columns change these rows again, but column 1 of a row not masked at column 1
        # and only masked at column 0 keeps the value of the first step
        for i in rows:
            if M[i, 1] == 0:
                j_next = next((j for j in range(1, 16) if M[i, j]), None)
                upto = j_next if j_next is not None else 16
                np.testing.assert_allclose(Wh[i, 1:upto], W1[i, 1:upto], atol=1e-12)
