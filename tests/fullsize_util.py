"""Checks of a full-size GPU sweep on a sample of rows the oracle can redo one by one.

The oracle replays the sampled rows under the GPU's own mask (teacher forcing) and, through the
per-block hook of its single-factorisation sweep, sees the weights every block actually saw.
Each decision of the GPU is then compared with the decision the oracle takes on those weights:
a difference is accepted only where the oracle's own margin says the decision is a near-tie
(relative gap below NEAR_TIE).  W_hat is compared row by row (1e-3 relative) and so is the
reconstruction error Delta_i H Delta_i^T (1 %).
"""
import numpy as np

from oracle import thanos_oracle as orc

NEAR_TIE = 1e-4


def sample_rows(c, n=64, seed=0):
    """>= n distinct rows: tile edges of the 128-row tiles, the middle, the ends, random ones."""
    fixed = [0, 1, 127, 128, 255, 256, c // 2 - 1, c // 2, c - 2, c - 1]
    fixed = [r for r in fixed if 0 <= r < c]
    g = np.random.default_rng(seed)
    rest = [int(r) for r in g.permutation(c) if int(r) not in fixed][:max(0, n - len(fixed))]
    return np.array(sorted(set(fixed + rest)))


def per_row_checks(W, H, Wg, Wt, tag):
    """Rows of the GPU result Wg against the oracle's Wt (same mask): 1e-3 relative per row and
    reconstruction error Delta_i H Delta_i^T within 1 % per row."""
    W = W.astype(np.float64)
    num = np.linalg.norm(Wg - Wt, axis=1)
    den = np.linalg.norm(Wt, axis=1)
    assert np.all(num <= 1e-3 * den), (tag, float((num / den).max()))
    Dg, Dt = Wg - W, Wt - W
    eg = np.einsum("ij,ij->i", Dg @ H, Dg)
    et = np.einsum("ij,ij->i", Dt @ H, Dt)
    assert np.all(np.abs(eg - et) <= 0.01 * et + 1e-30), (tag, float(np.max(np.abs(eg - et) / et)))
    return float((num / den).max()), float(np.max(np.abs(eg - et) / np.maximum(et, 1e-300)))


def check_nm_rows(W, H, U, Wg, Mg, n, m, B, damp, tag):
    """W, Wg, Mg: the sampled rows (input weights, GPU result, GPU mask)."""
    xn2 = np.diag(H)
    stats = {"groups": 0, "differ": 0}

    def on_block(j1, j2, Wcur):
        Mo = orc.nm_mask(Wcur[:, j1:j2], xn2[j1:j2], n, m)
        mg = orc._group_margins(Wcur[:, j1:j2], xn2[j1:j2], n, m, np.float32)
        diff = (Mo != Mg[:, j1:j2]).reshape(Mo.shape[0], -1, m).any(axis=2)
        stats["groups"] += diff.size
        stats["differ"] += int(diff.sum())
        assert np.all(mg[diff] < NEAR_TIE), (tag, j1, float(mg[diff].max()))

    Wt, _ = orc.prune_fast(W, H, mode="nm", n=n, m=m, B=B, damp=damp, U=U, mask_in=Mg,
                           on_block=on_block)
    assert stats["differ"] <= max(2, 1e-4 * stats["groups"]), (tag, stats)
    worst = per_row_checks(W, H, Wg, Wt, tag)
    # free-running oracle: rows are independent, so a row either matches entirely or has a
    # near-tie somewhere (checked above); most rows must match entirely
    Wf, Mf = orc.prune_fast(W, H, mode="nm", n=n, m=m, B=B, damp=damp, U=U)
    same = np.all(Mf == Mg, axis=1)
    assert same.mean() >= 0.9, (tag, float(same.mean()))
    per_row_checks(W[same], H, Wg[same], Wf[same], tag + " free-running")
    print(f"{tag}: {stats['differ']} of {stats['groups']} group decisions differ (all near-ties), "
          f"{int(same.sum())}/{len(same)} rows identical to the free-running oracle, "
          f"worst row error {worst[0]:.2e}, worst reconstruction-error gap {worst[1]:.2e}",
          flush=True)


def check_unstructured_rows(W, H, U, Wg, Mg, tau, p, B, damp, tag):
    """tau: the GPU's threshold per block (fp32).  A weight is removed if its fp32 metric on the
    weights the block saw is below tau_j, kept if above; equal to tau_j: either (ties are taken in
    (row, column) order over ALL rows, which a sample cannot replay)."""
    xn2 = np.diag(H)
    stats = {"n": 0, "differ": 0, "ties": 0}

    def on_block(j1, j2, Wcur):
        t = np.float32(tau[j1 // B])
        mu = orc.metric(Wcur[:, j1:j2], xn2[j1:j2], np.float32)
        got = Mg[:, j1:j2].astype(bool)
        if t < 0:                                   # nothing left to remove
            assert not got.any(), (tag, j1)
            return
        want = mu < t
        tie = mu == t
        diff = (want != got) & ~tie
        stats["n"] += diff.size
        stats["differ"] += int(diff.sum())
        stats["ties"] += int(tie.sum())
        gap = np.abs(mu.astype(np.float64) - float(t)) / max(float(t), 1e-300)
        assert np.all(gap[diff] < NEAR_TIE), (tag, j1, float(gap[diff].max()))

    Wt, _ = orc.prune_fast(W, H, mode="unstructured", p=p, B=B, damp=damp, U=U, mask_in=Mg,
                           on_block=on_block)
    assert stats["differ"] <= max(2, 1e-4 * stats["n"]), (tag, stats)
    worst = per_row_checks(W, H, Wg, Wt, tag)
    print(f"{tag}: {stats['differ']} of {stats['n']} decisions differ (all within {NEAR_TIE:g} of "
          f"the threshold), {stats['ties']} exactly at it, worst row error {worst[0]:.2e}, worst "
          f"reconstruction-error gap {worst[1]:.2e}", flush=True)
