"""GPU parity: thanos_prune_layer against the CPU oracle.

Bar: masks bit-exact on inputs without near-ties; W_hat within 1e-3 relative Frobenius error;
reconstruction error within 1 % of the oracle's.  Both sides receive the same fp32 Hessian, so
the first block's selection is taken on identical numbers on both sides; later blocks see
weights that differ by fp32 rounding, which can only flip decisions whose margin is at that
level (checked through the margins the oracle reports).
"""
import numpy as np
import pytest

from oracle import thanos_oracle as orc
from synth import LayerSpec, make_weight, make_calibration

pytestmark = pytest.mark.gpu


def _layer(c, b, T, dtype="f32", rho=0.7, seed=0, outliers=False):
    spec = LayerSpec("t", c=c, b=b, tokens=T, dtype=dtype, rho=rho, k_mix=16, seed=seed,
                     outliers=outliers)
    W = make_weight(spec)
    X = make_calibration(spec)
    H32 = orc.hessian(X).astype(np.float32)
    return W, H32


def _rel(a, b):
    return np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300)


def _check(W, H32, Wg, Mg, Wo, Mo, exact_mask=True):
    H = H32.astype(np.float64)
    if exact_mask:
        np.testing.assert_array_equal(Mg, Mo)
    assert np.all(Wg[Mg == 1] == 0.0)
    if np.array_equal(Mg, Mo):
        assert _rel(Wg, Wo) < 1e-3
    eo = orc.reconstruction_error(W, Wo, H)
    eg = orc.reconstruction_error(W, Wg.astype(np.float64), H)
    assert abs(eg - eo) <= 0.01 * eo + 1e-12


# --------------------------------------------------------------------------- configuration 1
@pytest.mark.parametrize("rho", [0.0, 0.7])
def test_cfg1_unstructured(rho):
    from tests.gpu_util import gpu_prune
    # seeds searched on the CPU so that the oracle's smallest decision margin is > 5e-6
    W, H32 = _layer(512, 512, 2048, "f32", rho=rho, seed={0.0: 0, 0.7: 4}[rho])
    print(f"cfg1 unstructured rho={rho}", flush=True)
    Wg, Mg, info = gpu_prune(W, H32, mode="unstructured", p=0.5, B=128)
    assert info == 0
    assert int(Mg.sum()) == 512 * 512 // 2
    Wo, Mo, margins = orc.prune_unstructured(W, H32.astype(np.float64), 0.5, 128, 0.01,
                                             return_margins=True)
    assert margins.min() > 5e-6, "seed has a near-tie; pick another"
    _check(W, H32, Wg, Mg, Wo, Mo)
    # the same decisions when the oracle ranks the plain float64 metric instead of the one rounded
    # to float32 like the kernel's: with margins > 5e-6 a rounding of ~2e-7 decides nothing
    _, Mo64 = orc.prune_unstructured(W, H32.astype(np.float64), 0.5, 128, 0.01,
                                     metric_dtype=np.float64)
    np.testing.assert_array_equal(Mg, Mo64)
    Wm, _ = orc.magnitude_prune(W, p=0.5)
    H = H32.astype(np.float64)
    assert orc.reconstruction_error(W, Wg.astype(np.float64), H) <= orc.reconstruction_error(W, Wm, H)


@pytest.mark.parametrize("n,m,rho", [(2, 4, 0.0), (2, 4, 0.7), (4, 8, 0.7), (1, 4, 0.7), (3, 4, 0.7)])
def test_cfg1_nm(n, m, rho):
    from tests.gpu_util import gpu_prune
    W, H32 = _layer(512, 512, 2048, "f32", rho=rho, seed=1)
    print(f"cfg1 {n}:{m} rho={rho}", flush=True)
    Wg, Mg, info = gpu_prune(W, H32, mode="nm", n=n, m=m, B=128)
    assert info == 0
    assert np.all(Mg.reshape(512, 512 // m, m).sum(axis=2) == n)
    Wo, Mo, mg = orc.prune_nm(W, H32.astype(np.float64), n, m, 128, 0.01, return_margins=True)
    bad_rows = np.unique(np.nonzero(Mg != Mo)[0])
    # a differing group must be a near-tie in the oracle (fp32 vs fp64 weights after updates)
    if len(bad_rows):
        gi, gj = np.nonzero((Mg != Mo).reshape(512, 512 // m, m).any(axis=2))
        first = {}
        for i, j in zip(gi, gj):
            first.setdefault(i, j)
        for i, j in first.items():
            assert mg[i, j] < 1e-4, (i, j, mg[i, j])
        assert len(bad_rows) <= 2
    print(f"  rows whose mask differs from the free-running oracle: {len(bad_rows)}", flush=True)
    # every decision of every block (not only the first differing one of a row) against the
    # oracle's decision on the weights that block saw; W_hat and reconstruction error per row
    from tests.fullsize_util import check_nm_rows
    Hd64 = H32.astype(np.float64)
    check_nm_rows(W, Hd64, orc.inverse_factor(orc.damped(Hd64, 0.01)), Wg.astype(np.float64), Mg,
                  n, m, 128, 0.01, f"cfg1 {n}:{m} rho={rho}")
    ok = np.setdiff1d(np.arange(512), bad_rows)
    np.testing.assert_array_equal(Mg[ok], Mo[ok])
    assert _rel(Wg[ok], Wo[ok]) < 1e-3
    _check(W, H32, Wg, Mg, Wo, Mo, exact_mask=False)
    # oracle ranking the plain float64 metric: same masks wherever its own margins are clear
    _, Mo64, mg64 = orc.prune_nm(W, H32.astype(np.float64), n, m, 128, 0.01,
                                 metric_dtype=np.float64, return_margins=True)
    clear = np.all(mg64 > 1e-5, axis=1)
    assert clear.mean() > 0.95
    np.testing.assert_array_equal(Mg[clear & np.isin(np.arange(512), ok)],
                                  Mo64[clear & np.isin(np.arange(512), ok)])


# --------------------------------------------------------------------------- ragged shapes
@pytest.mark.parametrize("c,b,B,mode", [
    (100, 328, 128, "unstructured"),    # c not a multiple of anything, last block 72 wide
    (100, 328, 128, "nm"),
    (67, 200, 64, "unstructured"),      # one column per lane
    (67, 200, 32, "nm"),
    (130, 260, 100, "unstructured"),    # B not a power of two
    (50, 150, 50, "unstructured"),      # B and b not multiples of 4: scalar load paths
    (96, 768, 256, "unstructured"),     # block size 256 (configuration 5), 4 wavefronts per row
    (64, 640, 256, "nm"),               # last block 128 wide
    (40, 450, 200, "unstructured"),     # wide block, nothing aligned
    (9, 40, 128, "unstructured"),       # single narrow block
    (5, 16, 1, "unstructured"),         # B = 1
    (70, 1216, 512, "nm"),              # block 512 (the n:m setting of the Experiments section): 256 unknowns per row,
                                        # last block 192 wide
    (48, 768, 256, "nm14"),             # 1:4 at block 256: 64 unknowns per row in a wide block
    # b not a multiple of 8 at more than toy size: the scalar / 8-byte paths of the sweep
    (300, 1100, 128, "unstructured"),   # b % 8 == 4
    (300, 1100, 128, "nm"),
    (257, 1030, 128, "unstructured"),   # b % 4 == 2: nothing 16-byte aligned from row to row
    # large blocks of the block-size ablation: more than 256 unknowns per row, tile grids in
    # global memory, workgroups that walk the rows
    (40, 2304, 1024, "nm"),             # 512 unknowns per row; last block 256 wide (LDS path)
    (30, 1100, 512, "unstructured"),    # up to 512 unknowns, ragged last block of 76
    (600, 1536, 1024, "nm"),            # more rows than resident workgroups
    (24, 4608, 2048, "nm"),             # 1024 unknowns per row
    (16, 4096, 4096, "nm14"),           # one block of 4096 columns, 1024 unknowns per row
    # rows that lose more than half of a block are solved through the inverse of the block's G
    # (complement form: bw - s unknowns)
    (32, 1024, 512, "nm34"),            # 3:4: 384 removed per row and block -> 128 unknowns
    (20, 2048, 1024, "unstructured"),   # up to 512 unknowns either way: tile grids in global memory
    (48, 1024, 256, "unstructured70"),  # 70 %: most rows go the complement way, some do not
])
def test_ragged_shapes(c, b, B, mode):
    from tests.gpu_util import gpu_prune
    W, H32 = _layer(c, b, 4 * b, "f32", seed=c + b)
    print(f"ragged c={c} b={b} B={B} {mode}", flush=True)
    H = H32.astype(np.float64)
    from tests.fullsize_util import check_nm_rows, check_unstructured_rows
    if mode.startswith("unstructured"):
        p = 0.7 if mode.endswith("70") else 0.5
        Wg, Mg, info, tau = gpu_prune(W, H32, mode="unstructured", p=p, B=B, tau=True)
        Wo, Mo = orc.prune_unstructured(W, H, p, B, 0.01)
        assert int(Mg.sum()) == orc.num_to_remove(p, c, b)
    else:
        n, m = {"nm14": (1, 4), "nm34": (3, 4)}.get(mode, (2, 4))
        Wg, Mg, info = gpu_prune(W, H32, mode="nm", n=n, m=m, B=B)
        Wo, Mo = orc.prune_nm(W, H, n, m, B, 0.01)
    assert info == 0
    if np.array_equal(Mg, Mo):
        _check(W, H32, Wg, Mg, Wo, Mo)
        return
    # the masks differ: every differing decision must be a near-tie of the oracle on the weights
    # the block saw, and W_hat must match the oracle under the GPU's mask row by row
    print(f"  masks differ at {int((Mg != Mo).sum())} positions: checking decision by decision",
          flush=True)
    assert (Mg != Mo).mean() < 1e-3
    U = orc.inverse_factor(orc.damped(H, 0.01))
    if mode.startswith("unstructured"):
        check_unstructured_rows(W, H, U, Wg.astype(np.float64), Mg, tau, p, B, 0.01, f"ragged {c}x{b}")
    else:
        check_nm_rows(W, H, U, Wg.astype(np.float64), Mg, n, m, B, 0.01, f"ragged {c}x{b}")


def test_cfg5_like_block256_heavy_tailed():
    # configuration 5 in small: N(0, 0.015^2) fp16 weights, outlier channels, 60 % unstructured,
    # block 256
    from tests.gpu_util import gpu_prune
    spec = LayerSpec("t", c=160, b=1024, tokens=4096, dtype="f16", w_std=0.015, rho=0.7, k_mix=16,
                     seed=11, outliers=True)
    W, X = make_weight(spec), make_calibration(spec)
    H32 = orc.hessian(X).astype(np.float32)
    H = H32.astype(np.float64)
    Wg, Mg, info = gpu_prune(W, H32, mode="unstructured", p=0.6, B=256)
    assert info == 0
    assert int(Mg.sum()) == orc.num_to_remove(0.6, 160, 1024)
    Wo, Mo = orc.prune_fast(W, H, mode="unstructured", p=0.6, B=256, damp=0.01)
    assert (Mg != Mo).mean() < 1e-4
    Wt, _ = orc.prune_fast(W, H, mode="unstructured", p=0.6, B=256, damp=0.01, mask_in=Mg)
    assert _rel(Wg, Wt) < 1e-3
    eo = orc.reconstruction_error(W, Wo, H)
    eg = orc.reconstruction_error(W, Wg.astype(np.float64), H)
    assert abs(eg - eo) <= 0.01 * eo
    # 4:8 at block 256: s = 128 per row
    Wg, Mg, info = gpu_prune(W, H32, mode="nm", n=4, m=8, B=256)
    assert info == 0
    assert np.all(Mg.reshape(160, 128, 8).sum(axis=2) == 4)
    Wt, _ = orc.prune_fast(W, H, mode="nm", n=4, m=8, B=256, damp=0.01, mask_in=Mg)
    assert _rel(Wg, Wt) < 1e-3
    _, Mo = orc.prune_fast(W, H, mode="nm", n=4, m=8, B=256, damp=0.01)
    assert (Mg != Mo).mean() < 1e-3


# --------------------------------------------------------------------------- outlier rows
@pytest.mark.parametrize("alpha,n,m,B,use_factor", [(0.1, 2, 4, 128, False), (0.25, 4, 8, 64, True)])
def test_nm_with_outlier_rows(alpha, n, m, B, use_factor):
    """n:m algorithm with alpha > 0 (App. G.4.4): the ceil(alpha c) rows of largest loss
    h_i = W_i H W_i^T stay dense and untouched, the others are pruned as usual."""
    from tests.gpu_util import gpu_factor, gpu_prune
    c, b = 200, 384
    W, H32 = _layer(c, b, 2048, "f16", rho=0.7, seed=21)
    # spread the row norms: the ranking of the row losses is then decided far above fp32 noise
    scale = np.linspace(0.5, 2.0, c)[np.random.default_rng(5).permutation(c)]
    W = (W.astype(np.float64) * scale[:, None]).astype(np.float16)
    H = H32.astype(np.float64)
    n_out = orc.num_outlier_rows(alpha, c)
    h = np.sort(orc.row_losses(W.astype(np.float64), H))
    assert (h[c - n_out] - h[c - n_out - 1]) / h[c - n_out] > 1e-3   # margin at the cut
    rows = orc.pruned_rows(W.astype(np.float64), H, alpha)
    print(f"outlier rows alpha={alpha} {n}:{m} B={B}", flush=True)
    kw = {}
    if use_factor:   # H is still needed for the row losses
        U, xn2, info = gpu_factor(H32, 0.01)
        assert info == 0
        kw = dict(U=U, xnorm2=xn2)
    Wg, Mg, info = gpu_prune(W, H32, mode="nm", n=n, m=m, B=B, alpha=alpha, **kw)
    assert info == 0
    # outlier rows: untouched, no mask
    np.testing.assert_array_equal(Mg[~rows], 0)
    np.testing.assert_array_equal(Wg[~rows], W[~rows].astype(np.float32))
    assert (~rows).sum() == n_out
    # pruned rows: exact n:m pattern, parity with the oracle
    assert np.all(Mg[rows].reshape(rows.sum(), b // m, m).sum(axis=2) == n)
    Wo, Mo, mg = orc.prune_nm(W, H, n, m, B, 0.01, return_margins=True, alpha=alpha)
    diff_rows = np.unique(np.nonzero(Mg != Mo)[0])
    for i in diff_rows:   # a differing group must be a near-tie in the oracle
        j = np.nonzero((Mg[i] != Mo[i]).reshape(b // m, m).any(axis=1))[0][0]
        assert mg[i, j] < 1e-4, (i, j, mg[i, j])
    assert len(diff_rows) <= 2
    ok = np.setdiff1d(np.arange(c), diff_rows)
    assert _rel(Wg[ok], Wo[ok]) < 1e-3
    Wt, _ = orc.prune_fast(W, H, mode="nm", n=n, m=m, B=B, damp=0.01, mask_in=Mg)
    assert _rel(Wg, Wt) < 1e-3


def test_outlier_rows_argument_checks():
    import torch
    import paper_2504_05346_amd as th
    o = th.PruneOpts(mode=th.THANOS_UNSTRUCTURED, sparsity=0.5, block_size=128, damping=0.01,
                     outlier_fraction=0.1)
    assert th.thanos_prune_workspace_bytes(64, 128, o) == 0          # not defined for Alg. 1
    o = th.PruneOpts(mode=th.THANOS_NM, n=2, m=4, block_size=128, damping=0.01,
                     outlier_fraction=1.0)
    assert th.thanos_prune_workspace_bytes(64, 128, o) == 0          # alpha must be < 1
    o0 = th.PruneOpts(mode=th.THANOS_NM, n=2, m=4, block_size=128, damping=0.01)
    o1 = th.PruneOpts(mode=th.THANOS_NM, n=2, m=4, block_size=128, damping=0.01,
                      outlier_fraction=0.1)
    assert th.thanos_prune_workspace_bytes(64, 128, o1) > th.thanos_prune_workspace_bytes(64, 128, o0)


# --------------------------------------------------------------------------- structured (Alg. 2)
@pytest.mark.parametrize("c,b,p,alpha,dtype", [(200, 384, 0.5, 0.0, "f16"), (150, 300, 0.3, 0.1, "f32"),
                                               (64, 1000, 0.25, 0.2, "f16"),
                                               (1536, 2048, 0.25, 0.05, "f16")])   # several tiles each way
def test_structured(c, b, p, alpha, dtype):
    """Alg. 2: s = ceil(p b / (1 - alpha)) columns of smallest loss removed from the
    non-outlier rows in one shot."""
    from tests.gpu_util import gpu_prune
    W, H32 = _layer(c, b, 4 * b, dtype, rho=0.7, seed=31)
    rng = np.random.default_rng(9)
    W = (W.astype(np.float64) * np.linspace(0.5, 2.0, c)[rng.permutation(c)][:, None]
         * np.linspace(0.6, 1.8, b)[rng.permutation(b)][None, :]).astype(W.dtype)
    H = H32.astype(np.float64)
    s = orc.num_columns_to_remove(p, alpha, b)
    rows = orc.pruned_rows(W.astype(np.float64), H, alpha)
    v = np.sort(orc.column_losses(W.astype(np.float64), np.diag(H), rows))
    assert (v[s] - v[s - 1]) / v[s] > 1e-4            # margin at the column cut
    print(f"structured {c}x{b} p={p} alpha={alpha}", flush=True)
    Wg, Mg, info = gpu_prune(W, H32, mode="structured", p=p, alpha=alpha, cast=True)[:3]
    assert info == 0
    Wo, Mo = orc.prune_structured(W, H, p, alpha, 0.01)
    np.testing.assert_array_equal(Mg, Mo)
    assert np.all(Wg[Mg == 1] == 0.0)
    np.testing.assert_array_equal(Wg[~rows], W[~rows].astype(np.float32))
    assert _rel(Wg, Wo) < 1e-3
    eo = orc.reconstruction_error(W, Wo, H)
    eg = orc.reconstruction_error(W, Wg.astype(np.float64), H)
    assert abs(eg - eo) <= 0.01 * eo


def test_structured_argument_checks():
    import paper_2504_05346_amd as th
    ok = th.PruneOpts(mode=th.THANOS_STRUCTURED, sparsity=0.5, damping=0.01, outlier_fraction=0.1)
    assert th.thanos_prune_workspace_bytes(64, 128, ok) > 0
    bad = th.PruneOpts(mode=th.THANOS_STRUCTURED, sparsity=0.8, damping=0.01, outlier_fraction=0.5)
    assert th.thanos_prune_workspace_bytes(64, 128, bad) == 0        # p / (1 - alpha) > 1


# --------------------------------------------------------------------------- forced masks
def test_given_mask_with_empty_and_full_rows():
    from tests.gpu_util import gpu_prune
    c, b, B = 96, 384, 128
    W, H32 = _layer(c, b, 2048, "f32", seed=5)
    g = np.random.default_rng(0)
    M = (g.random((c, b)) < g.random((c, 1))).astype(np.uint8)   # per-row density 0..1
    M[0] = 0
    M[1] = 1
    M[2, :128] = 1
    M[3, 128:256] = 0
    Wg, Mg, info = gpu_prune(W, H32, mode="unstructured", p=0.5, B=B, mask_in=M)
    assert info == 0
    np.testing.assert_array_equal(Mg, M)
    Wo, Mo = orc.prune_fast(W, H32.astype(np.float64), mode="unstructured", p=0.5, B=B, damp=0.01,
                            mask_in=M)
    assert np.all(Wg[M == 1] == 0.0)
    np.testing.assert_array_equal(Wg[0], W[0])           # nothing removed: row untouched
    assert np.all(Wg[1] == 0.0)
    assert _rel(Wg, Wo) < 1e-3
    rows = np.linalg.norm(Wg - Wo, axis=1) / np.maximum(np.linalg.norm(Wo, axis=1), 1e-30)
    assert rows.max() < 1e-3


def test_factor_reuse_matches_internal_factor():
    from tests.gpu_util import gpu_prune, gpu_factor
    W, H32 = _layer(64, 256, 1024, "f32", seed=6)
    U, xn2, info = gpu_factor(H32, 0.01)
    a = gpu_prune(W, H32, mode="nm", n=2, m=4, B=128)
    b_ = gpu_prune(W, None, mode="nm", n=2, m=4, B=128, U=U, xnorm2=xn2)
    np.testing.assert_array_equal(a[1], b_[1])
    np.testing.assert_array_equal(a[0], b_[0])


# --------------------------------------------------------------------------- ties
@pytest.mark.parametrize("B", [64, 128, 256])   # one block size per per-row solver
def test_exact_ties_follow_row_major_order(B):
    # Diagonal Hessian: no surviving weight moves, so every block sees heavily tied metrics
    # (weights from a 5-value set); the mask must equal one global psi with (row, col) ties.
    from tests.gpu_util import gpu_prune
    g = np.random.default_rng(1)
    c, b = 40, 512
    W = g.choice(np.array([-2.0, -1.0, 0.5, 1.0, 2.0], dtype=np.float32), size=(c, b))
    H32 = np.diag(g.choice(np.array([1.0, 4.0], dtype=np.float32), size=b))
    for p in (0.5, 0.3):
        print(f"ties B={B} p={p}", flush=True)
        Wg, Mg, info = gpu_prune(W, H32, mode="unstructured", p=p, B=B, damp=0.01)
        assert info == 0
        Mref = orc.psi(W, np.diag(H32), orc.num_to_remove(p, c, b))
        np.testing.assert_array_equal(Mg, Mref)
        np.testing.assert_array_equal(Wg, W * (1 - Mref))
    Wg, Mg, _ = gpu_prune(W, H32, mode="nm", n=2, m=4, B=64)
    np.testing.assert_array_equal(Mg, orc.nm_mask(W, np.diag(H32), 2, 4))


@pytest.mark.parametrize("need", [1, 5, 14])
def test_few_ties_at_the_threshold_in_later_blocks(need):
    """Distinct metrics except 15 equal ones exactly at the threshold, scattered over all blocks,
    of which `need` are removed: every block after the first resolves its threshold from the
    window the previous update counted and must rank the ties in (row, column) order over its
    residual.  Diagonal Hessian: no weight moves, so the mask is one global psi."""
    from tests.gpu_util import gpu_prune
    g = np.random.default_rng(3)
    c, b, N = 64, 512, 64 * 512
    vals = (np.arange(1, N + 1, dtype=np.float32) / np.float32(N))       # exact in fp32, distinct
    r = N // 2
    lo = r - need                                    # ranks lo+1 .. lo+15 become ties
    vals[lo:lo + 15] = vals[lo]
    W = (g.permutation(vals) * g.choice(np.array([-1.0, 1.0], dtype=np.float32), size=N)
         ).reshape(c, b).astype(np.float32)
    H32 = np.eye(b, dtype=np.float32)
    tie_cols = np.nonzero(np.abs(W) == vals[lo])[1]
    assert len(tie_cols) == 15 and len(set(tie_cols // 128)) >= 3      # ties in several blocks
    Wg, Mg, info = gpu_prune(W, H32, mode="unstructured", p=0.5, B=128, damp=0.01)
    assert info == 0
    Mref = orc.psi(W, np.ones(b), r)
    assert int(Mref[np.abs(W) == vals[lo]].sum()) == need               # the cut is inside the ties
    np.testing.assert_array_equal(Mg, Mref)
    np.testing.assert_array_equal(Wg, W * (1 - Mref))


@pytest.mark.parametrize("mode", ["unstructured", "nm"])
def test_seventeen_row_tiles(mode):
    # 2176 rows = 17 row tiles of the trailing update: its tile order by XCD (bands of
    # ceil(17 / 8) = 3 row tiles, the last XCDs with a short band or none) is only used from 16
    # row tiles on.
    from tests.gpu_util import gpu_prune
    c, b = 2176, 384
    W, H32 = _layer(c, b, 1536, "f32", rho=0.7, seed=21)
    print(f"17 row tiles {mode}", flush=True)
    H = H32.astype(np.float64)
    if mode == "nm":
        Wg, Mg, info = gpu_prune(W, H32, mode="nm", n=2, m=4, B=128)
        Wo, Mo = orc.prune_nm(W, H, 2, 4, 128, 0.01)
        assert np.all(Mg.reshape(c, b // 4, 4).sum(axis=2) == 2)
    else:
        Wg, Mg, info = gpu_prune(W, H32, mode="unstructured", p=0.5, B=128)
        Wo, Mo = orc.prune_unstructured(W, H, 0.5, 128, 0.01)
        assert int(Mg.sum()) == orc.num_to_remove(0.5, c, b)
    assert info == 0
    # fp32 against fp64 weights after the updates: a few near-ties may fall the other way
    assert np.mean(Mg != Mo) < 2e-4
    same = np.all(Mg == Mo, axis=1)
    assert same.mean() > 0.9
    assert _rel(Wg[same], Wo[same]) < 1e-3
    _check(W, H32, Wg, Mg, Wo, Mo, exact_mask=False)


def test_threshold_jumps_between_blocks():
    # Column blocks of very different scale: the global threshold moves by orders of magnitude
    # from block to block, far outside the window predicted from the previous block's, so every
    # block after the first takes the full radix passes; the third block loses all its 128
    # columns in every row (s = B), the second nearly none.
    from tests.gpu_util import gpu_prune
    W, H32 = _layer(96, 512, 2048, "f32", rho=0.0, seed=11)
    scale = np.repeat(np.array([1.0, 300.0, 0.01, 20.0], dtype=np.float32), 128)
    W = (W * scale).astype(np.float32)
    print("threshold jumps", flush=True)
    Wg, Mg, info = gpu_prune(W, H32, mode="unstructured", p=0.5, B=128)
    assert info == 0
    Wo, Mo, margins = orc.prune_unstructured(W, H32.astype(np.float64), 0.5, 128, 0.01,
                                             return_margins=True)
    assert margins.min() > 2e-5, "seed has a near-tie; pick another"
    per_block = Mo.reshape(96, 4, 128).sum(axis=(0, 2))
    assert per_block[2] == 96 * 128 and per_block[1] < 96
    _check(W, H32, Wg, Mg, Wo, Mo)
    _, Mo64 = orc.prune_unstructured(W, H32.astype(np.float64), 0.5, 128, 0.01,
                                     metric_dtype=np.float64)
    np.testing.assert_array_equal(Mg, Mo64)


@pytest.mark.parametrize("growth", [1.002, 1.006, 1.02])
def test_threshold_drifts_steadily(growth):
    # Column blocks whose scale grows by a constant factor: the global threshold moves by a
    # steady step from block to block -- a fraction of the narrowest selection window, about its
    # half-width, and beyond the widest one -- so the sweep meets windows of every bin width and
    # blocks that fall back to the radix passes.
    from tests.gpu_util import gpu_prune
    from tests.fullsize_util import check_unstructured_rows
    c, b, B = 96, 2048, 128
    W, H32 = _layer(c, b, 4096, "f32", rho=0.0, seed=21)
    W = (W * (growth ** (np.arange(b) // B)).astype(np.float32)[None, :]).astype(np.float32)
    print(f"threshold drift, growth {growth} per block", flush=True)
    Wg, Mg, info, tau = gpu_prune(W, H32, mode="unstructured", p=0.5, B=B, tau=True)
    assert info == 0 and int(Mg.sum()) == c * b // 2
    H = H32.astype(np.float64)
    Wo, Mo = orc.prune_unstructured(W, H, 0.5, B, 0.01)
    step = np.abs(np.diff(tau)) / tau[:-1]
    print(f"  relative step of the threshold per block: median {np.median(step):.1e}, "
          f"max {step.max():.1e}; masks differ at {int((Mg != Mo).sum())} positions", flush=True)
    assert (Mg != Mo).mean() < 1e-4
    check_unstructured_rows(W, H, orc.inverse_factor(orc.damped(H, 0.01)), Wg.astype(np.float64), Mg,
                            tau, 0.5, B, 0.01, f"drift {growth}")


def test_sparsity_edge_values():
    from tests.gpu_util import gpu_prune
    W, H32 = _layer(16, 128, 512, "f32", seed=7)
    Wg, Mg, info = gpu_prune(W, H32, mode="unstructured", p=0.0, B=64)
    assert Mg.sum() == 0
    np.testing.assert_array_equal(Wg, W)
    Wg, Mg, info = gpu_prune(W, H32, mode="unstructured", p=0.6, B=64)
    assert int(Mg.sum()) == orc.num_to_remove(0.6, 16, 128)
    Wo, Mo = orc.prune_unstructured(W, H32.astype(np.float64), 0.6, 64, 0.01)
    np.testing.assert_array_equal(Mg, Mo)


# --------------------------------------------------------------------------- dtypes, determinism
def test_fp16_weights_cast_output_and_determinism():
    from tests.gpu_util import gpu_prune
    W, H32 = _layer(128, 512, 2048, "f16", seed=8)
    Wg, Mg, info, Wc = gpu_prune(W, H32, mode="nm", n=2, m=4, B=128, cast=True)
    assert Wc.dtype == np.float16
    np.testing.assert_array_equal(Wc, Wg.astype(np.float16))
    Wo, Mo = orc.prune_nm(W, H32.astype(np.float64), 2, 4, 128, 0.01)
    ok = np.all(Mg == Mo, axis=1)
    assert ok.mean() > 0.98
    assert _rel(Wg[ok], Wo[ok]) < 1e-3
    W2, M2, _, _ = gpu_prune(W, H32, mode="nm", n=2, m=4, B=128, cast=True)
    np.testing.assert_array_equal(W2, Wg)
    np.testing.assert_array_equal(M2, Mg)
    a = gpu_prune(W, H32, mode="unstructured", p=0.5, B=128)
    b_ = gpu_prune(W, H32, mode="unstructured", p=0.5, B=128)
    np.testing.assert_array_equal(a[0], b_[0])
    np.testing.assert_array_equal(a[1], b_[1])


# --------------------------------------------------------------------------- several tiles
@pytest.mark.parametrize("mode", ["unstructured", "nm"])
def test_medium_layer_teacher_forced(mode):
    # 300 x 1024 spans several 128-tiles in both directions and 8 blocks.  The free-running
    # mask may differ from the float64 oracle at near-ties only; W_hat is compared under the
    # GPU's own mask (the oracle re-run with that mask forced).
    from tests.gpu_util import gpu_prune
    c, b, B = 300, 1024, 128
    W, H32 = _layer(c, b, 4096, "f16", seed=9)
    H = H32.astype(np.float64)
    print(f"medium {mode}", flush=True)
    if mode == "unstructured":
        Wg, Mg, info = gpu_prune(W, H32, mode=mode, p=0.5, B=B)
        Wo, Mo = orc.prune_fast(W, H, mode=mode, p=0.5, B=B, damp=0.01)
        assert int(Mg.sum()) == c * b // 2
    else:
        Wg, Mg, info = gpu_prune(W, H32, mode=mode, n=2, m=4, B=B)
        Wo, Mo = orc.prune_fast(W, H, mode=mode, n=2, m=4, B=B, damp=0.01)
        assert np.all(Mg.reshape(c, b // 4, 4).sum(axis=2) == 2)
    assert info == 0
    assert (Mg != Mo).mean() < 1e-4
    Wt, _ = orc.prune_fast(W, H, mode=mode, p=0.5, n=2, m=4, B=B, damp=0.01, mask_in=Mg)
    assert _rel(Wg, Wt) < 1e-3
    eo = orc.reconstruction_error(W, Wo, H)
    eg = orc.reconstruction_error(W, Wg.astype(np.float64), H)
    assert abs(eg - eo) <= 0.01 * eo


@pytest.mark.parametrize("B", [64, 128, 256])
def test_singular_row_system_is_reported(B):
    # A factor with a zero column makes G = U_kk^T U_kk singular in that column: the one row
    # whose mask contains it must be reported as -(row + 1); the three block sizes reach the
    # three per-row solvers (register tiles, 128 threads, LDS tiles).
    from tests.gpu_util import gpu_prune, gpu_factor
    c, b, bad_row, bad_col = 12, 2 * B, 3, 5
    W, H32 = _layer(c, b, 4 * b, "f32", seed=B)
    U, xn2, info = gpu_factor(H32, 0.01)
    assert info == 0
    U[:, bad_col] = 0.0
    rng = np.random.default_rng(B)
    M = (rng.random((c, b)) < 0.6).astype(np.uint8)
    M[:, bad_col] = 0
    M[bad_row, bad_col] = 1
    print(f"singular system B={B}", flush=True)
    Wg, Mg, info = gpu_prune(W, H32, mode="unstructured", p=0.5, B=B, mask_in=M, U=U, xnorm2=xn2)
    assert info == -(bad_row + 1)
    np.testing.assert_array_equal(Mg, M)
    ok = np.arange(c) != bad_row
    assert np.all(np.isfinite(Wg[ok]))
    assert np.all(Wg[ok][M[ok] == 1] == 0.0)


@pytest.mark.parametrize("p", [0.72, 0.85])
def test_block128_rows_split_between_two_solvers(p):
    # B = 128 unstructured: rows with at most 96 removed weights in a block go to the
    # one-wavefront matrix-core solver, the others to the 128-thread one.  p = 0.72 puts rows on
    # both sides of that limit in every block, p = 0.85 nearly all of them above it.
    from tests.gpu_util import gpu_prune
    c, b = 192, 512
    W, H32 = _layer(c, b, 2048, "f32", rho=0.7, seed=77)
    print(f"split solvers p={p}", flush=True)
    Wg, Mg, info = gpu_prune(W, H32, mode="unstructured", p=p, B=128)
    assert info == 0
    assert int(Mg.sum()) == orc.num_to_remove(p, c, b)
    per_block = Mg.reshape(c, b // 128, 128).sum(axis=2)
    assert per_block.max() > 96
    if p < 0.8:
        assert per_block.min() <= 96
    H = H32.astype(np.float64)
    Wt, _ = orc.prune_fast(W, H, mode="unstructured", p=p, B=128, damp=0.01, mask_in=Mg)
    assert np.all(Wg[Mg == 1] == 0.0)
    assert _rel(Wg, Wt) < 1e-3
    _, Mo = orc.prune_fast(W, H, mode="unstructured", p=p, B=128, damp=0.01)
    assert (Mg != Mo).mean() < 1e-3


# --------------------------------------------------------------------------- conditioning
@pytest.mark.parametrize("T,rho,damp,mode,B", [
    (512, 0.7, 0.01, "nm", 128),              # fewer tokens than channels: H is rank deficient
    (256, 0.9, 0.01, "unstructured", 128),    # rank 256 of 1024, strongly correlated channels
    (4096, 0.95, 0.001, "unstructured", 256),  # small damping, condition number > 1e4
    (4096, 0.7, 0.0001, "nm", 128),
])
def test_ill_conditioned_hessians(T, rho, damp, mode, B):
    """Damping is all that keeps these Hessians positive definite (condition numbers of the
    damped matrix 5e3 .. 4e4); the fp32 factor and solves must still give the oracle's W_hat."""
    from tests.gpu_util import gpu_prune
    c, b = 256, 1024
    W, H32 = _layer(c, b, T, "f16", rho=rho, seed=5)
    H = H32.astype(np.float64)
    kw = dict(n=2, m=4) if mode == "nm" else dict(p=0.5)
    print(f"ill-conditioned {mode} T={T} rho={rho} damping={damp} B={B}", flush=True)
    Wg, Mg, info = gpu_prune(W, H32, mode=mode, B=B, damp=damp, **kw)
    assert info == 0
    Wt, _ = orc.prune_fast(W, H, mode=mode, B=B, damp=damp, mask_in=Mg, **kw)
    assert np.all(Wg[Mg == 1] == 0.0)
    assert _rel(Wg, Wt) < 1e-3
    eo = orc.reconstruction_error(W, Wt, H)
    eg = orc.reconstruction_error(W, Wg.astype(np.float64), H)
    assert abs(eg - eo) <= 0.01 * eo


@pytest.mark.parametrize("mode", ["unstructured", "nm"])
def test_dead_input_channels(mode):
    """Input channels that are zero in every calibration token: H_jj = 0, so the metric of their
    weights is 0 and they go first (ties in (row, column) order); the damping alone keeps the
    Hessian positive definite.  No special case anywhere: masks as the oracle's, W_hat within
    the usual bound."""
    from tests.gpu_util import gpu_prune
    c, b, T, B = 96, 512, 2048, 128
    spec = LayerSpec("t", c=c, b=b, tokens=T, dtype="f16", rho=0.7, k_mix=16, seed=12)
    W, X = make_weight(spec), make_calibration(spec)
    dead = np.array([0, 5, 6, 130, 255, 256, 300, 511])        # 5 and 6 share a group of four
    X[:, dead] = 0
    H32 = orc.hessian(X).astype(np.float32)
    H = H32.astype(np.float64)
    assert np.all(np.diag(H)[dead] == 0.0)
    kw = dict(n=2, m=4) if mode == "nm" else dict(p=0.5)
    Wg, Mg, info = gpu_prune(W, H32, mode=mode, B=B, **kw)
    assert info == 0
    assert Mg[:, dead].all()                                   # every weight of a dead channel goes
    if mode == "nm":
        assert np.all(Mg.reshape(c, b // 4, 4).sum(axis=2) == 2)
        assert not Mg[:, [4, 7]].any()                         # the group 4..7 is used up by 5 and 6
    else:
        assert int(Mg.sum()) == c * b // 2
    Wo, Mo = orc.prune_fast(W, H, mode=mode, B=B, damp=0.01, **kw)
    ndiff = int((Mg != Mo).sum())
    assert ndiff <= 4, ndiff                                   # near-ties only (none at the dead channels)
    np.testing.assert_array_equal(Mg[:, dead], Mo[:, dead])
    Wt, _ = orc.prune_fast(W, H, mode=mode, B=B, damp=0.01, mask_in=Mg, **kw)
    assert np.all(Wg[Mg == 1] == 0.0)
    assert _rel(Wg, Wt) < 1e-3


# --------------------------------------------------------------------------- invariances
@pytest.mark.parametrize("mode", ["unstructured", "nm"])
def test_hessian_scale_does_not_matter(mode):
    """The update u R_hat^{-1} R and the order of the metric are unchanged by H -> kappa H when
    the damping is relative (Sec. 4.1 / 4.2: H enters as 2 X X^T, (2/d) sum or X X^T alike).
    With kappa a power of four every intermediate scales exactly (the factor by the power of
    two sqrt(kappa)), so the results are identical bit for bit."""
    from tests.gpu_util import gpu_prune
    W, H32 = _layer(200, 640, 2560, "f16", rho=0.7, seed=21)
    kw = dict(n=2, m=4) if mode == "nm" else dict(p=0.5)
    W1, M1, i1 = gpu_prune(W, H32, mode=mode, B=128, **kw)
    W2, M2, i2 = gpu_prune(W, (4.0 * H32).astype(np.float32), mode=mode, B=128, **kw)
    W3, M3, i3 = gpu_prune(W, (0.0625 * H32).astype(np.float32), mode=mode, B=128, **kw)
    assert i1 == i2 == i3 == 0
    np.testing.assert_array_equal(M1, M2)
    np.testing.assert_array_equal(W1, W2)
    np.testing.assert_array_equal(M1, M3)
    np.testing.assert_array_equal(W1, W3)


def test_nm_rows_are_independent():
    """n:m: rows only meet in the shared inverse, so permuting the rows of W permutes the rows
    of (W_hat, M) and changes nothing else (bit for bit: a row's arithmetic does not depend on
    which tile or wavefront it lands in)."""
    from tests.gpu_util import gpu_prune
    W, H32 = _layer(300, 512, 2048, "f16", rho=0.7, seed=22)
    perm = np.random.default_rng(0).permutation(W.shape[0])
    W1, M1, _ = gpu_prune(W, H32, mode="nm", n=2, m=4, B=128)
    W2, M2, _ = gpu_prune(np.ascontiguousarray(W[perm]), H32, mode="nm", n=2, m=4, B=128)
    np.testing.assert_array_equal(M1[perm], M2)
    np.testing.assert_array_equal(W1[perm], W2)
