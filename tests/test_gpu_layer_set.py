"""GPU: q/k/v-style layer set sharing one Hessian and one factorisation."""
import numpy as np
import pytest

from oracle import thanos_oracle as orc
from synth import LayerSpec, make_weight, make_calibration

pytestmark = pytest.mark.gpu


def test_layer_set_matches_separate_calls_and_oracle():
    import torch
    import paper_2504_05346_amd as th
    from tests.gpu_util import dev, gpu_prune
    b, T = 384, 2048
    specs = [LayerSpec(f"w{k}", c=c, b=b, tokens=T, dtype="f16", rho=0.7, k_mix=16, seed=30 + k)
             for k, c in enumerate((256, 128, 200))]
    X = make_calibration(specs[0])
    Ws = [make_weight(s) for s in specs]
    Xd = dev(X)
    res, Hd = th.prune_layer_set([dev(W) for W in Ws], [Xd[:1000], Xd[1000:]], mode=th.THANOS_NM,
                                 n=2, m=4, block_size=128, cast=True)
    torch.cuda.synchronize()
    Hl = Hd.cpu().numpy()
    H32 = (np.tril(Hl) + np.tril(Hl, -1).T).astype(np.float32)
    H = H32.astype(np.float64)
    assert np.linalg.norm(H - orc.hessian(X)) <= 1e-5 * np.linalg.norm(H)
    for W, r in zip(Ws, res):
        assert int(r["info"].item()) == 0
        Wg, Mg = r["W"].cpu().numpy(), r["mask"].cpu().numpy()
        # same result as a call that factors for itself
        Ws_, Ms_, info = gpu_prune(W, H32, mode="nm", n=2, m=4, B=128)
        assert info == 0
        np.testing.assert_array_equal(Mg, Ms_)
        np.testing.assert_array_equal(Wg, Ws_)
        np.testing.assert_array_equal(r["W_cast"].cpu().numpy(), Wg.astype(np.float16))
        # and the oracle under the same mask
        Wt, _ = orc.prune_fast(W, H, mode="nm", n=2, m=4, B=128, damp=0.01, mask_in=Mg)
        assert np.linalg.norm(Wg - Wt) <= 1e-3 * np.linalg.norm(Wt)
