"""GPU parity: thanos_factor against the CPU oracle."""
import numpy as np
import pytest

from oracle import thanos_oracle as orc
from synth import LayerSpec, make_calibration

pytestmark = pytest.mark.gpu


def _h(b, T=None, rho=0.7, seed=0, outliers=False):
    X = make_calibration(LayerSpec("t", c=1, b=b, tokens=T or 4 * b, dtype="f16", rho=rho,
                                   k_mix=8, seed=seed, outliers=outliers))
    return orc.hessian(X).astype(np.float32)


@pytest.mark.parametrize("b", [128, 200, 512, 640, 1000, 1408, 2432])
def test_factor_matches_oracle(b):
    from tests.gpu_util import gpu_factor
    print(f"factor b={b}", flush=True)
    H32 = _h(b, seed=b)
    U, xn2, info = gpu_factor(H32, 0.01)
    assert info == 0
    np.testing.assert_array_equal(xn2, np.diag(H32))
    assert np.all(np.tril(U, -1) == 0.0)
    Hd = orc.damped(H32.astype(np.float64), 0.01)
    Uref = orc.inverse_factor(Hd)
    U64 = U.astype(np.float64)
    # fp32 factorisation: error ~ cond(scaled H_d) * 2^-24; these inputs have cond ~ 1e3
    assert np.linalg.norm(U64 - Uref) <= 2e-4 * np.linalg.norm(Uref)
    # defining property, independent of the oracle's route: U^T U H_d = I
    R = U64.T @ (U64 @ Hd) - np.eye(b)
    assert np.max(np.abs(R)) < 5e-3
    # every residual inverse (what Alg. 1 recomputes per block) is contained in U
    for j in (0, b // 3, b - 5):
        inv = np.linalg.inv(Hd[j:, j:])
        got = U64[j:, j:].T @ U64[j:, j:]
        assert np.linalg.norm(got - inv) <= 5e-4 * np.linalg.norm(inv)


def test_factor_heavy_tailed_channels():
    from tests.gpu_util import gpu_factor
    H32 = _h(640, seed=9, outliers=True)
    U, _, info = gpu_factor(H32, 0.01)
    assert info == 0
    Uref = orc.inverse_factor(orc.damped(H32.astype(np.float64), 0.01))
    assert np.linalg.norm(U - Uref) <= 5e-4 * np.linalg.norm(Uref)


def test_not_positive_definite_is_reported():
    from tests.gpu_util import gpu_factor
    H32 = _h(256, seed=1)
    H32[100, 100] = -1.0
    _, _, info = gpu_factor(H32, 0.0)
    assert info > 0
