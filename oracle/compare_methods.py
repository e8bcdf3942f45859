"""Reconstruction error ||(W_hat - W) X||_F^2 of magnitude pruning, Wanda, SparseGPT and Thanos
(all float64 CPU oracles) on seeded synthetic layers; prints a Markdown table.

    python -m oracle.compare_methods
"""
from __future__ import annotations

import numpy as np

from synth import LayerSpec, make_calibration, make_weight

from . import comparators as cmp
from . import thanos_oracle as orc


def main():
    print("| layer | pattern | magnitude | Wanda | SparseGPT | Thanos |")
    print("|---|---|---|---|---|---|")
    for (c, b, rho, outl) in [(256, 512, 0.7, False), (256, 512, 0.0, False), (256, 512, 0.7, True)]:
        spec = LayerSpec("cmp", c=c, b=b, tokens=4 * b, dtype="f16", rho=rho, k_mix=16, seed=1,
                         outliers=outl)
        W = make_weight(spec).astype(np.float64)
        H = orc.hessian(make_calibration(spec))
        name = f"{c}x{b}, rho={rho}" + (", outlier channels" if outl else "")
        for pat in ("50 % unstructured", "2:4", "4:8"):
            if pat.startswith("50"):
                kw = dict(p=0.5)
                th = orc.prune_fast(W, H, mode="unstructured", p=0.5, B=128, damp=0.01)[0]
            else:
                n, m = (2, 4) if pat == "2:4" else (4, 8)
                kw = dict(n=n, m=m)
                th = orc.prune_fast(W, H, mode="nm", n=n, m=m, B=128, damp=0.01)[0]
            errs = [orc.reconstruction_error(W, f(W, H, **kw)[0] if f is not orc.magnitude_prune
                                             else f(W, **kw)[0], H)
                    for f in (orc.magnitude_prune, cmp.wanda_prune, cmp.sparsegpt_prune)]
            errs.append(orc.reconstruction_error(W, th, H))
            ref = errs[0]
            print(f"| {name} | {pat} | 1.000 | " + " | ".join(f"{e / ref:.3f}" for e in errs[1:]) + " |")


if __name__ == "__main__":
    main()
