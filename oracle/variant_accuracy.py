"""End-to-end error of the approximate derivative, q(saved tensor) - f'(x), for the three ways of saving the
indicator (packed mask, precision bit, sign bit), by the oracle alone (CPU; test infrastructure like the rest
of this folder):

    python -m oracle.variant_accuracy

x ~ N(0, 1.5^2) rounded to the storage dtype, 2^20 values per row; max-abs / relative L2 over the sample.
The paper prints no such figures (its Fig. 3 plots the approximation); these are what its method yields.
"""
import numpy as np

import oracle as O
from paper_2407_15545_amd import synth


def main(n=1 << 20, seed=0):
    rng = np.random.default_rng(seed)
    ones = np.ones(n)
    print("| kind, storage | packed mask | precision bit | sign bit |")
    print("|---|---|---|---|")
    for kind in ("gelu_erf", "gelu_tanh", "silu"):
        for dtype in ("fp32", "bf16"):
            x = synth.storage_to_f64(synth.to_storage((rng.standard_normal(n) * 1.5).astype(np.float32), dtype), dtype)
            exact = O.df(kind, x)
            _, ys, m = O.invact_fwd(kind, dtype, x)
            _, yp = O.pbit_fwd(kind, dtype, x)
            _, yt = O.sbit_fwd(kind, dtype, x)
            cells = []
            for q in (O.invact_bwd(kind, ys, m, ones), O.pbit_bwd(kind, dtype, yp, ones), O.sbit_bwd(kind, yt, ones)):
                d = q - exact
                cells.append(f"{np.max(np.abs(d)):.2e} / {np.sqrt(np.sum(d ** 2) / np.sum(exact ** 2)):.1e}")
            print(f"| {kind}, {dtype} | " + " | ".join(cells) + " |")


if __name__ == "__main__":
    main()
