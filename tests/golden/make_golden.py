#!/usr/bin/env python3
"""Writes the stored expected values under tests/golden/ by calling ONLY the CPU oracle.

    python tests/golden/make_golden.py

tiny_fit.json holds, for each cell, a tiny seeded problem (inputs included) and the oracle's H(Q),
beta and RMSE for it.  The paper prints no worked example (no H or beta values anywhere in its text),
so these are regression values of the oracle, not values from the paper; the oracle itself is pinned
by closed forms, library special cases and brute force in tests/test_oracle_*.py.
"""
import json
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

from oracle import fit as ofit  # noqa: E402


def main() -> None:
    out = {}
    for cell, L, kw in (("elman", 4, dict(w_scale=1.0, spectral_radius=0.9)),
                        ("lstm", 3, dict(w_scale=0.5, forget_bias=1.0)),
                        ("gru", 3, dict(w_scale=0.5, zero_bias=True)),
                        ("elman_diag", 3, dict(w_scale=0.5)),
                        ("fc_multilag", 3, dict(w_scale=0.3))):
        rng = np.random.default_rng([1911, 13252, L])
        N, Q, d, m = 12, 4, 2, 2
        X = rng.uniform(-1, 1, (N, Q, d)).astype(np.float32)
        T = rng.uniform(-1, 1, (N, m)).astype(np.float32)
        r = ofit.fit(cell, X, T, L, seed=424242, **kw)
        out[cell] = dict(L=L, seed=424242, init=kw, X=X.tolist(), T=T.tolist(),
                         W=r["W"].tolist(), U=r["U"].tolist(), b=r["b"].tolist(),
                         H=r["H"].tolist(), beta=r["beta"].tolist(), rmse=r["rmse"])
    with open(os.path.join(HERE, "tiny_fit.json"), "w") as f:
        json.dump(out, f, indent=1)


if __name__ == "__main__":
    main()
