"""Stored expected values: the oracle reproduces them (CPU) and the HIP path matches them (GPU)."""
import json
import os

import numpy as np
import pytest

from oracle import fit as ofit
from oracle import weights as oweights

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def load():
    with open(os.path.join(GOLDEN, "tiny_fit.json")) as f:
        return json.load(f)


def test_splitmix64_vectors_file():
    for line in open(os.path.join(GOLDEN, "splitmix64_vectors.txt")):
        if line.startswith("#") or not line.strip():
            continue
        seed, idx, val = (int(t) for t in line.split())
        assert int(oweights.splitmix64(seed, idx + 1)[idx]) == val


@pytest.mark.parametrize("cell", ["elman", "lstm", "gru", "elman_diag", "fc_multilag"])
def test_oracle_reproduces_stored_values(cell):
    g = load()[cell]
    X, T = np.array(g["X"], np.float32), np.array(g["T"], np.float32)
    r = ofit.fit(cell, X, T, g["L"], g["seed"], **g["init"])
    np.testing.assert_array_equal(r["W"], np.array(g["W"], np.float32))
    np.testing.assert_allclose(r["U"], np.array(g["U"], np.float32), rtol=2e-7)
    np.testing.assert_allclose(r["H"], np.array(g["H"]), atol=1e-12)
    np.testing.assert_allclose(r["beta"], np.array(g["beta"]), rtol=1e-9, atol=1e-12)
    assert abs(r["rmse"] - g["rmse"]) < 1e-12


@pytest.mark.gpu
@pytest.mark.parametrize("cell", ["elman", "lstm", "gru", "elman_diag", "fc_multilag"])
def test_hip_path_matches_stored_values(elm, cell):
    import torch
    g = load()[cell]
    X, T = np.array(g["X"], np.float32), np.array(g["T"], np.float32)
    res = elm.fit(cell, torch.from_numpy(X).cuda(), torch.from_numpy(T).cuda(), g["L"], g["seed"], **g["init"])
    H = np.array(g["H"])
    rms = np.sqrt(np.mean(H ** 2))
    assert np.all(np.abs(res.H.cpu().numpy() - H) <= 1e-5 * np.maximum(np.abs(H), rms))
    beta = np.array(g["beta"])
    np.testing.assert_allclose(res.beta64.cpu().numpy(), beta, rtol=0, atol=1e-4 * np.abs(beta).max())
    assert abs(res.stats.rmse - g["rmse"]) <= 1e-4 * g["rmse"]
    res.model.close()


def test_chaos_rmse_file_is_consistent_with_the_yardstick_module():
    """tests/golden/chaos_rmse.json (regenerated only by tests/golden/make_chaos_golden.py, 20 minutes of
    oracle time): one float64 RMSE, one float32-yardstick RMSE per summation order and three perturbed
    float64 RMSEs per configuration, all close to each other but not equal."""
    import synthdata
    from oracle import float32_yardstick as y32
    with open(os.path.join(GOLDEN, "chaos_rmse.json")) as f:
        g = json.load(f)
    assert sorted(g) == ["cfg4", "cfg5"]
    for name, v in g.items():
        cfg = synthdata.get_config(name)
        assert v["seed"] == cfg.seed and cfg.L + cfg.m <= v["N"] <= cfg.N
        assert [tuple(x) for x in v["variants"]] == [tuple(x) for x in y32.VARIANTS]
        assert len(v["rmse32"]) == len(y32.VARIANTS) and len(v["rmse64_perturbed"]) == 3
        r64 = v["rmse64"]
        dev = [abs(r - r64) / r64 for r in v["rmse32"] + v["rmse64_perturbed"]]
        assert 0.0 < max(dev) < 5e-3 and 0.1 < r64 < 1.0
