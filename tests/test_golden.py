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
