"""Pins for the float32 yardstick (CPU only): on contractive inputs every summation-order variant must
reproduce the float64 oracle to float32 rounding, element by element (a wrong gate, sign or index gives
differences of order one), the variants must really differ in rounding, and on the chaotic benchmark
weights their spread must be what makes an element-wise 1e-5 comparison at full Q meaningless."""
import numpy as np
import pytest

import synthdata
from oracle import cells, weights
from oracle import float32_yardstick as y32

GATES = {"elman": 1, "lstm": 4, "gru": 3}


def small_problem(cell, N, Q, d, L, seed):
    k = GATES[cell]
    rng = np.random.default_rng(seed)
    a = 0.5 / np.sqrt(L)
    W = rng.uniform(-1, 1, (d, k * L)).astype(np.float32)
    U = rng.uniform(-a, a, (L, k * L)).astype(np.float32)
    b = rng.uniform(-0.5, 0.5, k * L).astype(np.float32)
    X = rng.uniform(-1, 1, (N, Q, d)).astype(np.float32)
    return X, W, U, b


@pytest.mark.parametrize("cell", ["elman", "lstm", "gru"])
def test_every_variant_reproduces_the_float64_oracle_on_contractive_inputs(cell):
    X, W, U, b = small_problem(cell, N=40, Q=7, d=3, L=70, seed=5)
    at = [1, 2, 5, 7]
    results = []
    for pieces, reverse in y32.VARIANTS + ((70, True),):
        got = y32.hidden32_at(cell, X, W, U, b, at, pieces, reverse)
        assert sorted(got) == at
        for q in at:
            ref = cells.hidden(cell, X, W, U, b, steps=q)
            assert got[q].dtype == np.float32
            assert np.abs(got[q] - ref).max() <= 3e-6, (cell, pieces, reverse, q)
        results.append(got[7])
        np.testing.assert_array_equal(y32.hidden32(cell, X, W, U, b, pieces=pieces, reverse=reverse), got[7])
    # the variants are different roundings of the same numbers, not one evaluation repeated
    assert any(not np.array_equal(results[0], r) for r in results[1:])


def test_initial_state_and_segments_chain():
    X, W, U, b = small_problem("lstm", N=10, Q=6, d=2, L=16, seed=6)
    whole = y32.hidden32_at("lstm", X, W, U, b, [3, 6])
    h3, c3 = cells.hidden_lstm(X, W, U, b, steps=3, return_cell=True)
    tail = y32.hidden32_at("lstm", X[:, 3:], W, U, b, [3], h0=h3, c0=c3)[3]
    assert np.abs(tail - whole[6]).max() <= 2e-6
    with pytest.raises(ValueError):
        y32.hidden32_at("lstm", X, W, U, b, [4, 2])
    with pytest.raises(ValueError):
        y32.hidden32_at("elman_diag", X, W, U, b, [1])


@pytest.mark.parametrize("name,rows", [("cfg4", 96), ("cfg5", 48)])
def test_spread_on_the_chaotic_benchmark_weights(name, rows):
    """What the yardstick is for: at full Q the float32 variants are far from the float64 result and
    from each other, while after four steps they agree with it to 1e-5."""
    cfg = synthdata.get_config(name)
    _, X, _ = synthdata.make_problem(cfg, N=rows)
    W, U, b = weights.draw(cfg.cell, cfg.d, cfg.L, cfg.seed, cfg.w_scale, cfg.spectral_radius,
                           cfg.forget_bias, cfg.zero_bias)
    ref4 = cells.hidden(cfg.cell, X, W, U, b, steps=4)
    refQ = cells.hidden(cfg.cell, X, W, U, b)
    for pieces, reverse in y32.VARIANTS[:2]:
        got = y32.hidden32_at(cfg.cell, X, W, U, b, [4, cfg.Q], pieces, reverse)
        assert np.abs(got[4] - ref4).max() <= 1e-5
        assert np.quantile(np.abs(got[cfg.Q] - refQ), 0.99) > 1e-3
