"""Full-window parity of the two largest benchmark configurations (and the LSTM one below them), whose maps
amplify a rounding error of one step over the rest of the window.

After Q = 50 or 100 steps any float32 evaluation of these recurrences is far from the float64 oracle
element by element, so "H within 1e-5" can only be asked on short horizons (tests/test_gpu_hidden.py).
What can be asked at full Q, with the configuration's own seeded windows and weights, is asked here:

  * the training RMSE of the GPU fit against the oracle's own fit (its float64 H, its Householder solve)
    at a number of windows the oracle can afford.  tests/golden/chaos_rmse.json (written by
    tests/golden/make_chaos_golden.py, which calls only oracle/) holds that RMSE and the RMSE of the same
    fit with H from the oracle's float32 yardstick in four summation orders: where those scatter by more
    than 1e-4 relative around the float64 value, no float32 path can do better, and the bar is three times
    their largest deviation (1e-4 otherwise);
  * the error of H against the float64 oracle, as quantiles over 1,024 windows after 4, 8, 16, 32, 64 and Q
    steps: at most twice the same quantile of the float32 yardstick (the worst of its summation orders);
    the largest single error, a noisy statistic, at most eight times.  A swapped gate, a dropped term or a
    biased activation late in the unroll moves these quantiles by orders of magnitude.
"""
import functools
import json
import os

import numpy as np
import pytest
import torch

import synthdata
from oracle import cells as ocells
from oracle import float32_yardstick as y32
from oracle import lstsq
from oracle import weights as oweights

pytestmark = pytest.mark.gpu

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "chaos_rmse.json")
MODES = ["fp32", "split16"]
QUANTILES = (0.5, 0.9, 0.99)


def cfg_kwargs(cfg):
    return dict(w_scale=cfg.w_scale, spectral_radius=cfg.spectral_radius,
                forget_bias=cfg.forget_bias, zero_bias=cfg.zero_bias)


def oracle_weights(cfg):
    return oweights.draw(cfg.cell, cfg.d, cfg.L, cfg.seed, cfg.w_scale, cfg.spectral_radius,
                         cfg.forget_bias, cfg.zero_bias)


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("name", ["cfg4", "cfg5"])
def test_training_rmse_against_the_oracles_own_fit_at_full_window_length(elm, name, mode):
    with open(GOLDEN) as f:
        g = json.load(f)[name]
    cfg = synthdata.get_config(name)
    N = g["N"]
    assert g["seed"] == cfg.seed
    _, X, T = synthdata.make_problem(cfg, N=N)
    Xd, Td = torch.from_numpy(X).cuda(), torch.from_numpy(T).cuda()
    res = elm.fit(cfg.cell, Xd, Td, cfg.L, cfg.seed, contraction=mode, **cfg_kwargs(cfg))
    # the stored values belong to the oracle's weights: the library's generator must give the same ones
    for got, want in zip(res.model.weights()[:3], oracle_weights(cfg)):
        np.testing.assert_array_equal(got, want)
    r64 = g["rmse64"]
    spread = max(abs(r - r64) for r in g["rmse32"]) / r64
    bar = max(1e-4, 3.0 * spread)
    assert abs(res.stats.rmse - r64) <= bar * r64, (res.stats.rmse, r64, bar)
    # stage-isolated, to the plain bars: the oracle's solve of the GPU's own H, and the residual of beta
    H = res.H.cpu().numpy()
    _, rss, _ = lstsq.solve_chunked(H, T, chunk=8192)
    iso = lstsq.rmse_from_rss(rss, N, cfg.m)
    assert abs(res.stats.rmse - iso) <= 1e-4 * iso
    assert lstsq.normal_equation_residual(H, T, res.beta64.cpu().numpy()) <= 1e-5
    res.model.close()


def step_counts(Q):
    return sorted({q for q in (4, 8, 16, 32, 64, Q) if q <= Q})


def oracle_states(cell, X, W, U, b, at):
    """Float64 final states after every step count in `at`, in one pass over the window: the oracle's
    cell function is continued from its own state segment by segment."""
    out, h, c, t0 = {}, None, None, 0
    for q in at:
        seg = X[:, t0:q]
        if cell == "lstm":
            h, c = ocells.hidden_lstm(seg, W, U, b, h0=h, c0=c, return_cell=True)
        else:
            h = ocells.hidden(cell, seg, W, U, b, h0=h)
        out[q], t0 = h, q
    return out


@functools.lru_cache(maxsize=None)
def yardstick(name, rows=1024):
    cfg = synthdata.get_config(name)
    _, X, _ = synthdata.make_problem(cfg, N=rows)
    W, U, b = oracle_weights(cfg)
    at = step_counts(cfg.Q)
    ref = oracle_states(cfg.cell, X, W, U, b, at)
    np.testing.assert_array_equal(ref[cfg.Q], ocells.hidden(cfg.cell, X, W, U, b))     # the segments chain exactly
    worst = {q: np.zeros(len(QUANTILES) + 1) for q in at}
    for pieces, reverse in y32.VARIANTS:
        got = y32.hidden32_at(cfg.cell, X, W, U, b, at, pieces, reverse)
        for q in at:
            e = np.abs(got[q].astype(np.float64) - ref[q])
            worst[q] = np.maximum(worst[q], np.append(np.quantile(e, QUANTILES), e.max()))
    return X, ref, worst


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("name", ["cfg3", "cfg4", "cfg5"])
def test_error_quantiles_per_step_count_follow_the_float32_yardstick(elm, name, mode):
    cfg = synthdata.get_config(name)
    X, ref, worst = yardstick(name)
    model = elm.Model.create(cfg.cell, cfg.Q, cfg.d, cfg.L, cfg.m, cfg.seed, contraction=mode, **cfg_kwargs(cfg))
    for got, want in zip(model.weights()[:3], oracle_weights(cfg)):
        np.testing.assert_array_equal(got, want)
    Xd = torch.from_numpy(X).cuda()
    rms = np.sqrt(np.mean(ref[cfg.Q] ** 2))
    for q in step_counts(cfg.Q):
        H = elm.hidden(model, Xd, Q_run=q).cpu().numpy().astype(np.float64)
        e = np.abs(H - ref[q])
        got = np.append(np.quantile(e, QUANTILES), e.max())
        # (an error below the element-wise bar of the short-horizon tests passes whatever the yardstick says)
        assert np.all(got[:-1] <= np.maximum(2.0 * worst[q][:-1], 1e-5 * rms)), (q, got, worst[q])
        assert got[-1] <= max(8.0 * worst[q][-1], 1e-5 * rms), (q, got, worst[q])
    # the yardstick itself says why full-Q element-wise parity is not asked of these maps
    if name != "cfg3":
        assert worst[cfg.Q][2] > 1e-2
    model.close()
