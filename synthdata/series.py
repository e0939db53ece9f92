"""Synthetic series, windows and the five benchmark configurations.

The paper evaluates on ten public univariate time-series datasets (its table
"Benchmarks Description": 2.5 k to 998 k instances, Q in {10, 50, 3197}).  They
are not available offline, so seeded synthetic series of the same kind stand in
for them: sums of sinusoids plus autoregressive noise, cut into sliding windows
of Q steps whose target is the next value (one-step-ahead prediction, the task
of the paper's section "Time Series Prediction Benchmarks").

Recipe (every choice the configuration strings leave open is fixed here):
  * each channel = 3 sinusoids, period ~ U(8, 64) samples (real-valued),
    amplitude ~ U(0.2, 1), phase ~ U(0, 2*pi), plus AR(2) noise
    e_t = 0.6 e_{t-1} - 0.3 e_{t-2} + N(0, sigma^2);
  * d == 1: min-max scaled to [0, 1] over the whole generated series;
  * d > 1: channels mixed by a random d x d matrix with entries ~ U(-1, 1),
    then every channel z-scored over the whole series;
  * N + Q points are generated so that window i = series[i : i+Q] always has a
    next value series[i+Q]; targets are the first m channels of that value.
All random draws come from numpy.random.default_rng([seed, 0]).
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np
from scipy.signal import lfilter


@dataclass(frozen=True)
class ElmConfig:
    name: str
    cell: str            # "elman" | "lstm" | "gru" | "elman_diag" | "fc_multilag"
    N: int               # number of windows (training samples)
    Q: int               # steps per window
    d: int               # input channels
    L: int               # hidden neurons
    m: int               # outputs
    w_scale: float       # weights ~ U(-w_scale, w_scale)
    spectral_radius: float   # > 0: recurrent matrix rescaled to this radius
    forget_bias: float   # added to LSTM forget-gate biases
    zero_bias: bool      # all biases exactly zero
    ar_sigma: float      # std of the AR(2) innovation
    seed: int            # master seed (data and weights)


CONFIGS = (
    ElmConfig("cfg1", "elman", 2_000, 10, 1, 32, 1, 1.0, 0.9, 0.0, False, 0.05, 13252),
    ElmConfig("cfg2", "elman", 100_000, 20, 1, 100, 1, 1.0, 0.9, 0.0, False, 0.05, 13253),
    ElmConfig("cfg3", "lstm", 200_000, 50, 4, 128, 1, 0.5, 0.0, 1.0, False, 0.05, 13254),
    ElmConfig("cfg4", "gru", 1_000_000, 50, 4, 256, 4, 0.5, 0.0, 0.0, True, 0.05, 13255),
    ElmConfig("cfg5", "lstm", 4_000_000, 100, 8, 512, 2, 0.3, 0.0, 1.0, False, 0.1, 13256),
)


# Workloads beyond the five benchmark configurations (same generator): the paper's own Elman cell
# (diagonal feedback over all earlier steps) at the shape of its largest runs (about 1e6 instances,
# Q = 50, M = 100, univariate).
EXTRA_CONFIGS = (
    ElmConfig("paper_elman", "elman_diag", 1_000_000, 50, 1, 100, 1, 0.3, 0.0, 0.0, False, 0.05, 13257),
    # the paper's fully connected multi-lag cell at Q = 10 (the window of most of its datasets), M = 100
    ElmConfig("paper_fc", "fc_multilag", 1_000_000, 10, 4, 100, 1, 0.1, 0.0, 0.0, False, 0.05, 13258),
    # ... and at the window of its three largest datasets, Q = 50, with about their 70 % training share of
    # 1e6 instances (the history of a window no longer fits on chip: one launch per step)
    ElmConfig("paper_fc_q50", "fc_multilag", 700_000, 50, 4, 100, 1, 0.05, 0.0, 0.0, False, 0.05, 13259),
)


def get_config(name: str) -> ElmConfig:
    for c in CONFIGS + EXTRA_CONFIGS:
        if c.name == name:
            return c
    raise KeyError(name)


def make_series(n_points: int, d: int, seed: int, ar_sigma: float) -> np.ndarray:
    """Return a float64 array [n_points, d] following the recipe above."""
    rng = np.random.default_rng([seed, 0])
    t = np.arange(n_points, dtype=np.float64)
    chans = np.empty((n_points, d), dtype=np.float64)
    for ch in range(d):
        period = rng.uniform(8.0, 64.0, size=3)
        amp = rng.uniform(0.2, 1.0, size=3)
        phase = rng.uniform(0.0, 2.0 * np.pi, size=3)
        s = np.zeros(n_points, dtype=np.float64)
        for k in range(3):
            s += amp[k] * np.sin(2.0 * np.pi * t / period[k] + phase[k])
        innov = rng.normal(0.0, ar_sigma, size=n_points)
        noise = lfilter([1.0], [1.0, -0.6, 0.3], innov)
        chans[:, ch] = s + noise
    if d == 1:
        lo, hi = chans.min(), chans.max()
        return (chans - lo) / (hi - lo)
    mix = rng.uniform(-1.0, 1.0, size=(d, d))
    mixed = chans @ mix
    mixed -= mixed.mean(axis=0, keepdims=True)
    mixed /= mixed.std(axis=0, keepdims=True)
    return mixed


def make_windows(series32: np.ndarray, N: int, Q: int, m: int, materialise: bool = True):
    """Cut a float32 series [N+Q, d] into X [N, Q, d] and T [N, m].

    With materialise=False X is a zero-copy strided view of the series.
    """
    n_points, d = series32.shape
    if n_points < N + Q:
        raise ValueError("series too short for N windows of Q steps plus a target")
    if m > d:
        raise ValueError("m targets need m channels")
    es = series32.strides
    X = np.lib.stride_tricks.as_strided(series32, shape=(N, Q, d),
                                        strides=(es[0], es[0], es[1]), writeable=False)
    if materialise:
        X = np.ascontiguousarray(X)
    T = np.ascontiguousarray(series32[Q:Q + N, :m])
    return X, T


def make_problem(cfg: ElmConfig, N: int | None = None, materialise: bool = True):
    """Series (float32), X, T for a configuration; N may be reduced for tests.

    The series is generated from the configuration's own seed with N + Q
    points; a reduced N therefore gives a shorter series of the same kind (its
    scaling statistics are those of the shorter series).
    """
    n = cfg.N if N is None else N
    series = make_series(n + cfg.Q, cfg.d, cfg.seed, cfg.ar_sigma).astype(np.float32)
    X, T = make_windows(series, n, cfg.Q, cfg.m, materialise)
    return series, X, T
