"""Oracle instrument: the dense cell recurrences evaluated in float32, in several summation orders.

Test infrastructure only; shares no code with the GPU path.

With the weight scales of the two largest benchmark configurations the LSTM and GRU maps amplify a
rounding error of one step over the rest of the window, so after Q = 50 or 100 steps ANY float32
evaluation differs from the float64 oracle by much more than float32 rounding.  How much is a property of
the map, not of an implementation, and this module measures it: the same equations as oracle/cells.py
(sections "Elman", "LSTM", "GRU": same gate order, same conventions), every operation rounded to float32,
with the recurrent contraction h U accumulated in `pieces` slices of its rows, taken first-to-last or
last-to-first.  The spread of these variants around the float64 result is the yardstick the GPU's
float32 kernels are held to on those configurations; it is never used as an expected value.

Pinned (tests/test_oracle_yardstick.py) against the float64 oracle on contractive inputs, where all
variants must agree with it to float32 rounding.
"""
from __future__ import annotations

import numpy as np

F = np.float32


def _sigmoid32(a: np.ndarray) -> np.ndarray:
    e = np.exp(-np.abs(a))
    one = F(1.0)
    return np.where(a >= 0, one / (one + e), e / (one + e)).astype(F)


def _contract32(h: np.ndarray, U: np.ndarray, pieces: int, reverse: bool) -> np.ndarray:
    """h U in float32, the rows of U taken in `pieces` slices whose partial products are added in order."""
    K = U.shape[0]
    edges = np.linspace(0, K, min(pieces, K) + 1).astype(int)
    spans = list(zip(edges[:-1], edges[1:]))
    if reverse:
        spans = spans[::-1]
    acc = None
    for lo, hi in spans:
        part = h[:, lo:hi] @ U[lo:hi]
        acc = part if acc is None else acc + part
    return acc


def hidden32_at(cell: str, X, W, U, b, at, pieces: int = 1, reverse: bool = False, h0=None, c0=None):
    """Final states after each step count in `at` (ascending, each <= Q): {q: H_q [N, L] float32}.

    cell in {"elman", "lstm", "gru"}; X [N, Q, d], W [d, kL], U [L, kL], b [kL] are rounded to float32 first
    (the benchmark's weights and windows already are).  Zero initial state unless h0 / c0 are given.
    """
    X = np.asarray(X, dtype=F)
    W = np.asarray(W, dtype=F)
    U = np.asarray(U, dtype=F)
    b = np.asarray(b, dtype=F)
    N, Q, d = X.shape
    L = U.shape[0]
    at = [int(q) for q in at]
    if at != sorted(at) or (at and (at[0] < 0 or at[-1] > Q)):
        raise ValueError("step counts must be ascending and lie in [0, Q]")
    h = np.zeros((N, L), F) if h0 is None else np.array(h0, dtype=F)
    c = np.zeros((N, L), F) if c0 is None else np.array(c0, dtype=F)
    out = {}
    if 0 in at:
        out[0] = h.copy()
    one = F(1.0)
    for t in range(at[-1] if at else 0):
        x = X[:, t, :]
        if cell == "elman":
            h = np.tanh((x @ W + b) + _contract32(h, U, pieces, reverse))
        elif cell == "lstm":
            a = (x @ W + b) + _contract32(h, U, pieces, reverse)
            gi = _sigmoid32(a[:, 0 * L:1 * L])
            gf = _sigmoid32(a[:, 1 * L:2 * L])
            go = _sigmoid32(a[:, 2 * L:3 * L])
            gg = np.tanh(a[:, 3 * L:4 * L])
            c = gf * c + gi * gg
            h = go * np.tanh(c)
        elif cell == "gru":
            azr = (x @ W[:, :2 * L] + b[:2 * L]) + _contract32(h, U[:, :2 * L], pieces, reverse)
            z = _sigmoid32(azr[:, :L])
            r = _sigmoid32(azr[:, L:])
            cand = np.tanh((x @ W[:, 2 * L:] + b[2 * L:]) + _contract32(r * h, U[:, 2 * L:], pieces, reverse))
            h = (one - z) * h + z * cand
        else:
            raise ValueError(f"no float32 yardstick for cell {cell!r}")
        assert h.dtype == F
        if t + 1 in at:
            out[t + 1] = h.copy()
    return out


def hidden32(cell: str, X, W, U, b, steps=None, pieces: int = 1, reverse: bool = False):
    """H(steps) in float32 (steps = Q by default)."""
    q = np.asarray(X).shape[1] if steps is None else int(steps)
    return hidden32_at(cell, X, W, U, b, [q], pieces, reverse)[q]


# the summation orders the yardstick is taken over: (pieces, reverse)
VARIANTS = ((1, False), (2, False), (4, True), (7, False))
