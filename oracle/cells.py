"""Oracle: hidden-matrix build H(Q) for the Elman, LSTM and GRU cells (float64).

Test infrastructure only; shares no code with the GPU path.

Conventions (the paper's section "RNN architectures" and Algorithm "S-R-ELM"):
  X  : [N, Q, d]   one window per sample, step t is X[:, t, :]
  W  : [d, k*L]    input weights, gate blocks side by side
  U  : [L, k*L]    recurrent weights
  b  : [k*L]       biases
  gate block order: LSTM (i, f, o, g), GRU (z, r, n), Elman one block (k = 1)
  the initial state is zero unless given; only the state after the last step
  enters the solve (step 3 of Algorithm "S-R-ELM" uses H(Q)).
Row i of the result is the final hidden state of sample i.  All arithmetic is
float64; inputs may be float32 and are promoted exactly.
"""
from __future__ import annotations

import numpy as np


def sigmoid(a: np.ndarray) -> np.ndarray:
    """Logistic function 1 / (1 + exp(-a)), evaluated without overflow."""
    a = np.asarray(a, dtype=np.float64)
    e = np.exp(-np.abs(a))
    return np.where(a >= 0, 1.0 / (1.0 + e), e / (1.0 + e))


def _prep(X, W, U, b, h0, steps):
    X = np.asarray(X, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    U = np.asarray(U, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    N, Q, d = X.shape
    L = U.shape[0]
    steps = Q if steps is None else int(steps)
    if not 0 <= steps <= Q:
        raise ValueError("steps must lie in [0, Q]")
    h = np.zeros((N, L)) if h0 is None else np.array(h0, dtype=np.float64)
    return X, W, U, b, N, L, steps, h


def hidden_elman(X, W, U, b, h0=None, steps=None):
    """Dense lag-1 Elman / fully connected cell with tanh.

    h_t = tanh(x_t W + h_{t-1} U + b): the paper's fully connected recurrence
    (section "Fully Connected RNN") restricted to the previous step only, which
    is what the benchmark configurations specify (dense recurrent matrix).
    With U = 0 it is the feed-forward ELM hidden layer of Eq. (h_comp).
    """
    X, W, U, b, N, L, steps, h = _prep(X, W, U, b, h0, steps)
    for t in range(steps):
        h = np.tanh(X[:, t, :] @ W + h @ U + b)
    return h


def hidden_lstm(X, W, U, b, h0=None, c0=None, steps=None, return_cell=False):
    """LSTM without peepholes (section "LSTM").

    in = sigma(.)_i, lambda = sigma(.)_f, o = sigma(.)_o, candidate = tanh(.)_g,
    each of x_t W_* + f(t-1) U_* + b_*;  c_t = lambda*c_{t-1} + in*candidate;
    f(t) = o * tanh(c_t).
    """
    X, W, U, b, N, L, steps, h = _prep(X, W, U, b, h0, steps)
    c = np.zeros((N, L)) if c0 is None else np.array(c0, dtype=np.float64)
    for t in range(steps):
        a = X[:, t, :] @ W + h @ U + b
        gi = sigmoid(a[:, 0 * L:1 * L])
        gf = sigmoid(a[:, 1 * L:2 * L])
        go = sigmoid(a[:, 2 * L:3 * L])
        gg = np.tanh(a[:, 3 * L:4 * L])
        c = gf * c + gi * gg
        h = go * np.tanh(c)
    return (h, c) if return_cell else h


def hidden_gru(X, W, U, b, h0=None, steps=None):
    """GRU in the paper's convention (section "GRU").

    z, r = sigma(x_t W_* + f(t-1) U_* + b_*);
    candidate = tanh(x_t W_n + (r * f(t-1)) U_n + b_n)   (reset applied before U_n);
    f(t) = (1 - z) * f(t-1) + z * candidate.
    """
    X, W, U, b, N, L, steps, h = _prep(X, W, U, b, h0, steps)
    for t in range(steps):
        x = X[:, t, :]
        azr = x @ W[:, :2 * L] + h @ U[:, :2 * L] + b[:2 * L]
        z = sigmoid(azr[:, :L])
        r = sigmoid(azr[:, L:])
        cand = np.tanh(x @ W[:, 2 * L:] + (r * h) @ U[:, 2 * L:] + b[2 * L:])
        h = (1.0 - z) * h + z * cand
    return h


def hidden_elman_diag(X, W, alpha, b, steps=None):
    """The paper's own Elman cell (section "Elman", Eq. hij_elman): every neuron feeds back only on
    itself, from all earlier steps of the window.

    h_j(t) = tanh( x(t) W[:, j] + b_j + sum_{k=1}^{t-1} alpha[j, k-1] h_j(t-k) ),  t = 1..steps,
    with alpha of shape [L, Q] (column k-1 holds the weight of lag k) and no state before t = 1.
    The printed equation and Algorithm "Basic-PR-ELM" omit the activation, index the bias by sample
    and let the lag loop include step t itself; this is the reading with g applied, a bias per
    neuron and strictly earlier steps only.
    """
    X = np.asarray(X, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    alpha = np.asarray(alpha, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    N, Q, d = X.shape
    L = W.shape[1]
    steps = Q if steps is None else int(steps)
    if not 0 <= steps <= Q or alpha.shape != (L, Q):
        raise ValueError("alpha must be [L, Q] and steps must lie in [0, Q]")
    hist = np.zeros((steps + 1, N, L))           # hist[t] = h(t), hist[0] unused (no state before t = 1)
    for t in range(1, steps + 1):
        a = X[:, t - 1, :] @ W + b
        if t > 1:
            # sum over the lags k = 1..t-1 of alpha[j, k-1] * h_j(t-k), taken in one array contraction:
            # past[k-1] = h(t-k)
            past = hist[t - 1:0:-1]
            a = a + np.einsum("knl,lk->nl", past, alpha[:, :t - 1])
        hist[t] = np.tanh(a)
    return hist[steps] if steps > 0 else np.zeros((N, L))


def hidden_fc_multilag(X, W, A, b, steps=None):
    """The paper's fully connected cell (section "Fully Connected RNN", Eq. hij_fc): every neuron is fed
    by every neuron's output of all earlier steps of the window.

    h(t) = tanh( x(t) W + b + sum_{k=1}^{t-1} h(t-k) A[k-1] ),   t = 1..steps,
    with A of shape [Q, L, L] (A[k-1][m, j] weighs neuron m's output of k steps ago into neuron j) and
    no state before t = 1; as for the Elman cell, g is applied, the bias is per neuron and only strictly
    earlier steps feed back, so A[Q-1] is never used.
    """
    X = np.asarray(X, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    A = np.asarray(A, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    N, Q, d = X.shape
    L = W.shape[1]
    steps = Q if steps is None else int(steps)
    if not 0 <= steps <= Q or A.shape != (Q, L, L):
        raise ValueError("A must be [Q, L, L] and steps must lie in [0, Q]")
    hist = np.zeros((steps + 1, N, L))           # hist[t] = h(t), hist[0] unused (no state before t = 1)
    for t in range(1, steps + 1):
        a = X[:, t - 1, :] @ W + b
        for k in range(1, t):
            a = a + hist[t - k] @ A[k - 1]
        hist[t] = np.tanh(a)
    return hist[steps] if steps > 0 else np.zeros((N, L))


GATES = {"elman": 1, "lstm": 4, "gru": 3, "elman_diag": 1, "fc_multilag": 1}


def hidden(cell: str, X, W, U, b, h0=None, c0=None, steps=None):
    """Dispatch on the cell name; returns the final hidden state [N, L]."""
    if cell == "elman":
        return hidden_elman(X, W, U, b, h0=h0, steps=steps)
    if cell == "lstm":
        return hidden_lstm(X, W, U, b, h0=h0, c0=c0, steps=steps)
    if cell == "gru":
        return hidden_gru(X, W, U, b, h0=h0, steps=steps)
    if cell == "elman_diag":
        if h0 is not None:
            raise ValueError("the multi-lag cell has no single initial state")
        return hidden_elman_diag(X, W, U, b, steps=steps)
    if cell == "fc_multilag":
        if h0 is not None:
            raise ValueError("the multi-lag cell has no single initial state")
        return hidden_fc_multilag(X, W, U, b, steps=steps)
    raise ValueError(f"unknown cell {cell!r}")


def hidden_chunked(cell: str, X, W, U, b, chunk: int = 8192, **kw):
    """Same as hidden() but over row chunks (rows are independent), for large N."""
    N = X.shape[0]
    L = np.asarray(W).shape[1] // GATES[cell]
    out = np.empty((N, L), dtype=np.float64)
    for s in range(0, N, chunk):
        e = min(N, s + chunk)
        sub = {k: (None if v is None else v[s:e]) if k in ("h0", "c0") else v for k, v in kw.items()}
        out[s:e] = hidden(cell, X[s:e], W, U, b, **sub)
    return out
