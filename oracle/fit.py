"""Oracle: Algorithm "S-R-ELM" end to end (weights -> H(Q) -> beta) and prediction.

Test infrastructure only; shares no code with the GPU path.
"""
from __future__ import annotations

import numpy as np

from . import cells, lstsq, weights


def fit(cell: str, X, T, L: int, seed: int, *, w_scale=1.0, spectral_radius=0.0,
        forget_bias=0.0, zero_bias=False, chunk: int = 8192):
    """Steps 1-3 of Algorithm "S-R-ELM".

    Returns a dict with W, U, b (float32), H (float64), beta [L, m] (float64),
    rss and rmse = sqrt(rss / (N m)).
    """
    X = np.asarray(X)
    T = np.asarray(T)
    if T.ndim == 1:
        T = T[:, None]
    N, Q, d = X.shape
    W, U, b = weights.draw(cell, d, L, seed, w_scale, spectral_radius, forget_bias, zero_bias, Q=Q)
    H = cells.hidden_chunked(cell, X, W, U, b, chunk=chunk)
    if N <= chunk:
        beta, rss, R = lstsq.solve(H, T)
    else:
        beta, rss, R = lstsq.solve_chunked(H, T, chunk=chunk)
    return dict(W=W, U=U, b=b, H=H, beta=beta, rss=rss, R=R,
                rmse=lstsq.rmse_from_rss(rss, N, T.shape[1]))


def predict(cell: str, X, W, U, b, beta, chunk: int = 8192):
    """Output equation y_hat = sum_i beta_i f_i(Q) for every window."""
    H = cells.hidden_chunked(cell, np.asarray(X), W, U, b, chunk=chunk)
    return H @ np.asarray(beta, dtype=np.float64)
