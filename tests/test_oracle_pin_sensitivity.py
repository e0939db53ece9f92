"""The inputs the oracle's pins use make plausible mistakes visible (CPU only).

A pin that compares the oracle with an independent reference on inputs for which a mistake would
not change the result (a symmetric recurrent matrix hides a transposition, equal gate blocks hide a
swapped gate order, a zero bias hides a dropped bias, a constant window hides a wrong step order)
proves nothing.  Each case below plants one such mistake in the *call* of the oracle, on inputs drawn
exactly as the pins draw theirs, and requires the result to move by far more than any tolerance the
pins use (1e-13 .. 1e-14): had the oracle made that mistake, its pin would have failed.
"""
import numpy as np
import pytest

from oracle import cells
from oracle import lstsq


def rnd(shape, seed, scale=1.0):
    return np.random.default_rng(seed).uniform(-scale, scale, size=shape)


def blocks(M, L, order):
    """Column blocks of width L re-ordered."""
    return np.concatenate([M[..., g * L:(g + 1) * L] for g in order], axis=-1)


def block_transposed(U, L):
    """Every L x L column block of the recurrent matrix transposed."""
    return np.concatenate([U[:, g * L:(g + 1) * L].T for g in range(U.shape[1] // L)], axis=1)


DENSE = {"elman": 1, "lstm": 4, "gru": 3}


@pytest.mark.parametrize("cell", ["elman", "lstm", "gru"])
def test_dense_cells(cell):
    k = DENSE[cell]
    N, Q, d, L = 6, 7, 3, 5
    X, W, U, b = rnd((N, Q, d), 25), rnd((d, k * L), 26), rnd((L, k * L), 27, 0.7), rnd(k * L, 28)
    ref = cells.hidden(cell, X, W, U, b)
    mistakes = {
        "transposed recurrent blocks": (X, W, block_transposed(U, L), b),
        "recurrent term with the wrong sign": (X, W, -U, b),
        "bias dropped": (X, W, U, np.zeros_like(b)),
        "steps in reverse order": (X[:, ::-1], W, U, b),
        "input weights of the last channel dropped": (X, np.vstack([W[:-1], np.zeros((1, k * L))]), U, b),
        "one step too few": (X[:, :-1], W, U, b),
    }
    if k > 1:
        swap = list(range(k))
        swap[0], swap[1] = swap[1], swap[0]
        mistakes["first two gate blocks swapped"] = (X, blocks(W, L, swap), blocks(U, L, swap), blocks(b, L, swap))
        last = list(range(k))
        last[-1], last[-2] = last[-2], last[-1]
        mistakes["last two gate blocks swapped"] = (X, blocks(W, L, last), blocks(U, L, last), blocks(b, L, last))
    for what, (x, w, u, bb) in mistakes.items():
        got = cells.hidden(cell, x, w, u, bb)
        assert np.abs(got - ref).max() > 1e-3, what


def test_the_papers_elman_cell():
    N, Q, d, L = 3, 5, 2, 4
    X, W, alpha, b = rnd((N, Q, d), 78), rnd((d, L), 79), rnd((L, Q), 80), rnd(L, 81)
    ref = cells.hidden_elman_diag(X, W, alpha, b)
    mistakes = {
        "lags shifted by one": np.roll(alpha, 1, axis=1),
        "lags in reverse order": np.concatenate([alpha[:, Q - 2::-1], alpha[:, Q - 1:]], axis=1),
        "feedback with the wrong sign": -alpha,
        "neurons' lag rows exchanged": alpha[::-1],
        "only the first lag kept": np.concatenate([alpha[:, :1], np.zeros((L, Q - 1))], axis=1),
    }
    for what, a in mistakes.items():
        assert np.abs(cells.hidden_elman_diag(X, W, a, b) - ref).max() > 1e-3, what
    # the last column (lag Q) can never act: strictly earlier steps only
    a = alpha.copy()
    a[:, Q - 1] += 5.0
    np.testing.assert_array_equal(cells.hidden_elman_diag(X, W, a, b), ref)


def test_the_papers_fully_connected_cell():
    N, Q, d, L = 3, 4, 2, 3
    X, W, A, b = rnd((N, Q, d), 90), rnd((d, L), 91), rnd((Q, L, L), 92, 0.8), rnd(L, 93)
    ref = cells.hidden_fc_multilag(X, W, A, b)
    mistakes = {
        "lag matrices transposed": A.transpose(0, 2, 1),
        "lags shifted by one": np.roll(A, 1, axis=0),
        "feedback with the wrong sign": -A,
        "only the first lag kept": np.concatenate([A[:1], np.zeros((Q - 1, L, L))], axis=0),
    }
    for what, a in mistakes.items():
        assert np.abs(cells.hidden_fc_multilag(X, W, a, b) - ref).max() > 1e-3, what
    a = A.copy()
    a[Q - 1] += 5.0                      # lag Q never acts
    np.testing.assert_array_equal(cells.hidden_fc_multilag(X, W, a, b), ref)


def test_householder_solve():
    rng = np.random.default_rng(3)
    N, L, m = 40, 6, 2
    H, T = rng.standard_normal((N, L)), rng.standard_normal((N, m))
    beta, rss, _ = lstsq.solve(H, T)
    # the pins compare with (H^T H)^-1 H^T T: these inputs tell that apart from near misses
    near = {
        "H used without transposition in the projection": np.linalg.solve(H.T @ H, (H[:L] @ T[:L])),
        "targets' columns exchanged": lstsq.solve(H, T[:, ::-1])[0],
        "one row dropped": lstsq.solve(H[:-1], T[:-1])[0],
        "ridge term added": np.linalg.solve(H.T @ H + 1e-3 * np.eye(L), H.T @ T),
    }
    for what, bad in near.items():
        assert np.abs(bad - beta).max() > 1e-6, what
    assert abs(rss - np.sum((H @ beta - T) ** 2)) <= 1e-10 * rss
    assert abs(lstsq.solve(H, T[:, :1])[1] - rss) > 1e-3          # RSS sums over all outputs
