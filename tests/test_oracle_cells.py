"""Pins for the oracle's cell recurrences (CPU only).

Each pin is independent of oracle/cells.py's own formula: closed forms,
scalar hand iterations, torch's library cells in float64, and element-wise
brute force written from the paper's equations with explicit loops.
"""
import math

import numpy as np
import pytest
import torch

from oracle import cells


def rnd(shape, seed, scale=1.0):
    return np.random.default_rng(seed).uniform(-scale, scale, size=shape)


# ----------------------------------------------------------------- Elman

def test_elman_zero_recurrence_is_feedforward_elm():
    # Eq. (h_comp): H_ij = g(w_j^T x_i + b_j); with U = 0 only the last step matters
    N, Q, d, L = 7, 5, 3, 4
    X, W, b = rnd((N, Q, d), 1), rnd((d, L), 2), rnd(L, 3)
    H = cells.hidden_elman(X, W, np.zeros((L, L)), b)
    ref = np.array([[math.tanh(sum(W[s, j] * X[i, Q - 1, s] for s in range(d)) + b[j])
                     for j in range(L)] for i in range(N)])
    np.testing.assert_allclose(H, ref, rtol=0, atol=1e-15)


def test_elman_single_step():
    N, d, L = 5, 2, 3
    X, W, U, b = rnd((N, 1, d), 4), rnd((d, L), 5), rnd((L, L), 6), rnd(L, 7)
    H = cells.hidden_elman(X, W, U, b)
    np.testing.assert_allclose(H, np.tanh(X[:, 0, :] @ W + b), atol=1e-15)


def test_elman_scalar_iteration_by_hand():
    w, u, b = 0.7, -0.4, 0.1
    x = [0.3, -0.2, 0.9, 0.5]
    h = 0.0
    for xt in x:
        h = math.tanh(w * xt + u * h + b)
    H = cells.hidden_elman(np.array(x).reshape(1, 4, 1), [[w]], [[u]], [b])
    assert abs(H[0, 0] - h) < 1e-15


def test_elman_diagonal_recurrence_decouples_neurons():
    # W = 0, U = u I: every neuron runs the scalar map h <- tanh(u h + b_j)
    L, Q, u = 4, 6, 0.8
    b = rnd(L, 8)
    H = cells.hidden_elman(np.zeros((2, Q, 1)), np.zeros((1, L)), u * np.eye(L), b)
    for j in range(L):
        h = 0.0
        for _ in range(Q):
            h = math.tanh(u * h + b[j])
        assert abs(H[0, j] - h) < 1e-15 and abs(H[1, j] - h) < 1e-15


def test_elman_dense_brute_force_catches_transposed_recurrence():
    # element-wise loops: a_j = sum_s W[s,j] x_s + sum_l U[l,j] h_l + b_j
    N, Q, d, L = 3, 4, 2, 3
    X, W, U, b = rnd((N, Q, d), 9), rnd((d, L), 10), rnd((L, L), 11), rnd(L, 12)
    ref = np.zeros((N, L))
    for i in range(N):
        h = [0.0] * L
        for t in range(Q):
            h = [math.tanh(sum(W[s][j] * X[i, t, s] for s in range(d))
                           + sum(U[l][j] * h[l] for l in range(L)) + b[j]) for j in range(L)]
        ref[i] = h
    np.testing.assert_allclose(cells.hidden_elman(X, W, U, b), ref, atol=1e-14)
    # the asymmetric U makes the transposed product visibly different
    assert np.abs(cells.hidden_elman(X, W, U.T, b) - ref).max() > 1e-3


def test_truncated_steps_and_initial_state_compose():
    N, Q, d, L = 4, 6, 2, 5
    X, W, U, b = rnd((N, Q, d), 13), rnd((d, L), 14), rnd((L, L), 15, 0.5), rnd(L, 16)
    full = cells.hidden_elman(X, W, U, b)
    h3 = cells.hidden_elman(X, W, U, b, steps=3)
    rest = cells.hidden_elman(X[:, 3:, :], W, U, b, h0=h3)
    np.testing.assert_allclose(rest, full, atol=1e-15)


# ----------------------------------------------------------------- LSTM

def sig(a):
    return 1.0 / (1.0 + math.exp(-a))


def test_lstm_single_step_closed_form():
    N, d, L = 4, 3, 5
    X, W, U, b = rnd((N, 1, d), 20), rnd((d, 4 * L), 21), rnd((L, 4 * L), 22), rnd(4 * L, 23)
    H = cells.hidden_lstm(X, W, U, b)
    a = X[:, 0, :] @ W + b
    for i in range(N):
        for j in range(L):
            c = sig(a[i, j]) * math.tanh(a[i, 3 * L + j])          # c(0) = 0: forget term drops
            ref = sig(a[i, 2 * L + j]) * math.tanh(c)
            assert abs(H[i, j] - ref) < 1e-15


def test_lstm_constant_gates_geometric_closed_form():
    # W = U = 0: gates constant, c_Q = i g (1 - f^Q) / (1 - f), h_Q = o tanh(c_Q)
    L, Q = 6, 9
    b = rnd(4 * L, 24, 1.5)
    H, C = cells.hidden_lstm(np.zeros((1, Q, 2)), np.zeros((2, 4 * L)), np.zeros((L, 4 * L)), b,
                             return_cell=True)
    for j in range(L):
        i_, f_, o_, g_ = sig(b[j]), sig(b[L + j]), sig(b[2 * L + j]), math.tanh(b[3 * L + j])
        cq = i_ * g_ * (1.0 - f_ ** Q) / (1.0 - f_)
        assert abs(C[0, j] - cq) < 1e-14
        assert abs(H[0, j] - o_ * math.tanh(cq)) < 1e-14


def test_lstm_matches_torch_float64_with_permuted_gates():
    N, Q, d, L = 6, 7, 3, 5
    X, W, U, b = rnd((N, Q, d), 25), rnd((d, 4 * L), 26), rnd((L, 4 * L), 27, 0.7), rnd(4 * L, 28)
    lstm = torch.nn.LSTM(d, L, batch_first=True).double()
    # torch rows are (i, f, g, o); ours are column blocks (i, f, o, g)
    perm = np.concatenate([np.arange(0, L), np.arange(L, 2 * L), np.arange(3 * L, 4 * L),
                           np.arange(2 * L, 3 * L)])
    with torch.no_grad():
        lstm.weight_ih_l0.copy_(torch.from_numpy(W.T[perm].copy()))
        lstm.weight_hh_l0.copy_(torch.from_numpy(U.T[perm].copy()))
        lstm.bias_ih_l0.copy_(torch.from_numpy(b[perm].copy()))
        lstm.bias_hh_l0.zero_()
        _, (hn, cn) = lstm(torch.from_numpy(X))
    H, C = cells.hidden_lstm(X, W, U, b, return_cell=True)
    np.testing.assert_allclose(H, hn[0].numpy(), atol=1e-13)
    np.testing.assert_allclose(C, cn[0].numpy(), atol=1e-13)


def test_lstm_brute_force_from_the_equations():
    # the paper's names: o, c, lambda, in; every gate reads f(t-1), none reads c
    N, Q, d, L = 2, 3, 2, 3
    X, W, U, b = rnd((N, Q, d), 29), rnd((d, 4 * L), 30), rnd((L, 4 * L), 31), rnd(4 * L, 32)

    def pre(blk, j, x, f):
        col = blk * L + j
        return sum(W[s][col] * x[s] for s in range(d)) + sum(U[l][col] * f[l] for l in range(L)) + b[col]

    ref = np.zeros((N, L))
    for i in range(N):
        f = [0.0] * L
        c = [0.0] * L
        for t in range(Q):
            x = X[i, t]
            inn = [sig(pre(0, j, x, f)) for j in range(L)]
            lam = [sig(pre(1, j, x, f)) for j in range(L)]
            o = [sig(pre(2, j, x, f)) for j in range(L)]
            cand = [math.tanh(pre(3, j, x, f)) for j in range(L)]
            c = [lam[j] * c[j] + inn[j] * cand[j] for j in range(L)]
            f = [o[j] * math.tanh(c[j]) for j in range(L)]
        ref[i] = f
    np.testing.assert_allclose(cells.hidden_lstm(X, W, U, b), ref, atol=1e-14)


# ----------------------------------------------------------------- GRU

def test_gru_single_step_closed_form():
    N, d, L = 4, 3, 5
    X, W, U, b = rnd((N, 1, d), 40), rnd((d, 3 * L), 41), rnd((L, 3 * L), 42), rnd(3 * L, 43)
    H = cells.hidden_gru(X, W, U, b)
    a = X[:, 0, :] @ W + b
    for i in range(N):
        for j in range(L):
            assert abs(H[i, j] - sig(a[i, j]) * math.tanh(a[i, 2 * L + j])) < 1e-15


def test_gru_constant_gates_closed_form():
    # W = U = 0: h_Q = cand (1 - (1 - z)^Q)
    L, Q = 5, 8
    b = rnd(3 * L, 44, 1.5)
    H = cells.hidden_gru(np.zeros((1, Q, 1)), np.zeros((1, 3 * L)), np.zeros((L, 3 * L)), b)
    for j in range(L):
        z, cand = sig(b[j]), math.tanh(b[2 * L + j])
        assert abs(H[0, j] - cand * (1.0 - (1.0 - z) ** Q)) < 1e-14


def test_gru_diagonal_candidate_matches_torch_with_negated_update_gate():
    # torch: h' = (1-z)n + z h, n = tanh(W x + b + r*(U_n h)); the paper: h' = (1-z)h + z n with
    # n = tanh(W x + U_n (r*h) + b).  Equal when U_n is diagonal and the z gate is negated.
    N, Q, d, L = 5, 6, 2, 4
    X, W, b = rnd((N, Q, d), 45), rnd((d, 3 * L), 46), rnd(3 * L, 47)
    U = rnd((L, 3 * L), 48, 0.8)
    U[:, 2 * L:] = np.diag(rnd(L, 49))
    gru = torch.nn.GRU(d, L, batch_first=True).double()
    # torch rows are (r, z, n); ours are column blocks (z, r, n)
    Wt, Ut, bt = W.T.copy(), U.T.copy(), b.copy()
    w_ih = np.concatenate([Wt[L:2 * L], -Wt[0:L], Wt[2 * L:]])
    w_hh = np.concatenate([Ut[L:2 * L], -Ut[0:L], Ut[2 * L:]])
    b_ih = np.concatenate([bt[L:2 * L], -bt[0:L], bt[2 * L:]])
    with torch.no_grad():
        gru.weight_ih_l0.copy_(torch.from_numpy(w_ih))
        gru.weight_hh_l0.copy_(torch.from_numpy(w_hh))
        gru.bias_ih_l0.copy_(torch.from_numpy(b_ih))
        gru.bias_hh_l0.zero_()
        _, hn = gru(torch.from_numpy(X))
    np.testing.assert_allclose(cells.hidden_gru(X, W, U, b), hn[0].numpy(), atol=1e-13)


def test_gru_brute_force_reset_before_recurrent_product():
    N, Q, d, L = 2, 4, 2, 3
    X, W, U, b = rnd((N, Q, d), 50), rnd((d, 3 * L), 51), rnd((L, 3 * L), 52), rnd(3 * L, 53)
    ref = np.zeros((N, L))
    wrong = np.zeros((N, L))          # reset applied after U_n (torch's order): must differ
    for i in range(N):
        for variant, out in ((0, ref), (1, wrong)):
            f = [0.0] * L
            for t in range(Q):
                x = X[i, t]

                def pre(blk, j, vec):
                    col = blk * L + j
                    return (sum(W[s][col] * x[s] for s in range(d))
                            + sum(U[l][col] * vec[l] for l in range(L)) + b[col])
                z = [sig(pre(0, j, f)) for j in range(L)]
                r = [sig(pre(1, j, f)) for j in range(L)]
                if variant == 0:
                    rf = [r[l] * f[l] for l in range(L)]
                    cand = [math.tanh(pre(2, j, rf)) for j in range(L)]
                else:
                    cand = [math.tanh(sum(W[s][2 * L + j] * x[s] for s in range(d)) + b[2 * L + j]
                                      + r[j] * sum(U[l][2 * L + j] * f[l] for l in range(L)))
                            for j in range(L)]
                f = [(1.0 - z[j]) * f[j] + z[j] * cand[j] for j in range(L)]
            out[i] = f
    got = cells.hidden_gru(X, W, U, b)
    np.testing.assert_allclose(got, ref, atol=1e-14)
    assert np.abs(got - wrong).max() > 1e-3


# ----------------------------------------------------------------- shared

def test_sigmoid_is_stable_and_exact_at_known_points():
    a = np.array([-800.0, -30.0, 0.0, 30.0, 800.0, math.log(3.0)])
    s = cells.sigmoid(a)
    assert np.all(np.isfinite(s))
    assert s[0] == 0.0 and s[4] == 1.0 and s[2] == 0.5
    assert abs(s[5] - 0.75) < 1e-15
    np.testing.assert_allclose(s[1] + s[3], 1.0, atol=1e-15)


@pytest.mark.parametrize("cell,k", [("elman", 1), ("lstm", 4), ("gru", 3)])
def test_rows_are_independent_and_chunking_is_exact(cell, k):
    # rows of H do not interact (the paper's section "Basic Parallel Implementation")
    N, Q, d, L = 37, 5, 2, 6
    X, W, U, b = rnd((N, Q, d), 60), rnd((d, k * L), 61), rnd((L, k * L), 62, 0.5), rnd(k * L, 63)
    full = cells.hidden(cell, X, W, U, b)
    perm = np.random.default_rng(64).permutation(N)
    np.testing.assert_allclose(cells.hidden(cell, X[perm], W, U, b), full[perm], atol=1e-15)
    np.testing.assert_allclose(cells.hidden_chunked(cell, X, W, U, b, chunk=8), full, atol=1e-15)
    one = cells.hidden(cell, X[11:12], W, U, b)
    np.testing.assert_allclose(one[0], full[11], atol=1e-15)


# ----------------------------------------------------------------- the paper's own (diagonal, multi-lag) Elman

def test_elman_diag_without_feedback_is_feedforward_elm():
    N, Q, d, L = 5, 4, 3, 6
    X, W, b = rnd((N, Q, d), 70), rnd((d, L), 71), rnd(L, 72)
    H = cells.hidden_elman_diag(X, W, np.zeros((L, Q)), b)
    np.testing.assert_allclose(H, np.tanh(X[:, Q - 1, :] @ W + b), atol=1e-15)
    H1 = cells.hidden_elman_diag(X[:, :1], W, rnd((L, 1), 73), b)     # Q = 1: no earlier step exists
    np.testing.assert_allclose(H1, np.tanh(X[:, 0, :] @ W + b), atol=1e-15)


def test_elman_diag_lag_one_only_equals_the_dense_cell_with_a_diagonal_matrix():
    N, Q, d, L = 6, 7, 2, 5
    X, W, b = rnd((N, Q, d), 74), rnd((d, L), 75), rnd(L, 76)
    u = rnd(L, 77)
    alpha = np.zeros((L, Q))
    alpha[:, 0] = u
    np.testing.assert_allclose(cells.hidden_elman_diag(X, W, alpha, b),
                               cells.hidden_elman(X, W, np.diag(u), b), atol=1e-15)


def test_elman_diag_scalar_iteration_by_hand():
    # one neuron, three steps: h1 = g(w x1 + b); h2 = g(w x2 + b + a1 h1); h3 = g(w x3 + b + a1 h2 + a2 h1)
    w, b, a1, a2, a3 = 0.6, -0.1, 0.5, -0.7, 0.9
    x = [0.2, -0.4, 0.8]
    h1 = math.tanh(w * x[0] + b)
    h2 = math.tanh(w * x[1] + b + a1 * h1)
    h3 = math.tanh(w * x[2] + b + a1 * h2 + a2 * h1)
    H = cells.hidden_elman_diag(np.array(x).reshape(1, 3, 1), [[w]], [[a1, a2, a3]], [b])
    assert abs(H[0, 0] - h3) < 1e-15
    H2 = cells.hidden_elman_diag(np.array(x).reshape(1, 3, 1), [[w]], [[a1, a2, a3]], [b], steps=2)
    assert abs(H2[0, 0] - h2) < 1e-15


def test_elman_diag_brute_force_from_the_equation():
    N, Q, d, L = 3, 5, 2, 4
    X, W, alpha, b = rnd((N, Q, d), 78), rnd((d, L), 79), rnd((L, Q), 80), rnd(L, 81)
    ref = np.zeros((N, L))
    for i in range(N):
        for j in range(L):
            h = {}
            for t in range(1, Q + 1):
                a = sum(W[s][j] * X[i, t - 1, s] for s in range(d)) + b[j]
                a += sum(alpha[j][k - 1] * h[t - k] for k in range(1, t))
                h[t] = math.tanh(a)
            ref[i, j] = h[Q]
    got = cells.hidden_elman_diag(X, W, alpha, b)
    np.testing.assert_allclose(got, ref, atol=1e-14)
    # neurons do not interact: changing one neuron's alpha row changes only that column
    alpha2 = alpha.copy()
    alpha2[2] += 0.3
    got2 = cells.hidden_elman_diag(X, W, alpha2, b)
    assert np.abs(got2[:, 2] - got[:, 2]).max() > 1e-3
    np.testing.assert_array_equal(np.delete(got2, 2, axis=1), np.delete(got, 2, axis=1))


# ----------------------------------------------------------------- the paper's fully connected (dense, multi-lag) cell

def test_fc_multilag_with_lag_one_only_is_the_dense_elman_cell():
    N, Q, d, L = 6, 5, 2, 4
    X, W, b = rnd((N, Q, d), 90), rnd((d, L), 91), rnd(L, 92)
    A = np.zeros((Q, L, L))
    A[0] = rnd((L, L), 93)
    np.testing.assert_allclose(cells.hidden_fc_multilag(X, W, A, b), cells.hidden_elman(X, W, A[0], b), atol=1e-15)
    # no feedback at all, or a single step: the feed-forward ELM layer
    np.testing.assert_allclose(cells.hidden_fc_multilag(X, W, np.zeros((Q, L, L)), b),
                               np.tanh(X[:, Q - 1, :] @ W + b), atol=1e-15)
    np.testing.assert_allclose(cells.hidden_fc_multilag(X[:, :1], W, rnd((1, L, L), 94), b),
                               np.tanh(X[:, 0, :] @ W + b), atol=1e-15)


def test_fc_multilag_with_diagonal_lag_matrices_is_the_papers_elman_cell():
    N, Q, d, L = 5, 6, 3, 4
    X, W, b = rnd((N, Q, d), 95), rnd((d, L), 96), rnd(L, 97)
    alpha = rnd((L, Q), 98)
    A = np.stack([np.diag(alpha[:, k]) for k in range(Q)])
    np.testing.assert_allclose(cells.hidden_fc_multilag(X, W, A, b), cells.hidden_elman_diag(X, W, alpha, b),
                               atol=1e-15)


def test_fc_multilag_brute_force_from_the_equation():
    N, Q, d, L = 2, 4, 2, 3
    X, W, A, b = rnd((N, Q, d), 99), rnd((d, L), 100), rnd((Q, L, L), 101), rnd(L, 102)
    ref = np.zeros((N, L))
    for i in range(N):
        h = {}
        for t in range(1, Q + 1):
            h[t] = [0.0] * L
            for j in range(L):
                a = sum(W[s][j] * X[i, t - 1, s] for s in range(d)) + b[j]
                for k in range(1, t):
                    a += sum(A[k - 1][m][j] * h[t - k][m] for m in range(L))
                h[t][j] = math.tanh(a)
        ref[i] = h[Q]
    got = cells.hidden_fc_multilag(X, W, A, b)
    np.testing.assert_allclose(got, ref, atol=1e-14)
    # the last lag block is never used; a transposed lag matrix is a different network
    A2 = A.copy()
    A2[Q - 1] += 1.0
    np.testing.assert_array_equal(cells.hidden_fc_multilag(X, W, A2, b), got)
    A3 = A.copy()
    A3[1] = A3[1].T
    assert np.abs(cells.hidden_fc_multilag(X, W, A3, b) - got).max() > 1e-3
    np.testing.assert_allclose(cells.hidden_fc_multilag(X, W, A, b, steps=2),
                               np.tanh(X[:, 1] @ W + b + np.tanh(X[:, 0] @ W + b) @ A[0]), atol=1e-15)
