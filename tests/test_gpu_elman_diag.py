"""GPU parity of the paper's own Elman cell (section "Elman": diagonal feedback over all earlier
steps of the window) against the float64 oracle, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import cells as ocells
from oracle import fit as ofit
from oracle import lstsq

pytestmark = pytest.mark.gpu


def h_close(got, ref, tol=1e-5):
    ref = np.asarray(ref, dtype=np.float64)
    rms = max(np.sqrt(np.mean(ref ** 2)), 1e-30)
    return np.all(np.abs(np.asarray(got, dtype=np.float64) - ref) <= tol * np.maximum(np.abs(ref), rms))


def weights(Q, d, L, seed):
    rng = np.random.default_rng(seed)
    return (rng.uniform(-1, 1, (d, L)).astype(np.float32) / np.float32(np.sqrt(d)),
            (rng.uniform(-1, 1, (L, Q)) / max(Q - 1, 1)).astype(np.float32),     # sum_k |alpha_jk| < 1
            rng.uniform(-0.5, 0.5, L).astype(np.float32))


# every unrolled variant (8, 16, 32, 64 steps) at and next to its limits, the LDS-history kernel
# from 65 to 128 steps, ragged sample and neuron tails, windows staged in LDS and read directly
@pytest.mark.parametrize("N,Q,d,L", [
    (1, 1, 1, 1), (63, 2, 3, 31), (64, 8, 1, 32), (65, 9, 2, 33), (200, 16, 4, 100), (130, 17, 1, 7),
    (1000, 20, 1, 50), (257, 32, 2, 64), (100, 33, 1, 40), (300, 50, 3, 20), (70, 64, 1, 36),
    (90, 65, 1, 10), (66, 100, 2, 5), (10, 512, 1, 3),
    (150, 40, 16, 12),      # 640 window elements per sample: past the LDS tile, read directly
    (129, 12, 64, 9),       # widest input
    (5000, 10, 1, 512),     # largest L, neurons split over the second grid dimension
    # long windows (time axis spread over the lanes of a wave): 16, 32 and 64 register slots per lane at
    # and next to their limits, odd and even sample counts, the paper's longest window (3,197 steps)
    (70, 128, 1, 6), (33, 129, 2, 7), (50, 300, 1, 5), (9, 513, 1, 3), (17, 1024, 2, 5), (8, 1025, 1, 2), (23, 2048, 1, 3), (11, 2049, 3, 2), (20, 3197, 1, 4),
    (5, 4096, 1, 2),
])
def test_hidden_matches_oracle(elm, N, Q, d, L):
    W, alpha, b = weights(Q, d, L, seed=N + Q + L)
    X = np.random.default_rng(N * 7 + Q).uniform(-1, 1, (N, Q, d)).astype(np.float32)
    model = elm.Model.from_weights("elman_diag", Q, 1, W, alpha, b)
    H = elm.hidden(model, torch.from_numpy(X).cuda()).cpu().numpy()
    ref = ocells.hidden_elman_diag(X, W, alpha, b)
    assert h_close(H, ref)
    model.close()


def test_fewer_steps_and_sliding_windows_without_copy(elm):
    Q, d, L, N = 24, 2, 45, 3000
    W, alpha, b = weights(Q, d, L, seed=5)
    series = np.random.default_rng(6).uniform(-1, 1, (N + Q - 1, d)).astype(np.float32)
    dev = torch.from_numpy(series).cuda()
    Xview = dev.as_strided((N, Q, d), (d, d, 1))              # window i starts at series row i
    Xh = np.lib.stride_tricks.sliding_window_view(series, (Q, d)).reshape(N, Q, d)
    model = elm.Model.from_weights("elman_diag", Q, 1, W, alpha, b)
    assert h_close(elm.hidden(model, Xview).cpu().numpy(), ocells.hidden_elman_diag(Xh, W, alpha, b))
    for q in (1, 7, 16, 23):
        got = elm.hidden(model, Xview, Q_run=q).cpu().numpy()
        assert h_close(got, ocells.hidden_elman_diag(Xh, W, alpha, b, steps=q)), q
    model.close()


def test_long_window_model_run_for_fewer_steps(elm):
    """A 3,197-step model unrolled for fewer steps goes through every kernel family of the cell."""
    Q, d, L, N = 3197, 1, 3, 37
    W, alpha, b = weights(Q, d, L, seed=11)
    alpha *= 40.0                                  # the early lags matter at short horizons too
    alpha[:, 60:] /= 40.0
    X = np.random.default_rng(12).uniform(-1, 1, (N, Q, d)).astype(np.float32)
    Xd = torch.from_numpy(X).cuda()
    model = elm.Model.from_weights("elman_diag", Q, 1, W, alpha, b)
    for q in (5, 64, 65, 128, 129, 513, 1500, 3000, 3197):
        got = elm.hidden(model, Xd, Q_run=q).cpu().numpy()
        assert h_close(got, ocells.hidden_elman_diag(X, W, alpha, b, steps=q)), q
    model.close()


def test_lag_one_only_agrees_with_the_dense_kernel_on_a_diagonal_matrix(elm):
    # two independent kernels of the library against each other and against the oracle
    Q, d, L, N = 12, 3, 70, 500
    W, alpha, b = weights(Q, d, L, seed=8)
    alpha[:, 1:] = 0
    alpha[:, 0] = np.random.default_rng(9).uniform(-0.9, 0.9, L).astype(np.float32)
    X = np.random.default_rng(10).uniform(-1, 1, (N, Q, d)).astype(np.float32)
    Xd = torch.from_numpy(X).cuda()
    m1 = elm.Model.from_weights("elman_diag", Q, 1, W, alpha, b)
    m2 = elm.Model.from_weights("elman", Q, 1, W, np.diag(alpha[:, 0]).astype(np.float32), b)
    H1, H2 = elm.hidden(m1, Xd).cpu().numpy(), elm.hidden(m2, Xd).cpu().numpy()
    ref = ocells.hidden_elman_diag(X, W, alpha, b)
    assert h_close(H1, ref) and h_close(H2, ref)
    m1.close(), m2.close()


# w_scale chosen per case so that H is neither nearly linear in x (tiny weights: cond(H) ~ 1e5) nor
# chaotic in float32 (large lag weights amplify rounding by > 1e4 over the window)
@pytest.mark.parametrize("N,Q,d,L,m,seed,w_scale", [(4000, 10, 1, 20, 1, 3, 0.5), (20000, 30, 2, 60, 2, 4, 0.2)])
def test_fit_matches_oracle_fit(elm, N, Q, d, L, m, seed, w_scale):
    rng = np.random.default_rng(seed)
    X = rng.uniform(-1, 1, (N, Q, d)).astype(np.float32)
    T = (np.sin(X.sum(axis=(1, 2)))[:, None] * np.arange(1, m + 1) + 0.05 * rng.standard_normal((N, m))
         ).astype(np.float32)
    res = elm.fit("elman_diag", torch.from_numpy(X).cuda(), torch.from_numpy(T).cuda(), L, seed=seed,
                  w_scale=w_scale)
    ref = ofit.fit("elman_diag", X, T, L, seed, w_scale=w_scale)
    W, U, b, beta = res.model.weights()
    assert np.array_equal(W, ref["W"]) and np.array_equal(U, ref["U"]) and np.array_equal(b, ref["b"])
    assert U.shape == (L, Q)
    assert h_close(res.H.cpu().numpy(), ref["H"])
    assert abs(res.stats.rmse - ref["rmse"]) <= 1e-4 * ref["rmse"]
    assert lstsq.normal_equation_residual(res.H.cpu().numpy(), T, beta) <= 1e-5
    Y = elm.predict(res.model, torch.from_numpy(X[:777]).cuda()).cpu().numpy()
    # |dY| <= |dH| sum|beta|: the H tolerance carried through the output equation
    np.testing.assert_allclose(Y, ref["H"][:777] @ beta, rtol=0,
                               atol=2e-5 * np.abs(beta).sum(axis=0).max() + 1e-5)
    res.model.close()


def test_argument_errors(elm):
    W, alpha, b = weights(6, 2, 8, seed=1)
    model = elm.Model.from_weights("elman_diag", 6, 1, W, alpha, b)
    X = torch.zeros((5, 6, 2), device="cuda")
    h0 = torch.zeros((5, 8), device="cuda")
    with pytest.raises(elm.ElmRnnError) as ei:
        elm.hidden(model, X, h0=h0)                       # no single initial state for this cell
    assert ei.value.code == -1
    lib = elm.load_library()
    H = torch.empty((5, 8), device="cuda")
    # more steps than the model has lag weights for
    assert lib.elm_rnn_hidden(model._h, X.data_ptr(), 12, 2, 5, 7, None, None, H.data_ptr(), None, None, 0, None) == -1
    model.close()
    with pytest.raises(elm.ElmRnnError) as ei:
        elm.Model.create("elman_diag", 4097, 1, 4, 1, seed=1)
    assert ei.value.code == -5
