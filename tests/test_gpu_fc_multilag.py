"""GPU parity of the paper's fully connected multi-lag cell (section "Fully Connected RNN": every
neuron is fed by all neurons' outputs of all earlier steps) against the float64 oracle, through the
C ABI."""
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
    a = 0.7 / np.sqrt(L * max(Q - 1, 1))          # keeps the multi-lag map contractive
    return (rng.uniform(-1, 1, (d, L)).astype(np.float32) / np.float32(np.sqrt(d)),
            rng.uniform(-a, a, (Q, L, L)).astype(np.float32),
            rng.uniform(-0.5, 0.5, L).astype(np.float32))


# 64- and 32-row tiles (the operand row grows with (Q-1) L), every column-chunk count, narrow layers
# whose waves split the rows, ragged tails, a launch with enough tiles to keep 64-row blocks per wave
@pytest.mark.parametrize("N,Q,d,L", [
    (1, 1, 1, 1), (70, 2, 2, 5), (200, 5, 3, 33), (300, 10, 1, 50), (150, 10, 2, 100), (100, 4, 1, 300),
    (64, 3, 64, 64), (90, 2, 1, 512), (5000, 10, 1, 20), (70001, 6, 1, 30), (33, 25, 2, 48),
])
def test_hidden_matches_oracle(elm, N, Q, d, L):
    W, A, b = weights(Q, d, L, seed=N + Q + L)
    X = np.random.default_rng(N * 3 + Q).uniform(-1, 1, (N, Q, d)).astype(np.float32)
    model = elm.Model.from_weights("fc_multilag", Q, 1, W, A, b)
    H = elm.hidden(model, torch.from_numpy(X).cuda()).cpu().numpy()
    assert h_close(H, ocells.hidden_fc_multilag(X, W, A, b))
    model.close()


# Windows whose history does not fit LDS take one launch per step over a device-resident history:
# one, two and four column blocks per work-group, a short last group of column blocks (L = 300),
# the widest input, slot widths that are not multiples of 8, ragged row tails, Q barely past the limit
@pytest.mark.parametrize("N,Q,d,L", [
    (100, 200, 1, 8), (257, 60, 2, 33), (90, 14, 1, 100), (70, 6, 1, 300), (40, 4, 64, 512),
    (300, 50, 4, 100), (129, 50, 1, 50), (65, 300, 3, 5), (1, 130, 1, 10),
])
def test_hidden_per_step_path_matches_oracle(elm, N, Q, d, L):
    assert (Q - 1) * L + d + 1 > 1272
    W, A, b = weights(Q, d, L, seed=N + Q + L)
    X = np.random.default_rng(N * 3 + Q).uniform(-1, 1, (N, Q, d)).astype(np.float32)
    model = elm.Model.from_weights("fc_multilag", Q, 1, W, A, b)
    Xd = torch.from_numpy(X).cuda()
    H = elm.hidden(model, Xd).cpu().numpy()
    assert h_close(H, ocells.hidden_fc_multilag(X, W, A, b))
    for q in {1, 2, Q // 2, Q - 1}:
        got = elm.hidden(model, Xd, Q_run=q).cpu().numpy()
        assert h_close(got, ocells.hidden_fc_multilag(X, W, A, b, steps=q)), q
    model.close()


def pass_rows(N, Q, L):
    """Rows per pass of the launch-per-step form: the history buffer stays below 2 GiB and holds at most
    65,536 rows; the passes are equal multiples of 256 rows."""
    row_bytes = max(Q - 1, 1) * (-(-L // 8) * 8) * 4
    cap = min(65_536, max(256, (2 ** 31 - 1) // row_bytes // 256 * 256))
    passes = -(-N // cap)
    return -(-(-(-N // passes)) // 256) * 256


# Launches large enough for 64-row blocks per wave, and more rows than the history buffer holds (the rows
# are then taken in equal passes over the steps); rows are independent, so the oracle is evaluated on
# samples: the first and last rows, those around the pass boundary and random ones.  Layers of 65 to 96
# units with at least 256 tiles of 128 rows take the kernel whose waves split the rows (5 or 6 column
# units of 16) and that runs all steps of a pass in one launch; wider layers take the 32-column blocks.
@pytest.mark.parametrize("N,Q,d,L,ns", [(131_000, 21, 1, 64, 200), (40_000, 14, 2, 100, 200), (50_001, 15, 1, 97, 200),
                                        (33_000, 20, 1, 70, 200), (33_011, 16, 3, 90, 200), (34_000, 12, 1, 120, 200),
                                        (140_000, 19, 2, 72, 150),
                                        (66_000, 160, 1, 8, 150), (60_000, 100, 1, 100, 40)])
def test_hidden_per_step_path_many_rows(elm, N, Q, d, L, ns):
    W, A, b = weights(Q, d, L, seed=Q + L)
    X = np.random.default_rng(Q).uniform(-1, 1, (N, Q, d)).astype(np.float32)
    model = elm.Model.from_weights("fc_multilag", Q, 1, W, A, b)
    Xd = torch.from_numpy(X).cuda()
    H = elm.hidden(model, Xd).cpu().numpy()
    Hhalf = elm.hidden(model, Xd, Q_run=Q // 2).cpu().numpy()
    model.close()
    edge = pass_rows(N, Q, L)
    if (N, Q, L) in ((131_000, 21, 64), (66_000, 160, 8), (60_000, 100, 100), (140_000, 19, 72)):
        assert edge < N                              # these cases take two or three passes
    idx = np.unique(np.concatenate([np.arange(0, ns), np.arange(N - ns, N),
                                    np.clip(np.arange(edge - ns, edge + ns), 0, N - 1),
                                    np.random.default_rng(1).integers(0, N, ns)]))
    assert h_close(H[idx], ocells.hidden_fc_multilag(X[idx], W, A, b))
    assert h_close(Hhalf[idx], ocells.hidden_fc_multilag(X[idx], W, A, b, steps=Q // 2))
    assert np.all(np.isfinite(H)) and np.abs(H).max() <= 1.0


def test_fit_per_step_path_matches_oracle_fit(elm):
    N, Q, d, L, m, seed = 20000, 50, 2, 30, 2, 12
    rng = np.random.default_rng(seed)
    X = rng.uniform(-1, 1, (N, Q, d)).astype(np.float32)
    T = (np.sin(X[:, -8:].sum(axis=(1, 2)))[:, None] * np.arange(1, m + 1) + 0.05 * rng.standard_normal((N, m))
         ).astype(np.float32)
    w_scale = 0.08
    Xd, Td = torch.from_numpy(X).cuda(), torch.from_numpy(T).cuda()
    res = elm.fit("fc_multilag", Xd, Td, L, seed=seed, w_scale=w_scale)
    ref = ofit.fit("fc_multilag", X, T, L, seed, w_scale=w_scale)
    W, U, b, beta = res.model.weights()
    assert np.array_equal(W, ref["W"]) and np.array_equal(U, ref["U"]) and np.array_equal(b, ref["b"])
    assert h_close(res.H.cpu().numpy(), ref["H"])
    assert abs(res.stats.rmse - ref["rmse"]) <= 1e-4 * ref["rmse"]
    assert lstsq.normal_equation_residual(res.H.cpu().numpy(), T, beta) <= 1e-5
    Y = elm.predict(res.model, Xd[:700]).cpu().numpy()
    np.testing.assert_allclose(Y, ref["H"][:700] @ beta, rtol=0,
                               atol=2e-5 * np.abs(beta).sum(axis=0).max() + 1e-5)
    res.model.close()
    # the streamed fit recomputes H chunk by chunk through the same per-step launches
    st = elm.fit_streamed("fc_multilag", Xd, Td, L, seed=seed, w_scale=w_scale, chunk_rows=4096)
    assert abs(st.stats.rmse - ref["rmse"]) <= 1e-4 * ref["rmse"]
    assert lstsq.normal_equation_residual(ref["H"], T, st.model.weights()[3]) <= 1e-5
    st.model.close()


def test_fewer_steps_lag_one_only_and_diagonal_lags(elm):
    Q, d, L, N = 9, 2, 40, 700
    W, A, b = weights(Q, d, L, seed=5)
    X = np.random.default_rng(6).uniform(-1, 1, (N, Q, d)).astype(np.float32)
    Xd = torch.from_numpy(X).cuda()
    model = elm.Model.from_weights("fc_multilag", Q, 1, W, A, b)
    for q in (1, 2, 5, 8):
        got = elm.hidden(model, Xd, Q_run=q).cpu().numpy()
        assert h_close(got, ocells.hidden_fc_multilag(X, W, A, b, steps=q)), q
    model.close()
    # only lag 1: the dense Elman kernel run on the same matrix gives the same H
    A1 = np.zeros_like(A)
    A1[0] = A[0] * 3
    m1 = elm.Model.from_weights("fc_multilag", Q, 1, W, A1, b)
    m2 = elm.Model.from_weights("elman", Q, 1, W, A1[0], b)
    H1, H2 = elm.hidden(m1, Xd).cpu().numpy(), elm.hidden(m2, Xd).cpu().numpy()
    ref = ocells.hidden_elman(X, W, A1[0], b)
    assert h_close(H1, ref) and h_close(H2, ref)
    m1.close(), m2.close()
    # diagonal lag matrices: the paper's own Elman cell
    alpha = np.random.default_rng(7).uniform(-0.1, 0.1, (L, Q)).astype(np.float32)
    Ad = np.stack([np.diag(alpha[:, k]) for k in range(Q)]).astype(np.float32)
    m3 = elm.Model.from_weights("fc_multilag", Q, 1, W, Ad, b)
    m4 = elm.Model.from_weights("elman_diag", Q, 1, W, alpha, b)
    ref = ocells.hidden_elman_diag(X, W, alpha, b)
    assert h_close(elm.hidden(m3, Xd).cpu().numpy(), ref) and h_close(elm.hidden(m4, Xd).cpu().numpy(), ref)
    m3.close(), m4.close()


def test_fit_matches_oracle_fit(elm):
    N, Q, d, L, m, seed = 20000, 10, 2, 40, 2, 11
    rng = np.random.default_rng(seed)
    X = rng.uniform(-1, 1, (N, Q, d)).astype(np.float32)
    T = (np.sin(X.sum(axis=(1, 2)))[:, None] * np.arange(1, m + 1) + 0.05 * rng.standard_normal((N, m))
         ).astype(np.float32)
    w_scale = 0.2          # cond(H) ~ 50, rounding amplified ~6x over the window (oracle probe)
    res = elm.fit("fc_multilag", torch.from_numpy(X).cuda(), torch.from_numpy(T).cuda(), L, seed=seed,
                  w_scale=w_scale)
    ref = ofit.fit("fc_multilag", X, T, L, seed, w_scale=w_scale)
    W, U, b, beta = res.model.weights()
    assert U.shape == (Q, L, L)
    assert np.array_equal(W, ref["W"]) and np.array_equal(U, ref["U"]) and np.array_equal(b, ref["b"])
    assert h_close(res.H.cpu().numpy(), ref["H"])
    assert abs(res.stats.rmse - ref["rmse"]) <= 1e-4 * ref["rmse"]
    assert lstsq.normal_equation_residual(res.H.cpu().numpy(), T, beta) <= 1e-5
    Y = elm.predict(res.model, torch.from_numpy(X[:500]).cuda()).cpu().numpy()
    np.testing.assert_allclose(Y, ref["H"][:500] @ beta, rtol=0,
                               atol=2e-5 * np.abs(beta).sum(axis=0).max() + 1e-5)
    res.model.close()


def test_argument_errors(elm):
    W, A, b = weights(4, 2, 8, seed=1)
    model = elm.Model.from_weights("fc_multilag", 4, 1, W, A, b)
    X = torch.zeros((5, 4, 2), device="cuda")
    with pytest.raises(elm.ElmRnnError) as ei:
        elm.hidden(model, X, h0=torch.zeros((5, 8), device="cuda"))
    assert ei.value.code == -1
    with pytest.raises(elm.ElmRnnError) as ei:
        model.set_contraction("split16")
    assert ei.value.code == -5
    model.close()
    with pytest.raises(elm.ElmRnnError) as ei:
        elm.Model.create("fc_multilag", 4098, 1, 512, 1, seed=1)      # a history row above 8 MiB
    assert ei.value.code == -5
