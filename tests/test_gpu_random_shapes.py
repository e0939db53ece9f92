"""GPU parity on seeded random shapes: every cell, both contraction modes, sizes drawn across the
launch-variant boundaries (column blocks of 32, chunks of 128 columns, tiles of 32 / 64 / 128 / 256
rows, input groups of 8 / 16 columns), against the float64 oracle through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import cells as ocells

pytestmark = pytest.mark.gpu

GATES = {"elman": 1, "lstm": 4, "gru": 3}


def h_close(got, ref, tol=1e-5):
    ref = np.asarray(ref, dtype=np.float64)
    rms = max(np.sqrt(np.mean(ref ** 2)), 1e-30)
    err = np.abs(np.asarray(got, dtype=np.float64) - ref)
    return np.all(err <= tol * np.maximum(np.abs(ref), rms)), float(np.max(err / (tol * np.maximum(np.abs(ref), rms))))


def draw_case(rng):
    cell = rng.choice(["elman", "lstm", "gru", "elman_diag", "fc_multilag"])
    if cell == "elman_diag":
        Q, L, d = int(rng.integers(1, 70)), int(rng.integers(1, 130)), int(rng.integers(1, 9))
    elif cell == "fc_multilag":
        Q = int(rng.integers(1, 9))
        L = int(rng.integers(1, max(2, min(200, 1200 // max(Q - 1, 1)))))
        d = int(rng.integers(1, 9))
    else:
        Q = int(rng.integers(1, 5))
        L = int(rng.choice([rng.integers(1, 40), rng.integers(40, 140), rng.integers(140, 513)]))
        d = int(rng.choice([rng.integers(1, 16), rng.integers(16, 65)]))
    N = int(rng.choice([rng.integers(1, 300), rng.integers(300, 3000), rng.integers(17000, 40000)]))
    if N * L > 4_000_000:
        N = max(1, 4_000_000 // L)
    if cell == "elman_diag" and Q > 32:
        N = min(N, 5000)          # keeps the oracle's Q^2 / 2 lag terms per entry within seconds
    mode = "split16" if (cell in GATES and d <= 15 and rng.random() < 0.5) else "fp32"
    return cell, N, Q, d, L, mode


def make_weights(rng, cell, Q, d, L):
    if cell == "elman_diag":
        return (rng.uniform(-1, 1, (d, L)).astype(np.float32) / np.float32(np.sqrt(d)),
                (rng.uniform(-1, 1, (L, Q)) / max(Q - 1, 1)).astype(np.float32),
                rng.uniform(-0.5, 0.5, L).astype(np.float32))
    if cell == "fc_multilag":
        a = 0.7 / np.sqrt(L * max(Q - 1, 1))
        return (rng.uniform(-1, 1, (d, L)).astype(np.float32) / np.float32(np.sqrt(d)),
                rng.uniform(-a, a, (Q, L, L)).astype(np.float32),
                rng.uniform(-0.5, 0.5, L).astype(np.float32))
    k = GATES[cell]
    a = 1.0 / np.sqrt(L + d)
    return (rng.uniform(-a, a, (d, k * L)).astype(np.float32), rng.uniform(-a, a, (L, k * L)).astype(np.float32),
            rng.uniform(-0.5, 0.5, k * L).astype(np.float32))


@pytest.mark.parametrize("seed", range(40))
def test_random_shape(elm, seed):
    rng = np.random.default_rng(1000 + seed)
    cell, N, Q, d, L, mode = draw_case(rng)
    W, U, b = make_weights(rng, cell, Q, d, L)
    X = rng.uniform(-1, 1, (N, Q, d)).astype(np.float32)
    print(f"case: cell={cell} N={N} Q={Q} d={d} L={L} mode={mode}", flush=True)
    model = elm.Model.from_weights(cell, Q, 1, W, U, b)
    model.set_contraction(mode)
    H = elm.hidden(model, torch.from_numpy(X).cuda()).cpu().numpy()
    ok, worst = h_close(H, ocells.hidden_chunked(cell, X, W, U, b))
    assert ok, (cell, N, Q, d, L, mode, worst)
    model.close()


# the fully connected multi-lag cell where a window's history leaves the chip (a launch per step)
@pytest.mark.parametrize("seed", range(12))
def test_random_shape_multilag_launch_per_step(elm, seed):
    rng = np.random.default_rng(3000 + seed)
    Q = int(rng.choice([rng.integers(3, 12), rng.integers(12, 80)]))
    L = int(rng.integers(max(1, 1300 // (Q - 1) + 1), min(513, max(3, 6000 // (Q - 1))) + 1))
    d = int(rng.choice([rng.integers(1, 9), rng.integers(9, 65)]))
    N = int(rng.choice([rng.integers(1, 200), rng.integers(200, 1500)]))
    q_run = int(rng.choice([Q, rng.integers(1, Q + 1)]))
    assert (Q - 1) * L + d + 1 > 1272
    W, U, b = make_weights(rng, "fc_multilag", Q, d, L)
    X = rng.uniform(-1, 1, (N, Q, d)).astype(np.float32)
    print(f"case: N={N} Q={Q} d={d} L={L} Q_run={q_run}", flush=True)
    model = elm.Model.from_weights("fc_multilag", Q, 1, W, U, b)
    H = elm.hidden(model, torch.from_numpy(X).cuda(), Q_run=q_run).cpu().numpy()
    ok, worst = h_close(H, ocells.hidden_fc_multilag(X, W, U, b, steps=q_run))
    assert ok, (N, Q, d, L, q_run, worst)
    model.close()


@pytest.mark.parametrize("seed", range(8))
def test_random_long_window_of_the_papers_elman_cell(elm, seed):
    """Window lengths across the slot counts of the long-window kernel (129 .. 4096 steps)."""
    rng = np.random.default_rng(2000 + seed)
    Q = int(rng.choice([rng.integers(129, 600), rng.integers(600, 1100), rng.integers(1100, 2100),
                        rng.integers(2100, 3400), rng.integers(3400, 4097)]))
    N, L, d = int(rng.integers(1, 40)), int(rng.integers(1, 9)), int(rng.integers(1, 4))
    W, alpha, b = make_weights(rng, "elman_diag", Q, d, L)
    alpha[:, :30] *= np.float32(20.0)                       # recent lags dominate, all count
    alpha *= np.float32(0.9 / np.abs(alpha).sum(axis=1).max())
    X = rng.uniform(-1, 1, (N, Q, d)).astype(np.float32)
    q_run = int(rng.integers(1, Q + 1)) if seed % 2 else Q
    print(f"case: N={N} Q={Q} d={d} L={L} q_run={q_run}", flush=True)
    model = elm.Model.from_weights("elman_diag", Q, 1, W, alpha, b)
    H = elm.hidden(model, torch.from_numpy(X).cuda(), Q_run=q_run).cpu().numpy()
    ok, worst = h_close(H, ocells.hidden_elman_diag(X, W, alpha, b, steps=q_run))
    assert ok, (N, Q, d, L, q_run, worst)
    model.close()


@pytest.mark.parametrize("seed", range(12))
def test_random_streamed_fit(elm, seed):
    """The streamed fit on random shapes, chunk sizes and forms (in-kernel hand-off where it exists)."""
    from oracle import lstsq
    rng = np.random.default_rng(3000 + seed)
    cell = str(rng.choice(["elman", "lstm", "gru"]))
    wide = {"elman": 257, "lstm": 129, "gru": 257}[cell]
    L = int(rng.choice([rng.integers(4, 100), rng.integers(wide, 513)]))
    d, m, Q = int(rng.integers(3, 9)), int(rng.integers(1, 4)), int(rng.integers(2, 6))
    N = int(rng.integers(6 * L, 6 * L + 3000))
    hand_off = L >= 65 and rng.random() < 0.6          # the in-kernel hand-off exists above 64 units
    chunk = -1 if hand_off else int(rng.choice([0, rng.integers(128, 2000)]))
    mode = "split16" if (not hand_off and rng.random() < 0.4) else "fp32"
    X = rng.uniform(-1, 1, (N, Q, d)).astype(np.float32)
    T = (np.tanh(X[:, -1, :m] * 2.0) + 0.1 * rng.standard_normal((N, m))).astype(np.float32)
    kw = dict(w_scale=0.4, spectral_radius=0.9 if cell == "elman" else 0.0, forget_bias=1.0 if cell == "lstm" else 0.0)
    print(f"case: cell={cell} N={N} Q={Q} d={d} L={L} m={m} chunk={chunk} mode={mode}", flush=True)
    Xd, Td = torch.from_numpy(X).cuda(), torch.from_numpy(T).cuda()
    res = elm.fit_streamed(cell, Xd, Td, L, 77 + seed, chunk_rows=chunk, contraction=mode, **kw)
    H = elm.hidden(res.model, Xd).cpu().numpy()
    b64 = res.beta64.cpu().numpy()
    _, ref_rss, _ = lstsq.solve(H, T)
    ref_rmse = lstsq.rmse_from_rss(ref_rss, N, m)
    rmse = float(np.sqrt(np.mean((H.astype(np.float64) @ b64 - T) ** 2)))
    assert abs(rmse - ref_rmse) <= 1e-4 * ref_rmse, (rmse, ref_rmse)
    ne = lstsq.normal_equation_residual(H, T, b64)
    assert ne <= 1e-5, (ne, res.stats.refine_iters, res.stats.r_diag_min, res.stats.r_diag_max)
    res.model.close()
