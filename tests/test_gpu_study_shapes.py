"""GPU parity at the full sizes of the study workloads, in the launch configuration bench.py times:
the paper's own two cells at a million windows (the fully connected one also at Q = 50, where every step
is a launch over a device-resident history) and its Elman cell on the shape of its longest dataset
(4,500 windows of 3,197 steps, 100 units).  The oracle computes sampled rows one by one."""
import numpy as np
import pytest
import torch

import synthdata
from oracle import cells as ocells

pytestmark = pytest.mark.gpu


def h_close(got, ref, tol=1e-5):
    ref = np.asarray(ref, dtype=np.float64)
    rms = max(np.sqrt(np.mean(ref ** 2)), 1e-30)
    return np.all(np.abs(np.asarray(got, dtype=np.float64) - ref) <= tol * np.maximum(np.abs(ref), rms))


def sliding(series, N, Q, d):
    dev = torch.from_numpy(series).cuda()
    return dev, torch.as_strided(dev, (N, Q, d), (d, d, 1))          # zero-copy windows, as bench.py --sweep


@pytest.mark.parametrize("name", ["paper_elman", "paper_fc", "paper_fc_q50"])
def test_paper_cells_at_a_million_windows(elm, name):
    cfg = synthdata.get_config(name)
    series = synthdata.make_series(cfg.N + cfg.Q, cfg.d, cfg.seed, cfg.ar_sigma).astype(np.float32)
    dev, X = sliding(series, cfg.N, cfg.Q, cfg.d)
    model = elm.Model.create(cfg.cell, cfg.Q, cfg.d, cfg.L, cfg.m, seed=cfg.seed, w_scale=cfg.w_scale)
    H = elm.hidden(model, X)
    assert torch.isfinite(H).all()
    # (for paper_fc_q50 the rows come in 11 passes of 63,744: the samples include both sides of the first edges)
    rows = np.unique(np.concatenate([np.arange(70), np.random.default_rng(1).choice(cfg.N, 400), [cfg.N - 1],
                                     np.arange(63_744 - 40, 63_744 + 40), np.arange(2 * 63_744 - 40, 2 * 63_744 + 40)]))
    Xs = np.lib.stride_tricks.sliding_window_view(series, (cfg.Q, cfg.d))[rows, 0]
    W, U, b, _ = model.weights()
    ref = ocells.hidden(cfg.cell, Xs, W, U, b)
    assert h_close(H[torch.from_numpy(rows).cuda()].cpu().numpy(), ref)
    model.close()


def test_paper_elman_on_its_longest_window_shape(elm):
    N, Q, d, L = 4500, 3197, 1, 100
    rng = np.random.default_rng(31)
    W = rng.uniform(-1, 1, (d, L)).astype(np.float32)
    alpha = (rng.uniform(-1, 1, (L, Q)) / (Q - 1)).astype(np.float32)       # sum_k |alpha_jk| < 1
    alpha[:, :40] *= 30.0                                                    # recent lags dominate, all count
    alpha *= np.float32(0.9 / np.abs(alpha).sum(axis=1).max())
    b = rng.uniform(-0.5, 0.5, L).astype(np.float32)
    series = synthdata.make_series(N + Q, d, 77, 0.05).astype(np.float32)
    dev, X = sliding(series, N, Q, d)
    model = elm.Model.from_weights("elman_diag", Q, 1, W, alpha, b)
    H = elm.hidden(model, X)
    rows = np.array([0, 1, 7, 2250, 4493, 4499])
    Xs = np.lib.stride_tricks.sliding_window_view(series, (Q, d))[rows, 0]
    ref = ocells.hidden_elman_diag(Xs, W, alpha, b)
    assert h_close(H[torch.from_numpy(rows).cuda()].cpu().numpy(), ref)
    assert torch.isfinite(H).all()
    model.close()


def test_fully_connected_cell_on_the_longest_window_shape(elm):
    """4,500 windows of 3,197 steps, 50 units: a window's history is 716 KB, a pass holds 2,304 rows and
    its launches split the contraction over slices of the operand; 5.1 million lag products per window,
    so the oracle takes three rows."""
    N, Q, d, L = 4500, 3197, 1, 50
    rng = np.random.default_rng(41)
    W = rng.uniform(-1, 1, (d, L)).astype(np.float32)
    a = 0.7 / np.sqrt(L * (Q - 1))
    A = rng.uniform(-a, a, (Q, L, L)).astype(np.float32)
    A[:40] *= 8.0                                            # recent lags dominate, all count
    b = rng.uniform(-0.5, 0.5, L).astype(np.float32)
    series = synthdata.make_series(N + Q, d, 78, 0.05).astype(np.float32)
    dev, X = sliding(series, N, Q, d)
    model = elm.Model.from_weights("fc_multilag", Q, 1, W, A, b)
    H = elm.hidden(model, X)
    rows = np.array([0, 2303, 2304, 4499])                   # both sides of the pass edge
    Xs = np.lib.stride_tricks.sliding_window_view(series, (Q, d))[rows, 0]
    ref = ocells.hidden_fc_multilag(Xs, W, A, b)
    assert h_close(H[torch.from_numpy(rows).cuda()].cpu().numpy(), ref)
    assert torch.isfinite(H).all()
    model.close()
