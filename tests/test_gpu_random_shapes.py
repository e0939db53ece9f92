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
