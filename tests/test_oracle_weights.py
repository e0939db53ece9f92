"""Pins for the oracle's seeded weight generator (CPU only)."""
import numpy as np
import pytest

from oracle import weights


def test_splitmix64_known_answers():
    # published test vectors of the SplitMix64 generator (seed 1234567, and seed 0)
    got = weights.splitmix64(1234567, 5)
    want = np.array([6457827717110365317, 3203168211198807973, 9817491932198370423,
                     4593380528125082431, 16408922859458223821], dtype=np.uint64)
    np.testing.assert_array_equal(got, want)
    assert int(weights.splitmix64(0, 1)[0]) == 0xE220A8397B1DCDAF


def test_splitmix64_matches_scalar_python_integers():
    mask = (1 << 64) - 1
    state = 987654321
    ref = []
    for _ in range(20):
        state = (state + 0x9E3779B97F4A7C15) & mask
        z = state
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & mask
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & mask
        ref.append(z ^ (z >> 31))
    np.testing.assert_array_equal(weights.splitmix64(987654321, 20), np.array(ref, dtype=np.uint64))
    u = weights.uniform01(987654321, 20)
    np.testing.assert_array_equal(u, np.array([(r >> 11) / 2.0 ** 53 for r in ref]))


@pytest.mark.parametrize("cell,k", [("elman", 1), ("lstm", 4), ("gru", 3)])
def test_shapes_range_moments_and_draw_order(cell, k):
    d, L, a = 3, 64, 0.5
    W, U, b = weights.draw(cell, d, L, seed=7, w_scale=a)
    assert W.shape == (d, k * L) and U.shape == (L, k * L) and b.shape == (k * L,)
    assert W.dtype == U.dtype == b.dtype == np.float32
    allv = np.concatenate([W.ravel(), U.ravel(), b.ravel()])
    assert allv.min() >= -a and allv.max() <= a
    assert abs(U.mean()) < 0.02 and abs(U.var() - a * a / 3.0) < 0.01
    # draw order W, U, b from one stream
    v = ((2.0 * weights.uniform01(7, allv.size) - 1.0) * a).astype(np.float32)
    np.testing.assert_array_equal(allv, v)


def test_determinism_and_seed_sensitivity():
    a = weights.draw("lstm", 2, 8, seed=11, w_scale=0.3, forget_bias=1.0)
    b = weights.draw("lstm", 2, 8, seed=11, w_scale=0.3, forget_bias=1.0)
    c = weights.draw("lstm", 2, 8, seed=12, w_scale=0.3, forget_bias=1.0)
    for x, y in zip(a, b):
        np.testing.assert_array_equal(x, y)
    assert np.abs(a[1] - c[1]).max() > 0.01


def test_elman_spectral_radius_after_rounding():
    for L in (32, 100):
        _, U, _ = weights.draw("elman", 1, L, seed=13252, w_scale=1.0, spectral_radius_target=0.9)
        rho = np.max(np.abs(np.linalg.eigvals(U.astype(np.float64))))
        assert abs(rho - 0.9) < 1e-6


def test_spectral_radius_of_known_matrices():
    assert abs(weights.spectral_radius(np.diag([0.5, -2.0, 1.0])) - 2.0) < 1e-14
    rot = 3.0 * np.array([[np.cos(1.0), -np.sin(1.0)], [np.sin(1.0), np.cos(1.0)]])
    assert abs(weights.spectral_radius(rot) - 3.0) < 1e-14          # complex pair
    assert weights.spectral_radius(np.array([[0.0, 1.0], [0.0, 0.0]])) < 1e-12   # nilpotent


def test_forget_bias_and_zero_bias():
    L = 256
    _, _, b0 = weights.draw("lstm", 2, L, seed=5, w_scale=0.5)
    _, _, b1 = weights.draw("lstm", 2, L, seed=5, w_scale=0.5, forget_bias=1.0)
    np.testing.assert_array_equal(b1[:L], b0[:L])
    np.testing.assert_array_equal(b1[2 * L:], b0[2 * L:])
    np.testing.assert_allclose(b1[L:2 * L], b0[L:2 * L].astype(np.float64) + 1.0, atol=1e-7)
    assert abs(b1[L:2 * L].mean() - 1.0) < 0.1
    Wz, Uz, bz = weights.draw("gru", 2, L, seed=5, w_scale=0.5, zero_bias=True)
    Wn, Un, _ = weights.draw("gru", 2, L, seed=5, w_scale=0.5)
    assert np.all(bz == 0.0)
    np.testing.assert_array_equal(Wz, Wn)
    np.testing.assert_array_equal(Uz, Un)


def _scalar_stream(seed, a):
    """The generator written out with Python integers, one value per call."""
    mask = (1 << 64) - 1
    state = seed & mask
    while True:
        state = (state + 0x9E3779B97F4A7C15) & mask
        z = state
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & mask
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & mask
        z ^= z >> 31
        yield (2.0 * ((z >> 11) / 2.0 ** 53) - 1.0) * a


@pytest.mark.parametrize("cell", ["elman_diag", "fc_multilag"])
def test_multilag_cells_shape_and_stream_order_against_a_scalar_stream(cell):
    """alpha [L, Q] (lag k in column k-1) and A [Q, L, L] (lag k in block k-1, A[k-1][m][j]) take U's place
    in the stream: W row-major first, then the recurrent array row-major, then b; a wrong axis order or a
    swapped draw order moves values and fails the element-wise comparison."""
    d, L, Q, a, seed = 2, 3, 4, 0.25, 99
    W, U, b = weights.draw(cell, d, L, seed=seed, w_scale=a, Q=Q)
    g = _scalar_stream(seed, a)
    Wr = np.empty((d, L)); br = np.empty(L)
    for s in range(d):
        for j in range(L):
            Wr[s, j] = next(g)
    if cell == "elman_diag":
        Ur = np.empty((L, Q))
        for j in range(L):
            for k in range(Q):
                Ur[j, k] = next(g)
    else:
        Ur = np.empty((Q, L, L))
        for k in range(Q):
            for mm in range(L):
                for j in range(L):
                    Ur[k, mm, j] = next(g)
    for j in range(L):
        br[j] = next(g)
    assert W.shape == Wr.shape and U.shape == Ur.shape and b.shape == br.shape
    np.testing.assert_array_equal(W, Wr.astype(np.float32))
    np.testing.assert_array_equal(U, Ur.astype(np.float32))
    np.testing.assert_array_equal(b, br.astype(np.float32))
    # the non-square shapes make a transposed draw visible
    assert not np.array_equal(U.reshape(-1), np.swapaxes(U, -1, -2).reshape(-1))
    with pytest.raises(ValueError):
        weights.draw(cell, d, L, seed=seed, w_scale=a)          # the multi-lag cells need Q
