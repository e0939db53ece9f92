"""GPU edge cases through the C ABI: degenerate and maximum sizes, every kernel variant the
launchers can pick, error codes, determinism, caller streams, predict / set_beta."""
import numpy as np
import pytest
import torch

from oracle import cells as ocells
from oracle import lstsq

pytestmark = pytest.mark.gpu

GATES = {"elman": 1, "lstm": 4, "gru": 3}


def h_close(got, ref, tol=1e-5):
    ref = np.asarray(ref, dtype=np.float64)
    rms = max(np.sqrt(np.mean(ref ** 2)), 1e-30)
    return np.all(np.abs(np.asarray(got, dtype=np.float64) - ref) <= tol * np.maximum(np.abs(ref), rms))


def weights(cell, d, L, seed):
    k = GATES[cell]
    rng = np.random.default_rng(seed)
    a = 1.0 / np.sqrt(L + d)
    return (rng.uniform(-a, a, (d, k * L)).astype(np.float32),
            rng.uniform(-a, a, (L, k * L)).astype(np.float32),
            rng.uniform(-0.5, 0.5, k * L).astype(np.float32))


@pytest.mark.parametrize("cell,N,Q,d,L", [
    ("gru", 70, 2, 3, 512),      # two LDS operands do not fit at 64 rows: 32-row tiles
    ("gru", 90, 2, 2, 300),      # largest GRU that still runs 64-row tiles
    ("gru", 40, 3, 2, 330),      # first size on the 32-row path
    ("lstm", 100, 2, 64, 448),   # widest input, staged variant boundary
    ("lstm", 65, 3, 1, 289),     # three column chunks, ragged last block
    ("elman", 129, 2, 64, 512),  # largest Elman
    ("elman", 5, 1, 1, 2), ("lstm", 1, 1, 1, 1), ("gru", 2, 1, 1, 3),
])
def test_hidden_every_launch_variant(elm, cell, N, Q, d, L):
    W, U, b = weights(cell, d, L, seed=L + N)
    X = np.random.default_rng(N).uniform(-1, 1, (N, Q, d)).astype(np.float32)
    model = elm.Model.from_weights(cell, Q, 1, W, U, b)
    H = elm.hidden(model, torch.from_numpy(X).cuda()).cpu().numpy()
    assert h_close(H, ocells.hidden(cell, X, W, U, b))
    model.close()


def test_hidden_and_model_argument_errors(elm):
    W, U, b = weights("lstm", 2, 8, seed=1)
    model = elm.Model.from_weights("lstm", 4, 1, W, U, b)
    X = torch.zeros((5, 4, 2), device="cuda")
    lib = elm.load_library()
    # Q_run < 1 and N < 1 are invalid arguments (no launch happens)
    H = torch.empty((5, 8), device="cuda")
    assert lib.elm_rnn_hidden(model._h, X.data_ptr(), 8, 2, 5, 0, None, None, H.data_ptr(), None, None, 0, None) == -1
    assert lib.elm_rnn_hidden(model._h, X.data_ptr(), 8, 2, 0, 4, None, None, H.data_ptr(), None, None, 0, None) == -1
    assert lib.elm_rnn_hidden(model._h, None, 8, 2, 5, 4, None, None, H.data_ptr(), None, None, 0, None) == -1
    assert lib.elm_rnn_hidden(None, X.data_ptr(), 8, 2, 5, 4, None, None, H.data_ptr(), None, None, 0, None) == -1
    model.close()
    with pytest.raises(elm.ElmRnnError) as ei:
        elm.Model.create("lstm", 4, 2, 513, 1, seed=1, w_scale=0.1)
    assert ei.value.code == -5
    with pytest.raises(elm.ElmRnnError) as ei:
        elm.Model.create("lstm", 4, 2, 8, 1, seed=1, w_scale=0.1, spectral_radius=0.9)   # Elman only
    assert ei.value.code == -1
    with pytest.raises(elm.ElmRnnError) as ei:
        elm.Model.create("elman", 0, 2, 8, 1, seed=1)
    assert ei.value.code == -1
    # binding-side checks: host tensors and wrong dtypes never reach the library
    with pytest.raises(TypeError):
        elm.solve(torch.zeros((8, 2)), torch.zeros((8, 1)))
    with pytest.raises(TypeError):
        elm.solve(torch.zeros((8, 2), device="cuda", dtype=torch.float64), torch.zeros((8, 1), device="cuda"))


@pytest.mark.parametrize("N,L,m", [(1, 1, 1), (33, 33, 2), (512, 512, 1), (700, 40, 16), (3000, 500, 8),
                                   (127, 64, 5)])
def test_solve_degenerate_and_wide_targets(elm, N, L, m):
    rng = np.random.default_rng(N + L + m)
    H = rng.standard_normal((N, L)).astype(np.float32)
    if N == L:
        H += (3.0 * np.sqrt(L) * np.eye(L)).astype(np.float32)     # keep the square system well conditioned
    T = rng.standard_normal((N, m)).astype(np.float32)
    b32, b64, st = elm.solve(torch.from_numpy(H).cuda(), torch.from_numpy(T).cuda())
    ref, rss, _ = lstsq.solve(H, T, check_rank=False)
    np.testing.assert_allclose(b64.cpu().numpy(), ref, rtol=0, atol=2e-5 * max(np.abs(ref).max(), 1e-30))
    ref_rmse = lstsq.rmse_from_rss(rss, N, m)
    if N > L:
        assert abs(st.rmse - ref_rmse) <= 1e-4 * ref_rmse
        assert lstsq.normal_equation_residual(H, T, b64.cpu().numpy()) <= 1e-5
    else:
        assert st.rmse <= 1e-5 * np.abs(T).max()                   # square system: exact fit


def test_fit_is_deterministic_and_h_may_live_in_the_workspace(elm):
    rng = np.random.default_rng(4)
    X = torch.from_numpy(rng.uniform(-1, 1, (5000, 6, 3)).astype(np.float32)).cuda()
    T = torch.from_numpy(rng.standard_normal((5000, 2)).astype(np.float32)).cuda()
    a = elm.fit("gru", X, T, 72, seed=9, w_scale=0.4, zero_bias=True)
    b = elm.fit("gru", X, T, 72, seed=9, w_scale=0.4, zero_bias=True, keep_H=False)
    assert b.H is None
    assert torch.equal(a.beta64, b.beta64) and torch.equal(a.beta, b.beta)
    assert a.stats.rmse == b.stats.rmse
    c = elm.fit("gru", X, T, 72, seed=10, w_scale=0.4, zero_bias=True)
    assert not torch.equal(a.beta64, c.beta64)
    for r in (a, b, c):
        r.model.close()


def test_caller_stream_predict_and_set_beta(elm):
    rng = np.random.default_rng(5)
    Xh = rng.uniform(-1, 1, (3000, 5, 2)).astype(np.float32)
    Th = rng.standard_normal((3000, 3)).astype(np.float32)
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        X, T = torch.from_numpy(Xh).cuda(), torch.from_numpy(Th).cuda()
        res = elm.fit("lstm", X, T, 40, seed=3, w_scale=0.5, forget_bias=1.0, stream=stream)
        Y = elm.predict(res.model, X, stream=stream)
    stream.synchronize()
    W, U, b, beta = res.model.weights()
    Href = ocells.hidden("lstm", Xh, W, U, b)
    assert h_close(res.H.cpu().numpy(), Href)
    np.testing.assert_allclose(Y.cpu().numpy(), Href @ beta, atol=1e-4)
    # a loaded beta replaces the fitted one
    beta2 = np.arange(40 * 3, dtype=np.float64).reshape(40, 3) / 100.0
    res.model.set_beta(beta2)
    Y2 = elm.predict(res.model, X).cpu().numpy()
    np.testing.assert_allclose(Y2, Href @ beta2, atol=2e-4)
    res.model.close()


def test_ceilings_probe_reports_plausible_rates(elm):
    """The measured-ceilings diagnostic: rates below the published peaks, above half of them."""
    c = elm.probe_ceilings()
    assert 80.0 < c["mfma_f32_tflops"] <= 157.3 * 1.02
    assert 1000.0 < c["mfma_f16_tflops"] <= 2500.0 * 1.02
    assert 2000.0 < c["hbm_copy_gbs"] <= 8000.0 * 1.02
    # float32 matrix instructions keep the vector ALU of their SIMD busy (no overlap with another wave's
    # vector work), fp16 ones do not: the reason stage 2's chain and trailing update cannot be overlapped
    # by wave specialisation, and stage 1's gate math cannot hide behind its float32 contraction
    assert c["valu_overlap_with_mfma_f32"] < 0.25
    assert c["valu_overlap_with_mfma_f16"] > 0.6
    lib = elm.load_library()
    import ctypes as C
    x = C.c_double()
    assert lib.elm_rnn_probe_ceilings(C.byref(x), C.byref(x), C.byref(x), None, None, None, 0, None) == -2
