"""GPU tests of what the header promises beyond the arithmetic: the refinement policy of the fit, work on the
caller's stream only, a model that owns no per-call scratch (concurrent stage-1 calls on one model), and
the binding's argument checks."""
import ctypes as C

import numpy as np
import pytest
import torch

import synthdata
from oracle import cells as ocells
from oracle import lstsq

pytestmark = pytest.mark.gpu


def h_close(got, ref, tol=1e-5):
    ref = np.asarray(ref, dtype=np.float64)
    rms = max(np.sqrt(np.mean(ref ** 2)), 1e-30)
    return np.all(np.abs(np.asarray(got, dtype=np.float64) - ref) <= tol * np.maximum(np.abs(ref), rms))


def cfg_kwargs(cfg):
    return dict(w_scale=cfg.w_scale, spectral_radius=cfg.spectral_radius,
                forget_bias=cfg.forget_bias, zero_bias=cfg.zero_bias)


def test_fit_refine_argument_and_automatic_policy(elm):
    """refine = 0..4 steps, -1 = two steps exactly when max|R_jj| > 30 min|R_jj|.  On the ill-conditioned
    Elman configuration the unrefined float32 solution misses the residual bar and the automatic mode
    meets it; on a well-conditioned gated layer the automatic mode takes no step and still meets it."""
    cfg = synthdata.get_config("cfg2")
    _, X, T = synthdata.make_problem(cfg, N=20_000)
    Xd, Td = torch.from_numpy(X).cuda(), torch.from_numpy(T).cuda()
    res = {r: elm.fit(cfg.cell, Xd, Td, cfg.L, cfg.seed, refine=r, **cfg_kwargs(cfg)) for r in (-1, 0, 1, 2)}
    H = res[-1].H.cpu().numpy()
    for r in (0, 1, 2):
        assert res[r].stats.refine_iters == r
        assert torch.equal(res[r].H, res[-1].H)
    st = res[-1].stats
    assert st.r_diag_max > 30 * st.r_diag_min and st.refine_iters == 2
    assert torch.equal(res[-1].beta64, res[2].beta64)
    ne = {r: lstsq.normal_equation_residual(H, T, res[r].beta64.cpu().numpy()) for r in res}
    assert ne[-1] <= 1e-5 and ne[2] <= 1e-5
    assert ne[0] > ne[2]                          # refinement is what brings the residual down here
    for r in res.values():
        assert abs(r.stats.ne_resid - lstsq.normal_equation_residual(H, T, r.beta64.cpu().numpy())) <= \
            1e-3 * r.stats.ne_resid + 1e-12
        r.model.close()
    with pytest.raises(elm.ElmRnnError) as ei:
        elm.fit(cfg.cell, Xd, Td, cfg.L, cfg.seed, refine=5, **cfg_kwargs(cfg))
    assert ei.value.code == -1

    cfg = synthdata.get_config("cfg3")
    _, X, T = synthdata.make_problem(cfg, N=20_000)
    X = np.ascontiguousarray(X[:, :8, :])
    Xd, Td = torch.from_numpy(X).cuda(), torch.from_numpy(T).cuda()
    auto = elm.fit(cfg.cell, Xd, Td, cfg.L, cfg.seed, **cfg_kwargs(cfg))
    assert auto.stats.refine_iters == 0 and auto.stats.r_diag_max <= 30 * auto.stats.r_diag_min
    H = auto.H.cpu().numpy()
    assert lstsq.normal_equation_residual(H, T, auto.beta64.cpu().numpy()) <= 1e-5
    _, rss, _ = lstsq.solve_chunked(H, T)
    ref = lstsq.rmse_from_rss(rss, X.shape[0], cfg.m)
    assert abs(auto.stats.rmse - ref) <= 1e-4 * ref
    # the solve entry point has the same policy
    _, b64, st = elm.solve(auto.H, Td, refine=-1)
    assert st.refine_iters == 0 and torch.equal(b64, auto.beta64)
    auto.model.close()


def test_fit_with_spectral_radius_on_a_side_stream_keeps_beta_in_the_model(elm):
    """Everything the fit enqueues, the device part of the weight generation included (Elman layers of 64
    units or more), goes to the caller's stream; the model's beta is the returned one and a predict on
    the same stream uses it."""
    cfg = synthdata.get_config("cfg2")
    _, Xh, Th = synthdata.make_problem(cfg, N=6000)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        X, T = torch.from_numpy(Xh).cuda(), torch.from_numpy(Th).cuda()
        res = elm.fit(cfg.cell, X, T, cfg.L, cfg.seed, stream=side, **cfg_kwargs(cfg))
        Y = elm.predict(res.model, X, stream=side)
    side.synchronize()
    W, U, b, beta = res.model.weights()
    np.testing.assert_array_equal(beta, res.beta64.cpu().numpy())
    rho = np.max(np.abs(np.linalg.eigvals(U.astype(np.float64))))
    assert abs(rho - cfg.spectral_radius) < 1e-6
    Href = ocells.hidden(cfg.cell, Xh, W, U, b)
    assert h_close(res.H.cpu().numpy(), Href)
    # (beta is of order 1e2 on this ill-conditioned layer, so the product is compared on the device's own H)
    np.testing.assert_allclose(Y.cpu().numpy(), res.H.cpu().numpy().astype(np.float64) @ beta,
                               atol=2e-5 * max(1.0, np.abs(Th).max()))
    # a second model made without a stream (default stream) has the same weights
    again = elm.Model.create(cfg.cell, cfg.Q, cfg.d, cfg.L, cfg.m, cfg.seed, **cfg_kwargs(cfg))
    for a, b2 in zip(again.weights()[:3], (W, U, b)):
        np.testing.assert_array_equal(a, b2)
    assert np.all(again.weights()[3] == 0.0)       # beta is zero until a fit or set_beta stores one
    again.close()
    res.model.close()


def test_two_hidden_calls_of_one_multilag_model_on_two_streams(elm):
    """The launch-per-step multi-lag cell keeps the past states of a pass of rows in the caller's workspace,
    so one model serves concurrent calls: two streams, two workspaces, different inputs, both equal to
    the oracle (and to the same calls issued one after the other)."""
    Q, d, L, N = 40, 2, 40, 6000
    assert (Q - 1) * L + d + 1 > 1272
    rng = np.random.default_rng(12)
    a = 0.7 / np.sqrt(L * (Q - 1))
    W = (rng.uniform(-1, 1, (d, L)) / np.sqrt(d)).astype(np.float32)
    A = rng.uniform(-a, a, (Q, L, L)).astype(np.float32)
    b = rng.uniform(-0.5, 0.5, L).astype(np.float32)
    model = elm.Model.from_weights("fc_multilag", Q, 1, W, A, b)
    Xh = [rng.uniform(-1, 1, (N, Q, d)).astype(np.float32) for _ in range(2)]
    Xd = [torch.from_numpy(x).cuda() for x in Xh]
    need = elm.hidden_workspace_bytes("fc_multilag", N, Q, d, L)
    assert need >= (Q - 1) * 6144 * L * 4
    ws = [torch.empty(need, dtype=torch.uint8, device="cuda") for _ in range(2)]
    out = [torch.empty((N, L), dtype=torch.float32, device="cuda") for _ in range(2)]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    torch.cuda.synchronize()
    for rep in range(3):                  # several rounds, so that the two calls really overlap
        for i in range(2):
            elm.hidden(model, Xd[i], out=out[i], workspace=ws[i], stream=streams[i])
    for s in streams:
        s.synchronize()
    serial = [elm.hidden(model, Xd[i]) for i in range(2)]
    torch.cuda.synchronize()
    for i in range(2):
        assert torch.equal(out[i], serial[i])
        assert h_close(out[i].cpu().numpy(), ocells.hidden_fc_multilag(Xh[i], W, A, b))
    # a workspace that is too small is an error, not a fault
    lib = elm.load_library()
    H = out[0]
    rc = lib.elm_rnn_hidden(model._h, Xd[0].data_ptr(), Q * d, d, N, Q, None, None, H.data_ptr(), None,
                            ws[0].data_ptr(), need - 256, None)
    assert rc == -2
    rc = lib.elm_rnn_hidden(model._h, Xd[0].data_ptr(), Q * d, d, N, Q, None, None, H.data_ptr(), None, None, 0, None)
    assert rc == -2
    model.close()


def test_predict_of_the_per_step_multilag_cell_through_workspaces_of_any_size(elm):
    Q, d, L, N = 30, 1, 50, 3000
    rng = np.random.default_rng(13)
    a = 0.7 / np.sqrt(L * (Q - 1))
    W = rng.uniform(-1, 1, (d, L)).astype(np.float32)
    A = rng.uniform(-a, a, (Q, L, L)).astype(np.float32)
    b = rng.uniform(-0.5, 0.5, L).astype(np.float32)
    model = elm.Model.from_weights("fc_multilag", Q, 2, W, A, b)
    beta = rng.standard_normal((L, 2))
    model.set_beta(beta)
    Xh = rng.uniform(-1, 1, (N, Q, d)).astype(np.float32)
    Xd = torch.from_numpy(Xh).cuda()
    want = ocells.hidden_fc_multilag(Xh, W, A, b) @ beta
    lib = elm.load_library()
    full = int(lib.elm_rnn_predict_workspace_bytes(model._h, N))
    one = int(lib.elm_rnn_predict_workspace_bytes(model._h, 256))
    assert full == (N * L * 4 + 255) // 256 * 256 + elm.hidden_workspace_bytes("fc_multilag", N, Q, d, L) > one
    for nbytes in (full, (full + one) // 2, one):
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        Y = elm.predict(model, Xd, workspace=ws).cpu().numpy()
        np.testing.assert_allclose(Y, want, atol=2e-5 * np.abs(want).max())
    Y = torch.empty((N, 2), dtype=torch.float32, device="cuda")
    small = torch.empty(one - 256, dtype=torch.uint8, device="cuda")
    rc = lib.elm_rnn_predict(model._h, Xd.data_ptr(), Q * d, d, N, Y.data_ptr(), small.data_ptr(), small.numel(), None)
    assert rc == -2
    model.close()


def test_binding_checks_h_out_and_releases_the_model_of_a_rank_deficient_fit(elm):
    rng = np.random.default_rng(14)
    X = torch.from_numpy(rng.uniform(-1, 1, (500, 3, 2)).astype(np.float32)).cuda()
    T = torch.from_numpy(rng.standard_normal((500, 1)).astype(np.float32)).cuda()
    for bad in (torch.empty((499, 16), device="cuda"), torch.empty((500, 17), device="cuda"),
                torch.empty((500, 32), device="cuda")[:, ::2], torch.empty((500, 16), device="cuda", dtype=torch.float64),
                torch.empty((500, 16))):
        with pytest.raises((ValueError, TypeError)):
            elm.fit("elman", X, T, 16, seed=1, H_out=bad)
    # all-zero windows and zero biases: every pre-activation is exactly 0, so H = tanh(0) = 0 and every
    # column vanishes exactly (the case float32 is guaranteed to flag)
    Z = torch.zeros((500, 3, 2), device="cuda")
    with pytest.raises(elm.ElmRnnError) as ei:
        elm.fit("elman", Z, T, 16, seed=1, zero_bias=True)
    assert ei.value.code == -3
    with pytest.raises(elm.ElmRnnError) as ei:
        elm.fit_streamed("elman", Z, T, 16, seed=1, zero_bias=True)
    assert ei.value.code == -3
    res = elm.fit("elman", Z, T, 16, seed=1, zero_bias=True, allow_rank_deficient=True)
    assert res.stats.rank_deficient and float(res.H.abs().max()) == 0.0
    res.model.close()
