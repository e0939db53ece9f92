"""GPU parity of the streamed fit (H produced and folded into the TSQR chunk by chunk, never stored).

The streamed entry point returns no H, so the tests rebuild it with elm_rnn_hidden from the fitted
model (same kernels, same bits) and hold the returned beta to the bars of the ordinary fit on that H:
training RMSE within 1e-4 relative of the float64 Householder oracle, normal-equation residual <= 1e-5.
"""
import math

import numpy as np
import pytest
import torch

import synthdata
from oracle import lstsq

pytestmark = pytest.mark.gpu


def cfg_kwargs(cfg):
    return dict(w_scale=cfg.w_scale, spectral_radius=cfg.spectral_radius,
                forget_bias=cfg.forget_bias, zero_bias=cfg.zero_bias)


def problem(name, n, L=None, Q=None):
    cfg = synthdata.get_config(name)
    _, X, T = synthdata.make_problem(cfg, N=n)
    if Q is not None:
        X = np.ascontiguousarray(X[:, :Q, :])
    return cfg, X, T, (cfg.L if L is None else L)


def check_against_oracle(elm, res, Xd, T):
    """RMSE and normal-equation residual of res.beta64 on the H the model produces."""
    H = elm.hidden(res.model, Xd).cpu().numpy()
    b64 = res.beta64.cpu().numpy()
    n, m = T.shape
    solver = lstsq.solve if n <= 8192 else lstsq.solve_chunked
    _, ref_rss, _ = solver(H, T)
    ref_rmse = lstsq.rmse_from_rss(ref_rss, n, m)
    rmse = float(np.sqrt(np.mean((H.astype(np.float64) @ b64 - T) ** 2)))
    assert abs(rmse - ref_rmse) <= 1e-4 * ref_rmse, (rmse, ref_rmse)
    ne = lstsq.normal_equation_residual(H, T, b64)
    assert ne <= 1e-5, ne
    np.testing.assert_array_equal(res.model.weights()[3], b64)
    return H, rmse, ne


CASES = [  # name, N, L, chunk_rows, contraction
    ("cfg1", 2000, 32, 512, "fp32"),            # ill-conditioned Elman: the automatic mode refines
    ("cfg2", 20_000, 100, 4096, "fp32"),
    ("cfg2", 20_000, 100, 4096, "split16"),
    ("cfg3", 30_000, 128, 8192, "fp32"),        # ragged last chunk (30000 = 3 * 8192 + 5424)
    ("cfg3", 30_000, 128, 8192, "split16"),
    ("cfg4", 20_000, 256, 4096, "fp32"),
    ("cfg5", 12_345, 512, 4000, "fp32"),        # chunk rounded up to 4096, ragged blocks and tail
    ("cfg5", 12_345, 512, 4000, "split16"),
    ("paper_elman", 20_000, 100, 4096, "fp32"),
    ("paper_fc", 20_000, 100, 4096, "fp32"),
]


@pytest.mark.parametrize("name,n,L,chunk,mode", CASES)
def test_streamed_fit_meets_the_bars_of_the_ordinary_fit(elm, name, n, L, chunk, mode):
    cfg, X, T, L = problem(name, n, L)
    Xd, Td = torch.from_numpy(X).cuda(), torch.from_numpy(T).cuda()
    res = elm.fit_streamed(cfg.cell, Xd, Td, L, cfg.seed, contraction=mode, chunk_rows=chunk, **cfg_kwargs(cfg))
    assert res.H is None
    _, rmse, ne = check_against_oracle(elm, res, Xd, T)
    st = res.stats
    assert st.t_hidden_ms > 0 and st.t_solve_ms > 0
    assert abs(st.rmse_qr - rmse) <= 1e-3 * rmse
    if st.refine_iters > 0:        # statistics come from a float64 pass over the recomputed H
        assert st.refine_iters == 2 and st.r_diag_max > 30 * st.r_diag_min
        assert abs(st.rmse - rmse) <= 1e-9 * rmse + 1e-12
        assert abs(st.ne_resid - ne) <= 0.5 * ne + 1e-12
    else:                          # well conditioned: no second pass, statistics read off R
        assert st.r_diag_max <= 30 * st.r_diag_min
        assert st.rmse == st.rmse_qr and math.isnan(st.ne_resid)
    # the ordinary fit of the same problem returns the same model and (up to float32 factorisation
    # rounding, removed by refinement where it matters) the same beta
    ref = elm.fit(cfg.cell, Xd, Td, L, cfg.seed, contraction=mode, **cfg_kwargs(cfg))
    for a, b in zip(ref.model.weights()[:3], res.model.weights()[:3]):
        np.testing.assert_array_equal(a, b)
    assert abs(ref.stats.rmse - rmse) <= 1e-6 * rmse
    ref.model.close()
    res.model.close()


FUSED_CASES = [  # data, cell, N, L: every stage-1 variant that has the in-kernel hand-off (tile -> fold through LDS)
    ("cfg3", "lstm", 5000, 160),      # two column chunks
    ("cfg3", "lstm", 5001, 300),      # three chunks, two-pass with LDS staging
    ("cfg5", "lstm", 4003, 512),      # four chunks (the headline variant)
    ("cfg5", "lstm", 8300, 512),      # ... with enough rows for the combine levels to fold 128-row slices
    ("cfg5", "elman", 4100, 320),     # three chunks (8 input channels keep the wide layer well conditioned)
    ("cfg5", "elman", 4099, 512),     # four chunks
    ("cfg4", "gru", 4500, 288),       # 64-row tiles
    ("cfg4", "gru", 4501, 320),       # 32-row tiles, three chunks
    ("cfg4", "gru", 4001, 448),       # 32-row tiles, four chunks
    # layers of 65 .. 128 / 256 units: two work-groups per compute unit, 32-row folds
    ("cfg3", "lstm", 5003, 96),
    ("cfg3", "lstm", 3000, 128),
    ("cfg5", "elman", 4100, 100),
    ("cfg5", "elman", 4101, 200),
    ("cfg4", "gru", 4502, 72),
    ("cfg4", "gru", 4503, 256),
]


@pytest.mark.parametrize("name,cell,n,L", FUSED_CASES)
def test_fused_hand_off_meets_the_bars_of_the_ordinary_fit(elm, name, cell, n, L):
    """chunk_rows = -1: stage 1 folds every finished tile into the TSQR inside the kernel."""
    import dataclasses
    cfg, X, T, L = problem(name, n, L, Q=6)
    if cell != cfg.cell:
        cfg = dataclasses.replace(cfg, cell=cell, w_scale=0.3, spectral_radius=0.9, forget_bias=0.0, zero_bias=False)
    Xd, Td = torch.from_numpy(X).cuda(), torch.from_numpy(T).cuda()
    res = elm.fit_streamed(cfg.cell, Xd, Td, L, cfg.seed, chunk_rows=-1, **cfg_kwargs(cfg))
    H, rmse, ne = check_against_oracle(elm, res, Xd, T)
    assert abs(res.stats.rmse_qr - rmse) <= 1e-3 * rmse
    # the R factor is the one the chunked path builds from the stored tiles: same diagonal range, same beta
    alt = elm.fit_streamed(cfg.cell, Xd, Td, L, cfg.seed, chunk_rows=1024, **cfg_kwargs(cfg))
    assert alt.stats.refine_iters == res.stats.refine_iters
    assert abs(alt.stats.r_diag_min - res.stats.r_diag_min) <= 1e-3 * res.stats.r_diag_min
    assert abs(alt.stats.r_diag_max - res.stats.r_diag_max) <= 1e-4 * res.stats.r_diag_max
    b, a = res.beta64.cpu().numpy(), alt.beta64.cpu().numpy()
    # both are least-squares solutions to float32 factorisation accuracy: compare the fitted values
    Hd = H.astype(np.float64)
    assert np.abs(Hd @ (a - b)).max() <= 1e-4 * max(np.abs(T).max(), 1.0)
    alt.model.close()
    res.model.close()


def test_fused_hand_off_is_refused_where_no_variant_exists(elm):
    cfg, X, T, L = problem("cfg3", 3000, 64)       # at most 64 units: the waves split the rows of the tile
    Xd, Td = torch.from_numpy(X).cuda(), torch.from_numpy(T).cuda()
    with pytest.raises(elm.ElmRnnError) as err:
        elm.fit_streamed(cfg.cell, Xd, Td, L, cfg.seed, chunk_rows=-1, **cfg_kwargs(cfg))
    assert err.value.code == -5
    with pytest.raises(elm.ElmRnnError) as err:       # the split contraction has no fused form
        elm.fit_streamed(cfg.cell, Xd, Td, 160, cfg.seed, chunk_rows=-1, contraction="split16", **cfg_kwargs(cfg))
    assert err.value.code == -5
    with pytest.raises(elm.ElmRnnError) as err:
        elm.fit_streamed(cfg.cell, Xd, Td, L, cfg.seed, chunk_rows=-2, **cfg_kwargs(cfg))
    assert err.value.code == -1


def test_streamed_fit_is_independent_of_the_chunking(elm):
    cfg, X, T, L = problem("cfg3", 20_000, 96)
    Xd, Td = torch.from_numpy(X).cuda(), torch.from_numpy(T).cuda()
    betas = []
    for chunk in (20_000, 6000, 128):
        res = elm.fit_streamed(cfg.cell, Xd, Td, L, cfg.seed, chunk_rows=chunk, refine=2, **cfg_kwargs(cfg))
        assert res.stats.refine_iters == 2 and res.stats.ne_resid <= 1e-9
        betas.append(res.beta64.cpu().numpy())
        res.model.close()
    scale = np.abs(betas[0]).max()
    for b in betas[1:]:
        np.testing.assert_allclose(b, betas[0], rtol=0, atol=1e-7 * scale)


def test_streamed_fit_explicit_refinement_matches_the_ordinary_fit(elm):
    cfg, X, T, L = problem("cfg2", 20_000, 100)
    Xd, Td = torch.from_numpy(X).cuda(), torch.from_numpy(T).cuda()
    ref = elm.fit(cfg.cell, Xd, Td, L, cfg.seed, **cfg_kwargs(cfg))
    plain = elm.fit_streamed(cfg.cell, Xd, Td, L, cfg.seed, chunk_rows=4096, refine=0, **cfg_kwargs(cfg))
    fine = elm.fit_streamed(cfg.cell, Xd, Td, L, cfg.seed, chunk_rows=4096, refine=2, **cfg_kwargs(cfg))
    assert plain.stats.refine_iters == 0 and math.isnan(plain.stats.ne_resid)
    assert fine.stats.refine_iters == 2 and fine.stats.ne_resid <= 1e-5
    assert abs(fine.stats.rmse - ref.stats.rmse) <= 1e-9 * ref.stats.rmse
    # the unrefined float32 solution of this ill-conditioned system already has the right RMSE
    assert abs(plain.stats.rmse - ref.stats.rmse) <= 1e-4 * ref.stats.rmse
    # stage 1 ran three times as often with two refinement steps and the statistics pass
    assert fine.stats.t_hidden_ms > 2.0 * plain.stats.t_hidden_ms
    for r in (ref, plain, fine):
        r.model.close()


def test_streamed_fit_workspace(elm):
    n, L, m = 4_000_000, 512, 2
    streamed = elm.fit_streamed_workspace_bytes(n, L, m)
    whole = elm.fit_workspace_bytes(n, L, m, True)
    assert whole - streamed > 8_000_000_000 and streamed < 600_000_000
    assert elm.fit_streamed_workspace_bytes(n, L, m, 1000) - elm.solve_workspace_bytes(n, L, m) == 1024 * L * 4
    cfg, X, T, L = problem("cfg3", 5000, 64)
    Xd, Td = torch.from_numpy(X).cuda(), torch.from_numpy(T).cuda()
    small = torch.empty(elm.fit_streamed_workspace_bytes(5000, L, 1, 1024) - 256, dtype=torch.uint8, device="cuda")
    with pytest.raises(elm.ElmRnnError) as err:
        elm.fit_streamed(cfg.cell, Xd, Td, L, cfg.seed, chunk_rows=1024, workspace=small, **cfg_kwargs(cfg))
    assert err.value.code == -2
    with pytest.raises(elm.ElmRnnError):
        elm.fit_streamed(cfg.cell, Xd, Td, L, cfg.seed, refine=7, **cfg_kwargs(cfg))


def test_streamed_fit_cfg5_full_size(elm):
    """The headline configuration at full size in the default mode (in-kernel hand-off), as bench.py launches it."""
    cfg = synthdata.get_config("cfg5")
    series, _, T = synthdata.make_problem(cfg, materialise=False)
    sd = torch.from_numpy(series).cuda()
    Xd = torch.as_strided(sd, (cfg.N, cfg.Q, cfg.d), (cfg.d, cfg.d, 1)).contiguous()
    Td = torch.from_numpy(T).cuda()
    torch.cuda.reset_peak_memory_stats()
    base = torch.cuda.memory_allocated()
    res = elm.fit_streamed(cfg.cell, Xd, Td, cfg.L, cfg.seed, **cfg_kwargs(cfg))
    assert torch.cuda.max_memory_allocated() - base < 700_000_000      # no 8 GB hidden matrix
    assert res.stats.refine_iters == 0 and res.stats.r_diag_max <= 30 * res.stats.r_diag_min
    H = elm.hidden(res.model, Xd)
    del Xd
    b64 = res.beta64
    g = torch.zeros((cfg.L, cfg.m), dtype=torch.float64, device="cuda")
    rss = torch.zeros((), dtype=torch.float64, device="cuda")
    h2 = torch.zeros((), dtype=torch.float64, device="cuda")
    for s in range(0, cfg.N, 262144):
        Hc = H[s:s + 262144].double()
        rc = Hc @ b64 - Td[s:s + 262144].double()
        g += Hc.T @ rc
        rss += (rc * rc).sum()
        h2 += (Hc * Hc).sum()
    rmse = float(torch.sqrt(rss / (cfg.N * cfg.m)))
    ne = float(torch.linalg.norm(g) / (torch.sqrt(h2) * torch.sqrt(rss)))
    assert ne <= 1e-5, ne
    assert abs(res.stats.rmse - rmse) <= 1e-4 * rmse
    assert rmse < 1.0
    res.model.close()


def test_predict_through_a_small_workspace(elm):
    """elm_rnn_predict chunks H through whatever workspace it is given: same Y, bit for bit."""
    cfg, X, T, L = problem("cfg3", 10_000, 96)
    Xd, Td = torch.from_numpy(X).cuda(), torch.from_numpy(T).cuda()
    res = elm.fit_streamed(cfg.cell, Xd, Td, L, cfg.seed, **cfg_kwargs(cfg))
    Y = elm.predict(res.model, Xd)
    for rows in (256, 1000, 4096):
        ws = torch.empty(rows * L * 4, dtype=torch.uint8, device="cuda")
        assert torch.equal(elm.predict(res.model, Xd, workspace=ws), Y)
    H = elm.hidden(res.model, Xd).double()
    ref = (H @ res.beta64).cpu().numpy()
    np.testing.assert_allclose(Y.cpu().numpy(), ref, atol=2e-5 * max(1.0, np.abs(T).max()))
    with pytest.raises(elm.ElmRnnError) as err:
        elm.predict(res.model, Xd, workspace=torch.empty(255 * L * 4, dtype=torch.uint8, device="cuda"))
    assert err.value.code == -2
    res.model.close()
