"""End-to-end checks of the oracle on the small benchmark configuration (CPU only)."""
import numpy as np

import synthdata
from oracle import cells, fit, lstsq


def test_fit_cfg1_end_to_end_properties():
    cfg = synthdata.get_config("cfg1")
    _, X, T = synthdata.make_problem(cfg)
    out = fit.fit(cfg.cell, X, T, cfg.L, cfg.seed, w_scale=cfg.w_scale,
                  spectral_radius=cfg.spectral_radius)
    H, beta = out["H"], out["beta"]
    assert H.shape == (cfg.N, cfg.L) and beta.shape == (cfg.L, 1)
    assert np.all(np.abs(H) < 1.0)
    # the fit beats predicting the mean and the residual is orthogonal to H
    assert out["rmse"] < 0.5 * T.std()
    assert lstsq.normal_equation_residual(H, T, beta) < 1e-9
    np.testing.assert_allclose(out["rmse"], np.sqrt(np.mean((H @ beta - T) ** 2)), rtol=1e-9)
    # prediction on the training windows reproduces H beta
    yhat = fit.predict(cfg.cell, X, out["W"], out["U"], out["b"], beta)
    np.testing.assert_allclose(yhat, H @ beta, atol=1e-12)


def test_fit_large_N_path_equals_one_shot():
    cfg = synthdata.get_config("cfg3")
    _, X, T = synthdata.make_problem(cfg, N=1500)
    a = fit.fit(cfg.cell, X, T, 16, cfg.seed, w_scale=cfg.w_scale, forget_bias=1.0, chunk=8192)
    b = fit.fit(cfg.cell, X, T, 16, cfg.seed, w_scale=cfg.w_scale, forget_bias=1.0, chunk=400)
    np.testing.assert_allclose(b["H"], a["H"], atol=1e-14)
    np.testing.assert_allclose(b["beta"], a["beta"], rtol=0, atol=1e-9 * np.abs(a["beta"]).max())
    np.testing.assert_allclose(b["rmse"], a["rmse"], rtol=1e-10)
