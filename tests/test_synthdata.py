"""Checks of the seeded input generators (CPU only)."""
import numpy as np

import synthdata


def test_univariate_series_is_minmax_scaled():
    s = synthdata.make_series(2010, 1, 13252, 0.05)
    assert s.shape == (2010, 1) and s.min() == 0.0 and s.max() == 1.0


def test_multivariate_series_is_zscored():
    s = synthdata.make_series(5000, 4, 13254, 0.05)
    np.testing.assert_allclose(s.mean(axis=0), 0.0, atol=1e-12)
    np.testing.assert_allclose(s.std(axis=0), 1.0, atol=1e-12)


def test_windows_and_targets():
    cfg = synthdata.get_config("cfg3")
    series, X, T = synthdata.make_problem(cfg, N=300)
    assert X.shape == (300, cfg.Q, cfg.d) and T.shape == (300, cfg.m)
    assert X.dtype == np.float32 and T.dtype == np.float32
    for i in (0, 17, 299):
        for t in (0, 5, cfg.Q - 1):
            np.testing.assert_array_equal(X[i, t], series[i + t])
        np.testing.assert_array_equal(T[i], series[i + cfg.Q, :cfg.m])
    _, Xv, Tv = synthdata.make_problem(cfg, N=300, materialise=False)
    np.testing.assert_array_equal(Xv, X)
    assert Xv.strides[0] == series.strides[0]


def test_config_table_matches_the_benchmark_description():
    c = {x.name: x for x in synthdata.CONFIGS}
    assert (c["cfg1"].cell, c["cfg1"].N, c["cfg1"].Q, c["cfg1"].L) == ("elman", 2000, 10, 32)
    assert (c["cfg2"].N, c["cfg2"].Q, c["cfg2"].L) == (100000, 20, 100)
    assert (c["cfg3"].cell, c["cfg3"].N, c["cfg3"].Q, c["cfg3"].d, c["cfg3"].L, c["cfg3"].m) == ("lstm", 200000, 50, 4, 128, 1)
    assert (c["cfg4"].cell, c["cfg4"].N, c["cfg4"].L, c["cfg4"].m, c["cfg4"].zero_bias) == ("gru", 1000000, 256, 4, True)
    assert (c["cfg5"].cell, c["cfg5"].N, c["cfg5"].Q, c["cfg5"].d, c["cfg5"].L, c["cfg5"].m) == ("lstm", 4000000, 100, 8, 512, 2)


def test_determinism():
    a = synthdata.make_series(1000, 8, 13256, 0.1)
    b = synthdata.make_series(1000, 8, 13256, 0.1)
    np.testing.assert_array_equal(a, b)
