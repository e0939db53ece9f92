"""The solve entry point that allocates nothing (elm_rnn_solve_static: its workspace is a static device
array) against elm_rnn_solve with a caller workspace, through the C ABI: two calls in a row, the second
on a smaller system, so that what the first call left in the array must not leak into the second."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import lstsq

pytestmark = pytest.mark.gpu


def system(N, L, m, seed):
    rng = np.random.default_rng(seed)
    H = rng.standard_normal((N, L)).astype(np.float32)
    T = (H @ rng.standard_normal((L, m)) + 0.3 * rng.standard_normal((N, m))).astype(np.float32)
    return torch.from_numpy(H).cuda(), torch.from_numpy(T).cuda()


def call(lib, elm, fn_static, H, T, refine):
    from paper_1911_13252_amd.binding import _Stats
    N, L = H.shape
    m = T.shape[1]
    b32 = torch.empty((L, m), dtype=torch.float32, device="cuda")
    b64 = torch.empty((L, m), dtype=torch.float64, device="cuda")
    st = _Stats()
    stream = torch.cuda.current_stream().cuda_stream
    if fn_static:
        rc = lib.elm_rnn_solve_static(H.data_ptr(), T.data_ptr(), N, L, m, refine, b32.data_ptr(), b64.data_ptr(),
                                      C.byref(st), stream)
    else:
        ws = torch.empty(elm.solve_workspace_bytes(N, L, m), dtype=torch.uint8, device="cuda")
        rc = lib.elm_rnn_solve(H.data_ptr(), T.data_ptr(), N, L, m, refine, b32.data_ptr(), b64.data_ptr(),
                               C.byref(st), ws.data_ptr(), ws.numel(), stream)
    assert rc == 0, rc
    return b32.cpu().numpy(), b64.cpu().numpy(), st


def test_static_scratch_solve_matches_the_workspace_solve_on_two_calls_in_a_row(elm):
    lib = elm.load_library()
    limit = int(lib.elm_rnn_solve_static_scratch_bytes())
    assert limit == 64 << 20
    # first a wide system whose default plan does not fit the array (fewer level-0 R factors are used),
    # then a smaller one whose plan does fit (then both entry points run the same plan: identical bits),
    # then the wide one again
    cases = [(40_000, 300, 2, 1), (3000, 40, 3, 2), (40_000, 300, 2, 1)]
    for N, L, m, seed in cases:
        H, T = system(N, L, m, seed)
        fits = elm.solve_workspace_bytes(N, L, m) <= limit
        for refine in (0, 2):
            s32, s64, sst = call(lib, elm, True, H, T, refine)
            w32, w64, wst = call(lib, elm, False, H, T, refine)
            if fits:
                np.testing.assert_array_equal(s64, w64)
                np.testing.assert_array_equal(s32, w32)
                assert sst.rmse == wst.rmse
            else:
                np.testing.assert_allclose(s64, w64, rtol=0, atol=2e-6 * np.abs(w64).max())
            assert abs(sst.rmse - wst.rmse) <= 1e-6 * wst.rmse
            assert sst.refine_iters == refine
            # and against the oracle, to the same bars as the workspace solve
            Hh, Th = H.cpu().numpy(), T.cpu().numpy()
            ref, rss, _ = lstsq.solve_chunked(Hh, Th)
            ref_rmse = lstsq.rmse_from_rss(rss, N, m)
            assert abs(sst.rmse - ref_rmse) <= 1e-4 * ref_rmse
            if refine:
                assert lstsq.normal_equation_residual(Hh, Th, s64) <= 1e-5
    # a system that cannot fit: one 544 x 544 R factor is fine, but 16 outputs at 512 units need
    # 1024 x 8194 float64 partial sums
    H, T = system(1024, 512, 16, 3)
    b32 = torch.empty((512, 16), dtype=torch.float32, device="cuda")
    rc = lib.elm_rnn_solve_static(H.data_ptr(), T.data_ptr(), 1024, 512, 16, 0, b32.data_ptr(), None, None, None)
    assert rc == -5
    assert b"static scratch" in lib.elm_rnn_last_hip_error()
    assert lib.elm_rnn_solve_static(None, T.data_ptr(), 1024, 512, 16, 0, b32.data_ptr(), None, None, None) == -1
