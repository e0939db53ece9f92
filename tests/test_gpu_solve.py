"""GPU parity: TSQR + back-solve + refinement against the float64 Householder oracle.

Stage-isolated: the oracle solves the very H the GPU is given.  Bars (from the benchmark's
statement): training RMSE within 1e-4 relative; normal-equation residual
||H^T r|| / (||H|| ||r||) <= 1e-5, evaluated here independently in float64 on the returned beta.
beta itself is unique for full-column-rank H and is compared where the conditioning allows.
"""
import numpy as np
import pytest
import torch

from oracle import lstsq

pytestmark = pytest.mark.gpu


def make_system(N, L, m, seed, cond=10.0, noise=0.1):
    rng = np.random.default_rng(seed)
    H = rng.standard_normal((N, L))
    if L > 1:
        # spread the column scales to reach the requested conditioning (cheaply, no SVD of N x L)
        H = H @ (np.linalg.qr(rng.standard_normal((L, L)))[0] * np.geomspace(1.0, 1.0 / cond, L))
    beta_true = rng.standard_normal((L, m))
    T = H @ beta_true + noise * rng.standard_normal((N, m))
    return H.astype(np.float32), T.astype(np.float32)


def check_against_oracle(elm, H, T, beta_rtol):
    Hd, Td = torch.from_numpy(H).cuda(), torch.from_numpy(T).cuda()
    beta32, beta64, st = elm.solve(Hd, Td)
    b64 = beta64.cpu().numpy()
    N, L = H.shape
    m = T.shape[1]
    solver = lstsq.solve if N * (L + m) <= 4_000_000 else lstsq.solve_chunked
    ref_beta, ref_rss, _ = solver(H, T)
    ref_rmse = lstsq.rmse_from_rss(ref_rss, N, m)
    rmse_gpu_beta = float(np.sqrt(np.mean((H.astype(np.float64) @ b64 - T) ** 2)))
    assert abs(rmse_gpu_beta - ref_rmse) <= 1e-4 * ref_rmse
    assert abs(st.rmse - ref_rmse) <= 1e-4 * ref_rmse
    assert abs(st.rmse_qr - ref_rmse) <= 2e-3 * ref_rmse + 1e-6      # read off the float32 R factor
    ne = lstsq.normal_equation_residual(H, T, b64)
    assert ne <= 1e-5, ne
    assert abs(st.ne_resid - ne) <= 0.5 * ne + 1e-9
    if beta_rtol is not None:
        np.testing.assert_allclose(b64, ref_beta, rtol=0, atol=beta_rtol * np.abs(ref_beta).max())
    np.testing.assert_allclose(beta32.cpu().numpy(), b64.astype(np.float32), rtol=0, atol=0)
    assert st.r_diag_min > 0 and st.r_diag_max >= st.r_diag_min
    return st


@pytest.mark.parametrize("N,L,m", [
    (64, 8, 1), (100, 31, 2), (1000, 33, 1), (777, 64, 3), (5000, 100, 1), (3001, 129, 2),
    (20000, 260, 4), (9000, 512, 2), (70000, 96, 1), (600, 511, 16),
    # widths whose 128-row block does not fit LDS: twelve column tiles in registers, the rest in LDS (none at
    # 289 + 1 columns ... five at 512 + 16), ragged last block, single and several targets
    (8192, 289, 1), (16500, 330, 4), (12345, 384, 16), (33000, 448, 1), (8200, 496, 16),
])
def test_solve_matches_oracle(elm, N, L, m):
    H, T = make_system(N, L, m, seed=N + L)
    check_against_oracle(elm, H, T, beta_rtol=1e-6)


@pytest.mark.parametrize("N,L,m", [
    # either side of every switch between the fold kernels: 8,192 rows (64- or 128-row blocks), 288 padded
    # columns (128-row block in LDS or in registers), 384 padded columns (no tile or one tile left in LDS),
    # targets that straddle two column tiles
    (8191, 287, 1), (8192, 287, 1), (8191, 288, 1), (8192, 288, 1), (8193, 319, 2), (8192, 383, 1),
    (8192, 384, 1), (8320, 385, 16), (8191, 500, 16), (8192, 500, 16),
])
def test_solve_at_the_kernel_selection_boundaries(elm, N, L, m):
    H, T = make_system(N, L, m, seed=7 * N + L)
    check_against_oracle(elm, H, T, beta_rtol=1e-6)


def test_ill_conditioned_system_meets_the_residual_bar_after_refinement(elm):
    # cond ~ 1e5: a float32 factorisation alone leaves a residual of 1e-4 .. 1e-3
    H, T = make_system(20000, 80, 1, seed=9, cond=1e5, noise=0.02)
    st = check_against_oracle(elm, H, T, beta_rtol=None)
    Hd, Td = torch.from_numpy(H).cuda(), torch.from_numpy(T).cuda()
    _, b0, st0 = elm.solve(Hd, Td, refine=0)
    assert st0.refine_iters == 0 and st.refine_iters == 2
    assert st.ne_resid < st0.ne_resid


def test_planted_solution_and_scaling(elm):
    rng = np.random.default_rng(3)
    H = rng.standard_normal((4000, 50)).astype(np.float32)
    beta_star = rng.standard_normal((50, 2))
    T = (H.astype(np.float64) @ beta_star).astype(np.float32)
    Hd = torch.from_numpy(H).cuda()
    _, b64, st = elm.solve(Hd, torch.from_numpy(T).cuda())
    np.testing.assert_allclose(b64.cpu().numpy(), beta_star, atol=2e-6)
    assert st.rmse < 1e-6
    _, b3, _ = elm.solve(Hd, torch.from_numpy(3.0 * T).cuda())
    np.testing.assert_allclose(b3.cpu().numpy(), 3.0 * b64.cpu().numpy(), atol=1e-5)


def test_row_permutation_invariance(elm):
    H, T = make_system(6000, 40, 2, seed=21)
    perm = np.random.default_rng(22).permutation(6000)
    _, b1, _ = elm.solve(torch.from_numpy(H).cuda(), torch.from_numpy(T).cuda())
    _, b2, _ = elm.solve(torch.from_numpy(H[perm].copy()).cuda(), torch.from_numpy(T[perm].copy()).cuda())
    np.testing.assert_allclose(b1.cpu().numpy(), b2.cpu().numpy(), atol=1e-9)


def test_rank_deficiency_and_argument_errors(elm):
    # an exactly vanishing column survives float32 rounding as an exact zero on R's diagonal
    # (a duplicated column does not: its R_jj is rounding noise a few eps32 above the threshold)
    H, T = make_system(500, 12, 1, seed=5)
    H[:, 7] = 0.0
    Hd, Td = torch.from_numpy(H).cuda(), torch.from_numpy(T).cuda()
    with pytest.raises(elm.ElmRnnError) as ei:
        elm.solve(Hd, Td)
    assert ei.value.code == -3
    _, _, st = elm.solve(Hd, Td, allow_rank_deficient=True)
    assert st.rank_deficient
    with pytest.raises(lstsq.RankDeficient):
        lstsq.solve(H, T)
    # N < L
    with pytest.raises(elm.ElmRnnError) as ei:
        elm.solve(Hd[:5], Td[:5])
    assert ei.value.code == -1
    # workspace too small
    small = torch.empty(1024, dtype=torch.uint8, device="cuda")
    H2, T2 = make_system(500, 12, 1, seed=6)
    with pytest.raises(elm.ElmRnnError) as ei:
        elm.solve(torch.from_numpy(H2).cuda(), torch.from_numpy(T2).cuda(), workspace=small)
    assert ei.value.code == -2
