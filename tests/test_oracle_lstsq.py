"""Pins for the oracle's Householder least squares (CPU only).

Pinned against the normal equations, the SVD pseudo-inverse, planted
solutions, orthogonality of the residual, the Gram identity and invariances.
"""
import numpy as np
import pytest

from oracle import lstsq


def problem(N, L, m, seed, cond=None):
    rng = np.random.default_rng(seed)
    H = rng.standard_normal((N, L))
    if cond is not None:
        u, _, vt = np.linalg.svd(H, full_matrices=False)
        H = (u * np.geomspace(1.0, 1.0 / cond, L)) @ vt
    T = rng.standard_normal((N, m))
    return H, T


@pytest.mark.parametrize("N,L,m", [(64, 8, 3), (20, 5, 1), (9, 8, 2), (40, 1, 1)])
def test_equals_normal_equations_and_svd_pseudo_inverse(N, L, m):
    H, T = problem(N, L, m, seed=N + L, cond=1e3 if L > 1 else None)
    beta, rss, _ = lstsq.solve(H, T)
    ne = np.linalg.solve(H.T @ H, H.T @ T)            # (H^T H)^{-1} H^T T
    u, s, vt = np.linalg.svd(H, full_matrices=False)
    pinv = (vt.T / s) @ (u.T @ T)                     # V S^{-1} U^T T
    np.testing.assert_allclose(beta, pinv, rtol=0, atol=1e-10 * np.abs(pinv).max())
    np.testing.assert_allclose(beta, ne, rtol=0, atol=1e-8 * np.abs(ne).max())
    np.testing.assert_allclose(rss, np.sum((H @ pinv - T) ** 2), rtol=1e-10)


def test_planted_solution_is_recovered():
    H, _ = problem(200, 12, 1, seed=3)
    beta_star = np.random.default_rng(4).standard_normal((12, 3))
    beta, rss, _ = lstsq.solve(H, H @ beta_star)
    np.testing.assert_allclose(beta, beta_star, atol=1e-12)
    assert rss < 1e-22


def test_residual_is_orthogonal_to_the_columns_of_H():
    H, T = problem(500, 20, 2, seed=5, cond=1e4)
    beta, _, _ = lstsq.solve(H, T)
    assert lstsq.normal_equation_residual(H, T, beta) <= 1e-12


def test_gram_identity_and_residual_norm():
    H, T = problem(300, 10, 2, seed=6)
    beta, rss, R = lstsq.solve(H, T)
    A = np.hstack([H, T])
    G = A.T @ A
    L = 10
    np.testing.assert_allclose(R[:, :L].T @ R[:, :L], G[:L, :L], atol=1e-10)   # R11^T R11 = H^T H
    np.testing.assert_allclose(R[:, :L].T @ R[:, L:], G[:L, L:], atol=1e-10)   # R11^T R12 = H^T T
    np.testing.assert_allclose(R[:, L:].T @ R[:, L:], G[L:, L:] - (T - H @ beta).T @ (T - H @ beta),
                               atol=1e-9)
    np.testing.assert_allclose(rss, np.sum((T - H @ beta) ** 2), rtol=1e-12)
    assert np.all(np.tril(R[:, :L], -1) == 0.0)


def test_invariance_under_row_permutation_and_chunking():
    H, T = problem(1000, 16, 2, seed=7, cond=100)
    beta, rss, R = lstsq.solve(H, T)
    perm = np.random.default_rng(8).permutation(1000)
    beta_p, rss_p, R_p = lstsq.solve(H[perm], T[perm])
    np.testing.assert_allclose(beta_p, beta, atol=1e-11)
    np.testing.assert_allclose(np.abs(R_p), np.abs(R), atol=1e-10)   # R unique up to row signs
    for chunk in (16, 37, 250, 5000):
        beta_c, rss_c, R_c = lstsq.solve_chunked(H, T, chunk=chunk)
        np.testing.assert_allclose(beta_c, beta, atol=1e-11)
        np.testing.assert_allclose(rss_c, rss, rtol=1e-11)
        np.testing.assert_allclose(np.abs(R_c), np.abs(R), atol=1e-10)


def test_chunks_smaller_than_L_are_carried():
    H, T = problem(50, 12, 1, seed=9)
    beta, rss, _ = lstsq.solve(H, T)
    beta_c, rss_c, _ = lstsq.solve_chunked(H, T, chunk=5)
    np.testing.assert_allclose(beta_c, beta, atol=1e-12)
    np.testing.assert_allclose(rss_c, rss, rtol=1e-11)


def test_linear_in_T():
    H, T = problem(120, 7, 2, seed=10)
    b1, _, _ = lstsq.solve(H, T[:, :1])
    b2, _, _ = lstsq.solve(H, T[:, 1:])
    b12, _, _ = lstsq.solve(H, T)
    np.testing.assert_allclose(b12, np.hstack([b1, b2]), atol=1e-13)
    bs, rs, _ = lstsq.solve(H, 3.0 * T[:, :1] - 2.0 * T[:, 1:])
    np.testing.assert_allclose(bs, 3.0 * b1 - 2.0 * b2, atol=1e-12)


def test_square_system_is_a_linear_solve():
    H, T = problem(9, 9, 2, seed=11)
    beta, rss, _ = lstsq.solve(H, T, check_rank=False)
    np.testing.assert_allclose(beta, np.linalg.solve(H, T), atol=1e-10)
    assert rss == 0.0


def test_back_substitution_matches_library_triangular_solve():
    rng = np.random.default_rng(12)
    R = np.triu(rng.standard_normal((15, 15))) + 4.0 * np.eye(15)
    Z = rng.standard_normal((15, 3))
    np.testing.assert_allclose(lstsq.back_substitute(R, Z), np.linalg.solve(R, Z), atol=1e-12)


def test_sign_convention_and_zero_leading_entry():
    # alpha = -sign(x0) ||x||, sign(0) = +1: leading entry 0 gives a negative diagonal
    A = np.array([[0.0, 1.0], [3.0, 2.0], [4.0, 5.0]])
    R = lstsq.householder_reduce(A, 1)
    assert R[0, 0] == -5.0 and R[1, 0] == 0.0 and R[2, 0] == 0.0
    np.testing.assert_allclose(np.linalg.norm(R[:, 1]), np.linalg.norm(A[:, 1]), atol=1e-14)


def test_rank_deficiency_is_reported():
    H, T = problem(50, 6, 1, seed=13)
    H[:, 4] = H[:, 1]
    with pytest.raises(lstsq.RankDeficient):
        lstsq.solve(H, T)
    H[:, 4] = 0.0
    with pytest.raises(lstsq.RankDeficient):
        lstsq.solve(H, T)


def test_rmse_definition_multi_output():
    H, T = problem(80, 5, 3, seed=14)
    beta, rss, _ = lstsq.solve(H, T)
    assert abs(lstsq.rmse_from_rss(rss, 80, 3) - np.sqrt(np.mean((H @ beta - T) ** 2))) < 1e-13


def test_normal_equation_residual_on_non_solutions_with_loops():
    """The measure itself, away from zero: ||H^T r||_F / (||H||_F ||r||_F) with r = H beta - T written out
    entry by entry.  A version that dropped a factor, a norm or the transpose would pass where the
    residual vanishes and fail here."""
    rng = np.random.default_rng(21)
    N, L, m = 7, 3, 2
    H = rng.standard_normal((N, L))
    T = rng.standard_normal((N, m))
    for beta in (np.zeros((L, m)), rng.standard_normal((L, m)), 10.0 * np.ones((L, m))):
        r = [[sum(H[i, j] * beta[j, c] for j in range(L)) - T[i, c] for c in range(m)] for i in range(N)]
        g2 = sum(sum(H[i, j] * r[i][c] for i in range(N)) ** 2 for j in range(L) for c in range(m))
        h2 = sum(H[i, j] ** 2 for i in range(N) for j in range(L))
        r2 = sum(r[i][c] ** 2 for i in range(N) for c in range(m))
        want = (g2 ** 0.5) / ((h2 ** 0.5) * (r2 ** 0.5))
        got = lstsq.normal_equation_residual(H, T, beta)
        assert want > 1e-2                                  # far from a solution
        assert abs(got - want) <= 1e-14 * want
    # a hand case: H = e_1 (one column), T = (1, 1), beta = 0  ->  r = -T, H^T r = -1, ||H|| = 1, ||r|| = sqrt 2
    assert abs(lstsq.normal_equation_residual(np.array([[1.0], [0.0]]), np.array([1.0, 1.0]), np.zeros((1, 1)))
               - 1.0 / np.sqrt(2.0)) < 1e-15
    # scale invariance in H and in (beta, T) jointly
    beta = rng.standard_normal((L, m))
    base = lstsq.normal_equation_residual(H, T, beta)
    assert abs(lstsq.normal_equation_residual(3.0 * H, 3.0 * T, beta) - base) < 1e-14
    # a 1-d target is a single column
    assert abs(lstsq.normal_equation_residual(H, T[:, 0], beta[:, :1])
               - lstsq.normal_equation_residual(H, T[:, :1], beta[:, :1])) == 0.0


def test_rank_check_threshold_is_float32_epsilon_times_the_largest_diagonal():
    """min|R_jj| <= 2^-23 max|R_jj| is rank deficient, anything above is not; signs do not matter and the
    off-diagonal part is not looked at."""
    eps32 = 2.0 ** -23
    for dmax in (1.0, 37.5, 1e-6):
        for sign in (1.0, -1.0):
            R = np.triu(np.full((4, 4), 9.0))
            np.fill_diagonal(R, [dmax, -0.5 * dmax, sign * eps32 * dmax * (1.0 + 1e-9), 0.25 * dmax])
            lstsq.rank_check(R)                                         # just above: accepted
            R[2, 2] = sign * eps32 * dmax                               # at the threshold: rejected
            with pytest.raises(lstsq.RankDeficient):
                lstsq.rank_check(R)
            R[2, 2] = sign * eps32 * dmax * (1.0 - 1e-9)                # just below
            with pytest.raises(lstsq.RankDeficient):
                lstsq.rank_check(R)
    # through solve(): two columns that differ by a relative 2^-20 pass, by 2^-26 of the scale fail
    rng = np.random.default_rng(22)
    H = rng.standard_normal((40, 3))
    T = rng.standard_normal((40, 1))
    e = rng.standard_normal(40)
    e -= H[:, 0] * (H[:, 0] @ e) / (H[:, 0] @ H[:, 0])                  # orthogonal to column 0
    e *= np.linalg.norm(H[:, 0]) / np.linalg.norm(e)
    H[:, 2] = H[:, 0] + 2.0 ** -14 * e
    lstsq.solve(H, T)
    H[:, 2] = H[:, 0] + 2.0 ** -26 * e
    with pytest.raises(lstsq.RankDeficient):
        lstsq.solve(H, T)
