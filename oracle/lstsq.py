"""Oracle: beta = H^+ T by explicit Householder QR of the augmented matrix [H | T].

Test infrastructure only; shares no code with the GPU path.

The paper's section "Computing beta" factors H = QR, forms z = Q^T Y and solves
R beta = z by back substitution.  Applying the same reflectors to [H | T] gives
R (top-left L x L), z (top-right L x m) and, below them, a block whose squared
Frobenius norm is the residual sum of squares.  For full-column-rank H this is
the same beta as the pseudo-inverse formula of the section "Extreme Learning
Machine", (H^T H)^{-1} H^T T (the paper prints it without the last transpose).
All arithmetic is float64.
"""
from __future__ import annotations

import numpy as np


class RankDeficient(ValueError):
    pass


def householder_reduce(A: np.ndarray, ncols: int) -> np.ndarray:
    """Apply Householder reflectors that zero columns 0..ncols-1 below the diagonal.

    Works on a float64 copy of A (rows >= ncols) and returns it.  Column k:
    x = A[k:, k]; alpha = -sign(x_0) * ||x|| (sign(0) = +1); v = x - alpha e_1;
    A[k:, k:] -= (2 / v^T v) v (v^T A[k:, k:]).
    """
    A = np.array(A, dtype=np.float64)
    rows, cols = A.shape
    if rows < ncols:
        raise ValueError("need at least as many rows as reduced columns")
    for k in range(ncols):
        x = A[k:, k]
        s = np.sqrt(np.dot(x, x))
        if s == 0.0:
            raise RankDeficient(f"column {k} vanishes during the reduction")
        alpha = -s if x[0] >= 0.0 else s
        v = x.copy()
        v[0] -= alpha
        tau = 2.0 / np.dot(v, v)
        w = v @ A[k:, k:]
        A[k:, k:] -= tau * np.outer(v, w)
        A[k + 1:, k] = 0.0          # exact zeros below the diagonal
        A[k, k] = alpha
    return A


def back_substitute(R: np.ndarray, Z: np.ndarray) -> np.ndarray:
    """Solve the upper-triangular system R B = Z row by row from the bottom."""
    L = R.shape[0]
    B = np.zeros_like(Z, dtype=np.float64)
    for i in range(L - 1, -1, -1):
        B[i] = (Z[i] - R[i, i + 1:] @ B[i + 1:]) / R[i, i]
    return B


def rank_check(R11: np.ndarray) -> None:
    """Numerical rank test on the diagonal of R (H^T H must be invertible).

    H is treated as rank deficient when min|R_jj| <= eps32 * max|R_jj|: the
    device path factors in float32, so a diagonal ratio at float32 rounding
    level cannot be told from zero there.
    """
    dg = np.abs(np.diag(R11))
    if dg.min() <= np.finfo(np.float32).eps * dg.max():
        raise RankDeficient("H is numerically rank deficient")


def solve(H: np.ndarray, T: np.ndarray, check_rank: bool = True):
    """Least squares min ||H beta - T||_F.

    Returns (beta [L, m], rss, R [L, L+m] = [R11 | R12]).  rss is the squared
    Frobenius norm of what remains of the T columns below row L.
    """
    H = np.asarray(H, dtype=np.float64)
    T = np.asarray(T, dtype=np.float64)
    if T.ndim == 1:
        T = T[:, None]
    N, L = H.shape
    if N < L:
        raise ValueError("N must be at least L")
    A = householder_reduce(np.hstack([H, T]), L)
    R11 = np.triu(A[:L, :L])
    R12 = A[:L, L:]
    if check_rank:
        rank_check(R11)
    beta = back_substitute(R11, R12)
    rss = float(np.sum(A[L:, L:] ** 2))
    return beta, rss, A[:L, :].copy()


def solve_chunked(H: np.ndarray, T: np.ndarray, chunk: int = 4096, check_rank: bool = True):
    """Same result as solve(), processing rows in chunks: reduce([R_prev; chunk]).

    Only the first L columns are reduced in every chunk; the rows that fall
    below row L after a reduction carry residual mass only, so their squared
    norm in the T columns is accumulated and they are dropped.
    """
    H = np.asarray(H)
    T = np.asarray(T)
    if T.ndim == 1:
        T = T[:, None]
    N, L = H.shape
    carry = np.zeros((0, L + T.shape[1]), dtype=np.float64)
    rss = 0.0
    for s in range(0, N, chunk):
        e = min(N, s + chunk)
        blk = np.hstack([H[s:e].astype(np.float64), T[s:e].astype(np.float64)])
        stack = np.vstack([carry, blk])
        if stack.shape[0] < L:
            carry = stack
            continue
        A = householder_reduce(stack, L)
        rss += float(np.sum(A[L:, L:] ** 2))
        carry = A[:L, :]
    if carry.shape[0] < L:
        raise ValueError("N must be at least L")
    R11 = np.triu(carry[:, :L])
    if check_rank:
        rank_check(R11)
    beta = back_substitute(R11, carry[:, L:])
    return beta, rss, carry.copy()


def rmse_from_rss(rss: float, N: int, m: int) -> float:
    """Root of the mean over all N*m squared errors."""
    return float(np.sqrt(rss / (N * m)))


def normal_equation_residual(H, T, beta) -> float:
    """||H^T (H beta - T)||_F / (||H||_F ||H beta - T||_F) in float64."""
    H = np.asarray(H, dtype=np.float64)
    T = np.asarray(T, dtype=np.float64)
    if T.ndim == 1:
        T = T[:, None]
    r = H @ np.asarray(beta, dtype=np.float64) - T
    nr = np.linalg.norm(r)
    if nr == 0.0:
        return 0.0
    return float(np.linalg.norm(H.T @ r) / (np.linalg.norm(H) * nr))
