"""Oracle: the frozen random weights W, U, b drawn from one seed.

Test infrastructure only; shares no code with the GPU path (the library has its
own C++ implementation of the same counter-based generator).

Step 1 of Algorithm "S-R-ELM" only says "randomly assign W, alpha, b"; the
distribution and the generator are fixed here:
  * SplitMix64 stream: state += 0x9E3779B97F4A7C15; z = state;
    z = (z ^ z >> 30) * 0xBF58476D1CE4E5B9; z = (z ^ z >> 27) * 0x94D049BB133111EB;
    out = z ^ z >> 31; u = (out >> 11) * 2^-53 in [0, 1);
  * value = (2u - 1) * a in float64 (uniform on [-a, a));
  * draw order: W row-major [d, kL], then U row-major [L, kL], then b [kL];
  * spectral_radius > 0 (Elman): U *= spectral_radius / max|eig(U)|, in float64;
  * forget_bias is added to the LSTM forget block of b (block 1 of i, f, o, g);
  * zero_bias: b = 0 exactly (the draws are still consumed);
  * finally everything is rounded to float32.
"""
from __future__ import annotations

import numpy as np

GATES = {"elman": 1, "lstm": 4, "gru": 3, "elman_diag": 1, "fc_multilag": 1}

_GAMMA = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def splitmix64(seed: int, n: int) -> np.ndarray:
    """First n outputs of the SplitMix64 stream started at `seed` (uint64)."""
    with np.errstate(over="ignore"):
        idx = np.arange(1, n + 1, dtype=np.uint64)
        z = np.uint64(seed & 0xFFFFFFFFFFFFFFFF) + idx * _GAMMA
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        return z ^ (z >> np.uint64(31))


def uniform01(seed: int, n: int) -> np.ndarray:
    """n uniforms in [0, 1) with 53 random bits each (float64)."""
    return (splitmix64(seed, n) >> np.uint64(11)).astype(np.float64) * 2.0 ** -53


def spectral_radius(U: np.ndarray) -> float:
    return float(np.max(np.abs(np.linalg.eigvals(np.asarray(U, dtype=np.float64)))))


def draw(cell: str, d: int, L: int, seed: int, w_scale: float = 1.0,
         spectral_radius_target: float = 0.0, forget_bias: float = 0.0,
         zero_bias: bool = False, Q: int = 0):
    """Return (W [d,kL], U [L,kL], b [kL]) as float32 arrays.

    For the paper's own Elman cell ("elman_diag") the recurrent weights are alpha [L, Q] (lag k in
    column k-1), for its fully connected cell ("fc_multilag") A [Q, L, L] (lag k in block k-1), both
    drawn in the same place of the stream as U.
    """
    k = GATES[cell]
    kL = k * L
    ushape = (L, Q) if cell == "elman_diag" else (Q, L, L) if cell == "fc_multilag" else (L, kL)
    if cell in ("elman_diag", "fc_multilag") and Q < 1:
        raise ValueError("the multi-lag cells need Q")
    nu = int(np.prod(ushape))
    n = d * kL + nu + kL
    v = (2.0 * uniform01(seed, n) - 1.0) * float(w_scale)
    W = v[:d * kL].reshape(d, kL)
    U = v[d * kL:d * kL + nu].reshape(ushape)
    b = v[d * kL + nu:].copy()
    if spectral_radius_target > 0.0:
        if cell != "elman":
            raise ValueError("spectral-radius scaling is defined for the Elman cell only")
        U = U * (spectral_radius_target / spectral_radius(U))
    if zero_bias:
        b[:] = 0.0
    elif cell == "lstm" and forget_bias != 0.0:
        b[L:2 * L] += forget_bias
    return W.astype(np.float32), U.astype(np.float32), b.astype(np.float32)
