"""CPU float64 oracle for the ELM-RNN fit path (test infrastructure only).

A plain, slow, obviously-correct numpy implementation of what the GPU library
computes: frozen random weights from a seed, the Elman / LSTM / GRU hidden
matrix H(Q), and beta = H^+ T by explicit Householder least squares.

This package is TEST INFRASTRUCTURE.  Only tests, the smoke check and the
benchmark's cpu_baseline leg may import it; the product path never does and it
imports nothing from the product path.  It shares no code with the HIP kernels.

Parity status: every function is pinned by the CPU tests (closed forms,
library special cases, brute force, invariants); none is "parity unpinned".
"""
from . import cells, lstsq, weights, fit  # noqa: F401
