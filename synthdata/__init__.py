"""Seeded synthetic time-series inputs for the ELM-RNN fit path.

This module only produces *inputs* (series, sliding windows, targets and the
table of benchmark configurations).  It contains none of the method's
arithmetic (no cell recurrence, no weight generation, no least squares) and is
the only code shared by the CPU oracle's tests and the GPU path's tests.
"""
from .series import (CONFIGS, EXTRA_CONFIGS, ElmConfig, make_series, make_windows,
                     make_problem, get_config)

__all__ = ["CONFIGS", "EXTRA_CONFIGS", "ElmConfig", "make_series", "make_windows",
           "make_problem", "get_config"]
