"""MI355X-native ELM-RNN fit path: thin ctypes binding over libelmrnn.so.

Every step of the path (hidden-matrix build, TSQR, back-solve, refinement,
prediction) runs in the HIP kernels of the shared library; this module only
marshals arguments.  PyTorch tensors are used for device memory and streams.
Importing the package never touches the GPU; the library is loaded on first
use and a missing library is a hard error (there is no CPU fallback).
"""
from .binding import (CELLS, ElmRnnError, FitResult, Model, Stats, fit, hidden, lib_path,
                      load_library, predict, solve, solve_static, solve_workspace_bytes, hidden_workspace_bytes,
                      fit_workspace_bytes, fit_streamed, fit_streamed_workspace_bytes, probe_ceilings, DECLARED_SYMBOLS)

__all__ = ["CELLS", "ElmRnnError", "FitResult", "Model", "Stats", "fit", "hidden", "lib_path",
           "load_library", "predict", "solve", "solve_static", "solve_workspace_bytes", "hidden_workspace_bytes", "fit_workspace_bytes",
           "fit_streamed", "fit_streamed_workspace_bytes", "probe_ceilings", "DECLARED_SYMBOLS"]

# the C entry points' own names, for callers that think in terms of include/elm_rnn.h
elm_rnn_fit = fit
elm_rnn_fit_streamed = fit_streamed
elm_rnn_hidden = hidden
elm_rnn_solve = solve
elm_rnn_solve_static = solve_static
elm_rnn_predict = predict
elm_rnn_model_create = Model.create
elm_rnn_model_create_from_weights = Model.from_weights
