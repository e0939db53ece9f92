"""ctypes binding for libelmrnn.so: argument marshalling only (see include/elm_rnn.h)."""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import numpy as np

CELLS = {"elman": 0, "lstm": 1, "gru": 2, "elman_diag": 3, "fc_multilag": 4}
GATES = {"elman": 1, "lstm": 4, "gru": 3, "elman_diag": 1, "fc_multilag": 1}

ELM_OK, ELM_EINVAL, ELM_EWORKSPACE, ELM_ERANK, ELM_EHIP, ELM_EUNSUPPORTED = 0, -1, -2, -3, -4, -5

DECLARED_SYMBOLS = (
    "elm_rnn_model_create", "elm_rnn_model_create_from_weights", "elm_rnn_get_weights",
    "elm_rnn_model_set_contraction", "elm_rnn_set_beta", "elm_rnn_free", "elm_rnn_hidden_workspace_bytes",
    "elm_rnn_hidden", "elm_rnn_solve_workspace_bytes",
    "elm_rnn_solve", "elm_rnn_solve_static_scratch_bytes", "elm_rnn_solve_static",
    "elm_rnn_fit_workspace_bytes", "elm_rnn_fit",
    "elm_rnn_fit_streamed_workspace_bytes", "elm_rnn_fit_streamed",
    "elm_rnn_predict_workspace_bytes", "elm_rnn_predict", "elm_rnn_strerror",
    "elm_rnn_last_hip_error", "elm_rnn_probe_workspace_bytes", "elm_rnn_probe_ceilings",
)


class ElmRnnError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libelmrnn error {code}: {msg}")
        self.code = code


class _Init(C.Structure):
    _fields_ = [("w_scale", C.c_double), ("spectral_radius", C.c_double),
                ("forget_bias", C.c_double), ("zero_bias", C.c_int), ("contraction", C.c_int)]


class _Stats(C.Structure):
    _fields_ = [("t_hidden_ms", C.c_double), ("t_solve_ms", C.c_double), ("rmse", C.c_double),
                ("rmse_qr", C.c_double), ("ne_resid", C.c_double), ("r_diag_min", C.c_double),
                ("r_diag_max", C.c_double), ("refine_iters", C.c_int)]


@dataclass
class Stats:
    t_hidden_ms: float
    t_solve_ms: float
    rmse: float
    rmse_qr: float
    ne_resid: float
    r_diag_min: float
    r_diag_max: float
    refine_iters: int
    rank_deficient: bool = False


def lib_path() -> str:
    """In-tree library; ELMRNN_LIBRARY may name another build of the same sources (experiments)."""
    override = os.environ.get("ELMRNN_LIBRARY")
    if override:
        return override
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "libelmrnn.so")


_lib = None


def load_library():
    """Load libelmrnn.so (built in-tree by paper_1911_13252_amd.build); no fallback exists."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        raise ElmRnnError(ELM_EINVAL, f"{path} is missing: build it with "
                                      "`python -m paper_1911_13252_amd.build`")
    # PyTorch ships its own HIP runtime; loading it first makes the library bind to that copy, so that the
    # process holds one runtime (and one view of the device) whichever of the two is used first
    import torch  # noqa: F401
    lib = C.CDLL(path)
    vp, i64, u64, sz, dp, fp = C.c_void_p, C.c_int64, C.c_uint64, C.c_size_t, C.POINTER(C.c_double), C.POINTER(C.c_float)
    lib.elm_rnn_model_create.argtypes = [C.c_int] * 5 + [u64, C.POINTER(_Init), C.POINTER(vp)]
    lib.elm_rnn_model_create_from_weights.argtypes = [C.c_int] * 5 + [vp, vp, vp, C.POINTER(vp)]
    lib.elm_rnn_get_weights.argtypes = [vp, vp, vp, vp, vp]
    lib.elm_rnn_set_beta.argtypes = [vp, vp]
    lib.elm_rnn_model_set_contraction.argtypes = [vp, C.c_int]
    lib.elm_rnn_free.argtypes = [vp]
    lib.elm_rnn_free.restype = None
    lib.elm_rnn_hidden_workspace_bytes.argtypes = [C.c_int, i64, C.c_int, C.c_int, C.c_int]
    lib.elm_rnn_hidden_workspace_bytes.restype = sz
    lib.elm_rnn_hidden.argtypes = [vp, vp, i64, i64, i64, C.c_int, vp, vp, vp, vp, vp, sz, vp]
    lib.elm_rnn_solve_workspace_bytes.argtypes = [i64, C.c_int, C.c_int]
    lib.elm_rnn_solve_workspace_bytes.restype = sz
    lib.elm_rnn_solve.argtypes = [vp, vp, i64, C.c_int, C.c_int, C.c_int, vp, vp, C.POINTER(_Stats), vp, sz, vp]
    lib.elm_rnn_solve_static_scratch_bytes.argtypes = []
    lib.elm_rnn_solve_static_scratch_bytes.restype = sz
    lib.elm_rnn_solve_static.argtypes = [vp, vp, i64, C.c_int, C.c_int, C.c_int, vp, vp, C.POINTER(_Stats), vp]
    lib.elm_rnn_fit_workspace_bytes.argtypes = [C.c_int, i64, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int]
    lib.elm_rnn_fit_workspace_bytes.restype = sz
    lib.elm_rnn_fit.argtypes = [C.c_int, vp, i64, i64, vp, i64, C.c_int, C.c_int, C.c_int, C.c_int, u64,
                                C.POINTER(_Init), C.c_int, vp, sz, vp, vp, vp, vp, C.POINTER(_Stats), C.POINTER(vp)]
    lib.elm_rnn_fit_streamed_workspace_bytes.argtypes = [C.c_int, i64, C.c_int, C.c_int, C.c_int, C.c_int, i64]
    lib.elm_rnn_fit_streamed_workspace_bytes.restype = sz
    lib.elm_rnn_fit_streamed.argtypes = [C.c_int, vp, i64, i64, vp, i64, C.c_int, C.c_int, C.c_int, C.c_int, u64,
                                         C.POINTER(_Init), i64, C.c_int, vp, sz, vp, vp, vp, C.POINTER(_Stats),
                                         C.POINTER(vp)]
    lib.elm_rnn_predict_workspace_bytes.argtypes = [vp, i64]
    lib.elm_rnn_predict_workspace_bytes.restype = sz
    lib.elm_rnn_predict.argtypes = [vp, vp, i64, i64, i64, vp, vp, sz, vp]
    lib.elm_rnn_probe_workspace_bytes.argtypes = []
    lib.elm_rnn_probe_workspace_bytes.restype = sz
    lib.elm_rnn_probe_ceilings.argtypes = [C.POINTER(C.c_double)] * 5 + [vp, sz, vp]
    lib.elm_rnn_strerror.argtypes = [C.c_int]
    lib.elm_rnn_strerror.restype = C.c_char_p
    lib.elm_rnn_last_hip_error.restype = C.c_char_p
    _lib = lib
    return lib


def _check(rc: int, allow_rank: bool = False) -> None:
    if rc == ELM_OK or (allow_rank and rc == ELM_ERANK):
        return
    lib = load_library()
    msg = lib.elm_rnn_strerror(rc).decode()
    if rc == ELM_EHIP:
        msg += ": " + lib.elm_rnn_last_hip_error().decode()
    raise ElmRnnError(rc, msg)


def _stream_ptr(stream) -> int:
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return int(s.cuda_stream)


def _dev_f32(t, name: str):
    import torch
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == torch.float32):
        raise TypeError(f"{name} must be a float32 CUDA tensor")
    return t


def _x_strides(X):
    """(ldx_n, ldx_q) in elements for a [N, Q, d] tensor whose last axis is contiguous."""
    if X.dim() != 3 or (X.shape[2] > 1 and X.stride(2) != 1):
        raise ValueError("X must be [N, Q, d] with a contiguous channel axis")
    return int(X.stride(0)), int(X.stride(1))


CONTRACTIONS = {"fp32": 0, "split16": 1}


def _init_struct(w_scale, spectral_radius, forget_bias, zero_bias, contraction="fp32") -> _Init:
    return _Init(float(w_scale), float(spectral_radius), float(forget_bias), int(bool(zero_bias)),
                 CONTRACTIONS[contraction])


def _stats(s: _Stats, rank_deficient: bool) -> Stats:
    return Stats(s.t_hidden_ms, s.t_solve_ms, s.rmse, s.rmse_qr, s.ne_resid, s.r_diag_min,
                 s.r_diag_max, s.refine_iters, rank_deficient)


class Model:
    """Owner of an elm_rnn_model handle (frozen weights + beta)."""

    def __init__(self, handle: int, cell: str, Q: int, d: int, L: int, m: int):
        self._h = C.c_void_p(handle)
        self.cell, self.Q, self.d, self.L, self.m = cell, Q, d, L, m

    @classmethod
    def create(cls, cell: str, Q: int, d: int, L: int, m: int, seed: int, *, w_scale=1.0,
               spectral_radius=0.0, forget_bias=0.0, zero_bias=False, contraction="fp32") -> "Model":
        """elm_rnn_model_create: weights drawn from the seed on the host, uploaded."""
        lib = load_library()
        out = C.c_void_p()
        init = _init_struct(w_scale, spectral_radius, forget_bias, zero_bias, contraction)
        _check(lib.elm_rnn_model_create(CELLS[cell], Q, d, L, m, C.c_uint64(seed), C.byref(init), C.byref(out)))
        return cls(out.value, cell, Q, d, L, m)

    @classmethod
    def from_weights(cls, cell: str, Q: int, m: int, W, U, b) -> "Model":
        """elm_rnn_model_create_from_weights with host float32 arrays W [d,kL], U [L,kL], b [kL]
        (for "elman_diag" U is the lag-weight matrix alpha [L, Q], for "fc_multilag" the stack of lag
        matrices A [Q, L, L])."""
        lib = load_library()
        W = np.ascontiguousarray(W, dtype=np.float32)
        U = np.ascontiguousarray(U, dtype=np.float32)
        b = np.ascontiguousarray(b, dtype=np.float32)
        k = GATES[cell]
        d, L = W.shape[0], W.shape[1] // k
        ushape = (L, Q) if cell == "elman_diag" else (Q, L, L) if cell == "fc_multilag" else (L, k * L)
        if U.shape != ushape or W.shape != (d, k * L) or b.shape != (k * L,):
            raise ValueError("weight shapes do not match the cell")
        out = C.c_void_p()
        _check(lib.elm_rnn_model_create_from_weights(CELLS[cell], Q, d, L, m, W.ctypes.data, U.ctypes.data,
                                                     b.ctypes.data, C.byref(out)))
        return cls(out.value, cell, Q, d, L, m)

    def weights(self):
        """elm_rnn_get_weights -> (W, U, b, beta64) as numpy arrays."""
        lib = load_library()
        k = GATES[self.cell]
        W = np.empty((self.d, k * self.L), np.float32)
        ushape = ((self.L, self.Q) if self.cell == "elman_diag" else
                  (self.Q, self.L, self.L) if self.cell == "fc_multilag" else (self.L, k * self.L))
        U = np.empty(ushape, np.float32)
        b = np.empty(k * self.L, np.float32)
        beta = np.empty((self.L, self.m), np.float64)
        _check(lib.elm_rnn_get_weights(self._h, W.ctypes.data, U.ctypes.data, b.ctypes.data, beta.ctypes.data))
        return W, U, b, beta

    def set_contraction(self, contraction: str) -> None:
        """elm_rnn_model_set_contraction: "fp32" or "split16"."""
        _check(load_library().elm_rnn_model_set_contraction(self._h, CONTRACTIONS[contraction]))

    def set_beta(self, beta64) -> None:
        lib = load_library()
        beta = np.ascontiguousarray(beta64, dtype=np.float64).reshape(self.L, self.m)
        _check(lib.elm_rnn_set_beta(self._h, beta.ctypes.data))

    def close(self) -> None:
        if self._h is not None and self._h.value:
            load_library().elm_rnn_free(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def hidden_workspace_bytes(cell: str, N: int, Q: int, d: int, L: int) -> int:
    return int(load_library().elm_rnn_hidden_workspace_bytes(CELLS[cell], N, Q, d, L))


def hidden(model: Model, X, Q_run: Optional[int] = None, h0=None, c0=None, out=None, c_out=None,
           workspace=None, stream=None):
    """elm_rnn_hidden: H(Q_run) [N, L] for device windows X [N, Q, d]."""
    import torch
    lib = load_library()
    _dev_f32(X, "X")
    N, Q, d = X.shape
    if d != model.d:
        raise ValueError("X channel count does not match the model")
    q = Q if Q_run is None else int(Q_run)
    if not 1 <= q <= Q:
        raise ValueError("Q_run must lie in [1, Q]")
    ldn, ldq = _x_strides(X)
    H = torch.empty((N, model.L), dtype=torch.float32, device=X.device) if out is None else _dev_f32(out, "out")
    for name, t in (("h0", h0), ("c0", c0), ("c_out", c_out)):
        if t is not None:
            _dev_f32(t, name)
            if tuple(t.shape) != (N, model.L) or not t.is_contiguous():
                raise ValueError(f"{name} must be a contiguous [N, L] tensor")
    if tuple(H.shape) != (N, model.L) or not H.is_contiguous():
        raise ValueError("out must be a contiguous [N, L] tensor")
    if workspace is None:
        need = hidden_workspace_bytes(model.cell, N, model.Q, model.d, model.L)
        workspace = torch.empty(need, dtype=torch.uint8, device=X.device) if need else None
    _check(lib.elm_rnn_hidden(model._h, X.data_ptr(), ldn, ldq, N, q,
                              None if h0 is None else h0.data_ptr(),
                              None if c0 is None else c0.data_ptr(), H.data_ptr(),
                              None if c_out is None else c_out.data_ptr(),
                              None if workspace is None else workspace.data_ptr(),
                              0 if workspace is None else workspace.numel(), _stream_ptr(stream)))
    return H


def solve_workspace_bytes(N: int, L: int, m: int) -> int:
    return int(load_library().elm_rnn_solve_workspace_bytes(N, L, m))


def fit_workspace_bytes(N: int, L: int, m: int, h_in_workspace: bool, cell: str = "elman", Q: int = 1,
                        d: int = 1) -> int:
    """elm_rnn_fit_workspace_bytes; only the launch-per-step multi-lag cell depends on (cell, Q, d)."""
    return int(load_library().elm_rnn_fit_workspace_bytes(CELLS[cell], N, Q, d, L, m, int(h_in_workspace)))


def _release_on_error(rc: int, handle, allow_rank: bool) -> None:
    """A fit hands back a live model on ELM_ERANK too: free it when that code is about to be raised."""
    if rc != ELM_OK and not (allow_rank and rc == ELM_ERANK) and handle.value:
        load_library().elm_rnn_free(handle)
        handle.value = None


def solve(H, T, refine: int = 2, workspace=None, stream=None, allow_rank_deficient: bool = False):
    """elm_rnn_solve: returns (beta32 [L,m] device, beta64 [L,m] device, Stats)."""
    import torch
    lib = load_library()
    _dev_f32(H, "H")
    _dev_f32(T, "T")
    if T.dim() == 1:
        T = T[:, None]
    if not (H.is_contiguous() and T.is_contiguous()):
        raise ValueError("H and T must be contiguous")
    N, L = H.shape
    m = T.shape[1]
    need = solve_workspace_bytes(N, L, m)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=H.device)
    beta32 = torch.empty((L, m), dtype=torch.float32, device=H.device)
    beta64 = torch.empty((L, m), dtype=torch.float64, device=H.device)
    st = _Stats()
    rc = lib.elm_rnn_solve(H.data_ptr(), T.data_ptr(), N, L, m, refine, beta32.data_ptr(), beta64.data_ptr(),
                           C.byref(st), workspace.data_ptr(), workspace.numel(), _stream_ptr(stream))
    _check(rc, allow_rank=allow_rank_deficient)
    return beta32, beta64, _stats(st, rc == ELM_ERANK)


def solve_static(H, T, refine: int = 2, stream=None, allow_rank_deficient: bool = False):
    """elm_rnn_solve_static: elm_rnn_solve on the library's static device scratch array (the call itself
    allocates nothing; the result tensors are made here before it)."""
    import torch
    lib = load_library()
    _dev_f32(H, "H")
    _dev_f32(T, "T")
    if T.dim() == 1:
        T = T[:, None]
    if not (H.is_contiguous() and T.is_contiguous()):
        raise ValueError("H and T must be contiguous")
    N, L = H.shape
    m = T.shape[1]
    beta32 = torch.empty((L, m), dtype=torch.float32, device=H.device)
    beta64 = torch.empty((L, m), dtype=torch.float64, device=H.device)
    st = _Stats()
    rc = lib.elm_rnn_solve_static(H.data_ptr(), T.data_ptr(), N, L, m, refine, beta32.data_ptr(), beta64.data_ptr(),
                                  C.byref(st), _stream_ptr(stream))
    _check(rc, allow_rank=allow_rank_deficient)
    return beta32, beta64, _stats(st, rc == ELM_ERANK)


@dataclass
class FitResult:
    model: Model
    beta: "object"       # device float32 [L, m]
    beta64: "object"     # device float64 [L, m]
    H: "object"          # device float32 [N, L] (None when H was kept in the workspace)
    stats: Stats


def fit(cell: str, X, T, L: int, seed: int, *, w_scale=1.0, spectral_radius=0.0, forget_bias=0.0,
        zero_bias=False, contraction="fp32", refine: int = -1, keep_H: bool = True, workspace=None, H_out=None,
        stream=None, allow_rank_deficient: bool = False) -> FitResult:
    """elm_rnn_fit: Algorithm "S-R-ELM" end to end on device tensors X [N,Q,d], T [N,m]."""
    import torch
    lib = load_library()
    _dev_f32(X, "X")
    _dev_f32(T, "T")
    if T.dim() == 1:
        T = T[:, None]
    if not T.is_contiguous():
        raise ValueError("T must be contiguous")
    N, Q, d = X.shape
    m = T.shape[1]
    ldn, ldq = _x_strides(X)
    H = H_out
    if H is not None:
        _dev_f32(H, "H_out")
        if tuple(H.shape) != (N, L) or not H.is_contiguous():
            raise ValueError("H_out must be a contiguous [N, L] tensor")
    if H is None and keep_H:
        H = torch.empty((N, L), dtype=torch.float32, device=X.device)
    need = fit_workspace_bytes(N, L, m, H is None, cell, Q, d)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=X.device)
    beta32 = torch.empty((L, m), dtype=torch.float32, device=X.device)
    beta64 = torch.empty((L, m), dtype=torch.float64, device=X.device)
    st = _Stats()
    out = C.c_void_p()
    init = _init_struct(w_scale, spectral_radius, forget_bias, zero_bias, contraction)
    rc = lib.elm_rnn_fit(CELLS[cell], X.data_ptr(), ldn, ldq, T.data_ptr(), N, Q, d, L, m, C.c_uint64(seed),
                         C.byref(init), refine, workspace.data_ptr(), workspace.numel(), _stream_ptr(stream),
                         None if H is None else H.data_ptr(), beta32.data_ptr(), beta64.data_ptr(),
                         C.byref(st), C.byref(out))
    _release_on_error(rc, out, allow_rank_deficient)
    _check(rc, allow_rank=allow_rank_deficient)
    return FitResult(Model(out.value, cell, Q, d, L, m), beta32, beta64, H, _stats(st, rc == ELM_ERANK))


def fit_streamed_workspace_bytes(N: int, L: int, m: int, chunk_rows: int = 0, cell: str = "elman", Q: int = 1,
                                 d: int = 1) -> int:
    """elm_rnn_fit_streamed_workspace_bytes; only the launch-per-step multi-lag cell depends on (cell, Q, d)."""
    return int(load_library().elm_rnn_fit_streamed_workspace_bytes(CELLS[cell], N, Q, d, L, m, chunk_rows))


def fit_streamed(cell: str, X, T, L: int, seed: int, *, w_scale=1.0, spectral_radius=0.0, forget_bias=0.0,
                 zero_bias=False, contraction="fp32", chunk_rows: int = 0, refine: int = -1, workspace=None,
                 stream=None, allow_rank_deficient: bool = False) -> FitResult:
    """elm_rnn_fit_streamed: the fit with H produced and consumed chunk by chunk (FitResult.H is None)."""
    import torch
    lib = load_library()
    _dev_f32(X, "X")
    _dev_f32(T, "T")
    if T.dim() == 1:
        T = T[:, None]
    if not T.is_contiguous():
        raise ValueError("T must be contiguous")
    N, Q, d = X.shape
    m = T.shape[1]
    ldn, ldq = _x_strides(X)
    need = fit_streamed_workspace_bytes(N, L, m, chunk_rows, cell, Q, d)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=X.device)
    beta32 = torch.empty((L, m), dtype=torch.float32, device=X.device)
    beta64 = torch.empty((L, m), dtype=torch.float64, device=X.device)
    st = _Stats()
    out = C.c_void_p()
    init = _init_struct(w_scale, spectral_radius, forget_bias, zero_bias, contraction)
    rc = lib.elm_rnn_fit_streamed(CELLS[cell], X.data_ptr(), ldn, ldq, T.data_ptr(), N, Q, d, L, m,
                                  C.c_uint64(seed), C.byref(init), chunk_rows, refine, workspace.data_ptr(),
                                  workspace.numel(), _stream_ptr(stream), beta32.data_ptr(), beta64.data_ptr(),
                                  C.byref(st), C.byref(out))
    _release_on_error(rc, out, allow_rank_deficient)
    _check(rc, allow_rank=allow_rank_deficient)
    return FitResult(Model(out.value, cell, Q, d, L, m), beta32, beta64, None, _stats(st, rc == ELM_ERANK))


def probe_ceilings(stream=None) -> dict:
    """elm_rnn_probe_ceilings: measured matrix-instruction and streaming-copy rates of the current device."""
    import torch
    lib = load_library()
    ws = torch.empty(int(lib.elm_rnn_probe_workspace_bytes()), dtype=torch.uint8, device="cuda")
    f32, f16, gbs, o32, o16 = (C.c_double() for _ in range(5))
    _check(lib.elm_rnn_probe_ceilings(C.byref(f32), C.byref(f16), C.byref(gbs), C.byref(o32), C.byref(o16),
                                      ws.data_ptr(), ws.numel(), _stream_ptr(stream)))
    return {"mfma_f32_tflops": f32.value, "mfma_f16_tflops": f16.value, "hbm_copy_gbs": gbs.value,
            "valu_overlap_with_mfma_f32": o32.value, "valu_overlap_with_mfma_f16": o16.value}


def predict(model: Model, X, workspace=None, stream=None):
    """elm_rnn_predict: Y [N, m] = H(Q) beta for device windows X."""
    import torch
    lib = load_library()
    _dev_f32(X, "X")
    N, Q, d = X.shape
    if d != model.d or Q < model.Q:
        raise ValueError("X does not match the model")
    ldn, ldq = _x_strides(X)
    if workspace is None:      # one pass when H is small, else chunks of about 128 MiB of H
        need = int(lib.elm_rnn_predict_workspace_bytes(model._h, N))
        if need > (128 << 20):
            rows = max(256, (128 << 20) // (4 * model.L) // 256 * 256)
            if hidden_workspace_bytes(model.cell, N, model.Q, model.d, model.L) > 0:
                rows = 65536                      # whole passes of the launch-per-step multi-lag cell
            need = int(lib.elm_rnn_predict_workspace_bytes(model._h, min(N, rows)))
        workspace = torch.empty(need, dtype=torch.uint8, device=X.device)
    Y = torch.empty((N, model.m), dtype=torch.float32, device=X.device)
    _check(lib.elm_rnn_predict(model._h, X.data_ptr(), ldn, ldq, N, Y.data_ptr(), workspace.data_ptr(),
                               workspace.numel(), _stream_ptr(stream)))
    return Y
