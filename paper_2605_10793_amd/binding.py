"""Thin ctypes binding over libconqur.so (the C ABI declared in include/conqur.h).

Argument marshalling only: every step of the path runs in the library's HIP
kernels.  PyTorch supplies device memory (tensors) and the stream handle.  There
is no fallback: if the shared library is missing or the device call fails, the
binding raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Tuple

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libconqur.so")

OK, EINVAL, ESTATE, ENOMEM, EHIP, ENOCONV, ENONFINITE = range(7)
STATUS_NAMES = ["OK", "EINVAL", "ESTATE", "ENOMEM", "EHIP", "ENOCONV", "ENONFINITE"]
F32, BF16 = 0, 1

EXPORTS = [
    "conqur_init", "conqur_step_batch", "conqur_step_batch_heads", "conqur_step_batch_quant", "conqur_get_batch_stats", "conqur_update_rotation",
    "conqur_quant_error", "conqur_quant_error_zp", "conqur_rotate", "conqur_rotate_quant", "conqur_row_diagnostics", "conqur_get_state", "conqur_set_state", "conqur_get_last_corners",
    "conqur_score_rows_static", "conqur_set_taps", "conqur_set_timing", "conqur_get_timing", "conqur_get_clock_probe", "conqur_last_error", "conqur_destroy", "conqur_version",
]


class Config(ctypes.Structure):
    _fields_ = [("d", ctypes.c_uint32), ("heads", ctypes.c_uint32), ("act_dtype", ctypes.c_uint32),
                ("max_tokens", ctypes.c_uint32), ("prox_lambda", ctypes.c_float), ("polar_tol", ctypes.c_float),
                ("polar_max_iters", ctypes.c_uint32), ("polar_precision", ctypes.c_uint32),
                ("polar_verify", ctypes.c_uint32), ("device", ctypes.c_int32), ("stream", ctypes.c_void_p)]


class BatchStats(ctypes.Structure):
    _fields_ = [("rows", ctypes.c_uint64), ("skipped", ctypes.c_uint64), ("l1", ctypes.c_double),
                ("objective", ctypes.c_double)]


class UpdateStats(ctypes.Structure):
    _fields_ = [("iters", ctypes.c_uint32), ("accurate", ctypes.c_uint32), ("orth_err", ctypes.c_double),
                ("inner", ctypes.c_double), ("m_fro", ctypes.c_double), ("ms", ctypes.c_double),
                ("orth_measured", ctypes.c_uint32), ("reserved", ctypes.c_uint32), ("l1", ctypes.c_double),
                ("mfma_flop", ctypes.c_double)]


class ConqurError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"{STATUS_NAMES[status] if 0 <= status < 7 else status}: {msg}")
        self.status = status


_lib = None


def load() -> ctypes.CDLL:
    """Load libconqur.so; raises if it has not been built (run build.py / __graft_entry__.build())."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} not built: run `python -m paper_2605_10793_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        vp, u64, u32, i32 = ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint32, ctypes.c_int
        L.conqur_init.restype = i32
        L.conqur_init.argtypes = [ctypes.POINTER(Config), vp, ctypes.POINTER(vp)]
        L.conqur_step_batch.restype = i32
        L.conqur_step_batch.argtypes = [vp, vp, u64, u64]
        L.conqur_step_batch_heads.restype = i32
        L.conqur_step_batch_heads.argtypes = [vp, vp, u64, u64, ctypes.c_uint32, ctypes.c_uint32]
        L.conqur_step_batch_quant.restype = i32
        L.conqur_step_batch_quant.argtypes = [vp, vp, u64, u64, ctypes.c_uint32, ctypes.c_uint32, ctypes.c_float, vp, u64]
        L.conqur_get_batch_stats.restype = i32
        L.conqur_get_batch_stats.argtypes = [vp, vp]
        L.conqur_update_rotation.restype = i32
        L.conqur_update_rotation.argtypes = [vp, vp]
        L.conqur_quant_error.restype = i32
        L.conqur_quant_error.argtypes = [vp, vp, u64, u64, u32, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
        L.conqur_quant_error_zp.restype = i32
        L.conqur_quant_error_zp.argtypes = [vp, vp, u64, u64, u32, ctypes.c_float, ctypes.POINTER(ctypes.c_double),
                                            ctypes.POINTER(ctypes.c_double)]
        L.conqur_rotate.restype = i32
        L.conqur_rotate.argtypes = [vp, vp, u64, u64, vp, u64]
        L.conqur_rotate_quant.restype = i32
        L.conqur_rotate_quant.argtypes = [vp, vp, u64, u64, ctypes.c_uint32, ctypes.c_uint32, ctypes.c_float, vp, u64]
        L.conqur_row_diagnostics.restype = i32
        L.conqur_row_diagnostics.argtypes = [vp, vp, u64, u64, vp, vp]
        L.conqur_get_state.restype = i32
        L.conqur_get_state.argtypes = [vp, vp, vp, vp]
        L.conqur_set_state.restype = i32
        L.conqur_set_state.argtypes = [vp, vp, vp]
        L.conqur_get_last_corners.restype = i32
        L.conqur_get_last_corners.argtypes = [vp, vp, vp]
        L.conqur_score_rows_static.restype = i32
        L.conqur_score_rows_static.argtypes = [vp, u32, u64, u64, u64, u32, u32, ctypes.c_float, vp, vp]
        L.conqur_set_taps.restype = i32
        L.conqur_set_taps.argtypes = [vp, i32]
        L.conqur_set_timing.restype = i32
        L.conqur_set_timing.argtypes = [vp, i32]
        L.conqur_get_timing.restype = i32
        L.conqur_get_timing.argtypes = [vp, vp]
        L.conqur_get_clock_probe.restype = i32
        L.conqur_get_clock_probe.argtypes = [vp, vp]
        L.conqur_last_error.restype = ctypes.c_char_p
        L.conqur_last_error.argtypes = [vp]
        L.conqur_destroy.restype = None
        L.conqur_destroy.argtypes = [vp]
        L.conqur_version.restype = ctypes.c_char_p
        _lib = L
    return _lib


def _np_ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


class Calibrator:
    """One context: `heads` rotations of width d/heads, their statistics and workspaces."""

    def __init__(self, d: int, heads: int, dtype: str, R0: np.ndarray, max_tokens: int,
                 prox_lambda: float = 0.0, polar_tol: float = 0.0, polar_max_iters: int = 0, polar_precision: int = 0,
                 polar_verify: int = 0, device: int = 0, stream: Optional[int] = None):
        import torch
        self._lib = load()
        self.d, self.heads, self.dh, self.dtype = d, heads, d // max(heads, 1), dtype
        if stream is None:
            stream = torch.cuda.current_stream(device).cuda_stream
        cfg = Config(d, heads, BF16 if dtype == "bf16" else F32, max_tokens, prox_lambda, polar_tol,
                     polar_max_iters, polar_precision, polar_verify, device, ctypes.c_void_p(stream))
        R0 = np.ascontiguousarray(R0, dtype=np.float32)
        if R0.size != heads * self.dh * self.dh:
            raise ValueError("R0 must hold heads * dh * dh floats")
        h = ctypes.c_void_p()
        st = self._lib.conqur_init(ctypes.byref(cfg), _np_ptr(R0), ctypes.byref(h))
        if st != OK:
            raise ConqurError(st, "conqur_init failed")
        self._h = h

    def _check(self, st: int, allow: Tuple[int, ...] = ()) -> int:
        if st != OK and st not in allow:
            raise ConqurError(st, self._lib.conqur_last_error(self._h).decode())
        return st

    def close(self):
        if getattr(self, "_h", None):
            self._lib.conqur_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _x(self, X) -> Tuple[int, int, int]:
        import torch
        want = torch.bfloat16 if self.dtype == "bf16" else torch.float32
        if X.dim() != 2 or X.stride(1) != 1 or not X.is_cuda or X.dtype != want or X.shape[1] < self.d:
            raise ValueError(f"X must be a 2-D {want} device tensor with >= d columns and unit column stride")
        return X.data_ptr(), X.shape[0], X.stride(0)

    def step_batch(self, X) -> None:
        p, T, stride = self._x(X)
        self._check(self._lib.conqur_step_batch(self._h, p, T, stride))

    def step_batch_heads(self, X, head0: int, nheads: int) -> None:
        """One batch for the heads [head0, head0 + nheads) only; X holds their nheads * dh columns."""
        import torch
        want = torch.bfloat16 if self.dtype == "bf16" else torch.float32
        if X.dim() != 2 or X.stride(1) != 1 or not X.is_cuda or X.dtype != want or X.shape[1] < nheads * self.dh:
            raise ValueError(f"X must be a 2-D {want} device tensor with >= nheads * dh columns and unit column stride")
        self._check(self._lib.conqur_step_batch_heads(self._h, X.data_ptr(), X.shape[0], X.stride(0), head0, nheads))

    def step_batch_quant(self, X, bits: int = 4, zero_point: bool = True, clip_ratio: float = 1.0, Yq=None):
        """step_batch(X) and Yq = Q(X R_op) from one rotation of the batch (quantisation-aware calibration); asynchronous."""
        import torch
        p, T, stride = self._x(X)
        if Yq is None:
            Yq = torch.empty((T, self.d), dtype=X.dtype, device=X.device)
        if Yq.dtype != X.dtype or Yq.dim() != 2 or Yq.shape[0] != T or Yq.shape[1] < self.d or Yq.stride(1) != 1:
            raise ValueError("Yq must be a [T, >= d] tensor of X's dtype with unit column stride")
        self._check(self._lib.conqur_step_batch_quant(self._h, p, T, stride, bits, 1 if zero_point else 0,
                                                      ctypes.c_float(clip_ratio), ctypes.c_void_p(Yq.data_ptr()), Yq.stride(0)))
        return Yq

    def batch_stats(self) -> List[dict]:
        arr = (BatchStats * self.heads)()
        self._check(self._lib.conqur_get_batch_stats(self._h, arr))
        return [dict(rows=int(a.rows), skipped=int(a.skipped), l1=float(a.l1), objective=float(a.objective)) for a in arr]

    def objective(self) -> np.ndarray:
        """Eq. 1 of the rows accumulated since the last update, per head (conqur_batch_stats.objective)."""
        return np.array([a["objective"] for a in self.batch_stats()])

    def update_rotation(self, allow: Tuple[int, ...] = ()) -> Tuple[int, List[dict]]:
        arr = (UpdateStats * self.heads)()
        st = self._check(self._lib.conqur_update_rotation(self._h, arr), allow)
        return st, [dict(iters=int(a.iters), accurate=int(a.accurate), orth_err=float(a.orth_err),
                         inner=float(a.inner), m_fro=float(a.m_fro), ms=float(a.ms),
                         orth_measured=bool(a.orth_measured), l1=float(a.l1), mfma_flop=float(a.mfma_flop)) for a in arr]

    def quant_error(self, X, bits: int = 4) -> Tuple[float, float]:
        p, T, stride = self._x(X)
        sse, en = ctypes.c_double(), ctypes.c_double()
        self._check(self._lib.conqur_quant_error(self._h, p, T, stride, bits, ctypes.byref(sse), ctypes.byref(en)))
        return sse.value, en.value

    def quant_error_zp(self, X, bits: int = 4, clip_ratio: float = 1.0) -> Tuple[float, float]:
        p, T, stride = self._x(X)
        sse, en = ctypes.c_double(), ctypes.c_double()
        self._check(self._lib.conqur_quant_error_zp(self._h, p, T, stride, bits, ctypes.c_float(clip_ratio),
                                                    ctypes.byref(sse), ctypes.byref(en)))
        return sse.value, en.value

    def rotate(self, X, Y=None):
        """Y = X R_op per head into a device tensor of X's dtype (allocated here unless given); asynchronous."""
        import torch
        p, T, stride = self._x(X)
        if Y is None:
            Y = torch.empty((T, self.d), dtype=X.dtype, device=X.device)
        if Y.dtype != X.dtype or Y.dim() != 2 or Y.shape[0] != T or Y.shape[1] < self.d or Y.stride(1) != 1:
            raise ValueError("Y must be a [T, >= d] tensor of X's dtype with unit column stride")
        self._check(self._lib.conqur_rotate(self._h, p, T, stride, ctypes.c_void_p(Y.data_ptr()), Y.stride(0)))
        return Y

    def rotate_quant(self, X, bits: int = 4, zero_point: bool = True, clip_ratio: float = 1.0, Yq=None):
        """Yq = Q(X R_op): per-token fake-quantised rotated rows in X's dtype (allocated here unless given); asynchronous."""
        import torch
        p, T, stride = self._x(X)
        if Yq is None:
            Yq = torch.empty((T, self.d), dtype=X.dtype, device=X.device)
        if Yq.dtype != X.dtype or Yq.dim() != 2 or Yq.shape[0] != T or Yq.shape[1] < self.d or Yq.stride(1) != 1:
            raise ValueError("Yq must be a [T, >= d] tensor of X's dtype with unit column stride")
        self._check(self._lib.conqur_rotate_quant(self._h, p, T, stride, bits, 1 if zero_point else 0, ctypes.c_float(clip_ratio),
                                                  ctypes.c_void_p(Yq.data_ptr()), Yq.stride(0)))
        return Yq

    def row_diagnostics(self, X):
        """Per row of Y = X R_op: (PR/d, ||y||_inf^2/||y||_2^2) as two float32 arrays of length T."""
        p, T, stride = self._x(X)
        pr = np.empty(T, dtype=np.float32); rho = np.empty(T, dtype=np.float32)
        self._check(self._lib.conqur_row_diagnostics(self._h, p, T, stride, _np_ptr(pr), _np_ptr(rho)))
        return pr, rho

    def get_state(self, want_R: bool = True, want_M: bool = True):
        shape = (self.heads, self.dh, self.dh)
        R = np.empty(shape, dtype=np.float32) if want_R else None
        M = np.empty(shape, dtype=np.float32) if want_M else None
        n = np.zeros(self.heads, dtype=np.uint64)
        self._check(self._lib.conqur_get_state(self._h, _np_ptr(R), _np_ptr(M), _np_ptr(n)))
        return R, M, n

    def set_state(self, R: Optional[np.ndarray] = None, M: Optional[np.ndarray] = None) -> None:
        R = None if R is None else np.ascontiguousarray(R, dtype=np.float32)
        M = None if M is None else np.ascontiguousarray(M, dtype=np.float32)
        self._check(self._lib.conqur_set_state(self._h, _np_ptr(R), _np_ptr(M)))

    def last_corners(self, T: int):
        S = np.empty((T, self.d), dtype=np.int8)
        nrm = np.empty((self.heads, T), dtype=np.float32)
        self._check(self._lib.conqur_get_last_corners(self._h, _np_ptr(S), _np_ptr(nrm)))
        return S, nrm

    def set_taps(self, enable: bool) -> None:
        """Keep the corner signs of later steps for last_corners() (only the fused per-head step drops them by default)."""
        self._check(self._lib.conqur_set_taps(self._h, int(enable)))

    def set_timing(self, level) -> None:
        """0 off, 1 (or True) whole-call events, 2 per-stage events and GEMM clock probes as well."""
        self._check(self._lib.conqur_set_timing(self._h, int(level)))

    def timing(self) -> dict:
        out = np.zeros(12, dtype=np.float32)
        self._check(self._lib.conqur_get_timing(self._h, _np_ptr(out)))
        keys = ["prep", "rotate", "accumulate", "stats", "update", "quant_rotate", "quant_error", "step", "quant"]
        return {k: float(out[i]) for i, k in enumerate(keys)}

    def clock_probe(self) -> dict:
        """Sustained shader clock and prologue / main-loop / epilogue split of the last timed step's two GEMMs."""
        out = np.zeros(8, dtype=np.float32)
        self._check(self._lib.conqur_get_clock_probe(self._h, _np_ptr(out)))
        keys = ["clock_mhz", "loop_us", "prologue_us", "epilogue_us"]
        return {g: {k: float(out[4 * j + i]) for i, k in enumerate(keys)} for j, g in enumerate(("rotate", "accumulate"))}


def score_rows_static(Y, out, bits: int = 4, zero_point: bool = False, clip_ratio: float = 1.0, d: Optional[int] = None,
                      stream: Optional[int] = None) -> None:
    """conqur_score_rows_static on the rotated rows Y (2-D device tensor, bf16 or fp32): out (device tensor of 2 float64)
    receives {SSE, energy} once the stream has passed the call; d: row width used (default: all columns of Y).
    Allocates nothing and does not synchronise."""
    import torch
    if Y.dim() != 2 or Y.stride(1) != 1 or not Y.is_cuda or Y.dtype not in (torch.bfloat16, torch.float32):
        raise ValueError("Y must be a 2-D bf16 or fp32 device tensor with unit column stride")
    if out.dtype != torch.float64 or out.numel() < 2 or not out.is_cuda or not out.is_contiguous():
        raise ValueError("out must be a contiguous device tensor of 2 float64")
    if stream is None:
        stream = torch.cuda.current_stream(Y.device).cuda_stream
    st = load().conqur_score_rows_static(Y.data_ptr(), BF16 if Y.dtype == torch.bfloat16 else F32, Y.shape[0], Y.shape[1] if d is None else d,
                                         Y.stride(0), bits, 1 if zero_point else 0, ctypes.c_float(clip_ratio),
                                         out.data_ptr(), ctypes.c_void_p(stream))
    if st != OK:
        raise ConqurError(st, "conqur_score_rows_static failed")


def to_device(x: np.ndarray, dtype: str, device: str = "cuda:0"):
    """float32 numpy [T, d] (bf16-representable for dtype 'bf16') -> device tensor of the activation dtype."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32))
    if dtype == "bf16":
        t = t.to(torch.bfloat16)
    return t.to(device)
