"""ctypes wrapper over the fp64 CPU oracle (conqur_oracle.c) -- TEST INFRASTRUCTURE.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import
this module; the product path never does.  The wrapper marshals numpy arrays
and keeps the calibration state (R as fp32, M as fp64 accumulators, the l1
accumulator L and the row counts) the way Alg. 1 carries it between
mini-batches; all arithmetic of the method is in the C file.

Parity pins: see the header of conqur_oracle.c and tests/test_oracle_*.py.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "conqur_oracle.c")
_LIB = os.path.join(_HERE, "libconqur_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (fp64, no fast-math, OpenMP over independent rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fno-fast-math", "-ffp-contract=off", "-shared", "-fPIC",
               "-std=c11", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        u64, dbl, i32 = ctypes.c_uint64, ctypes.c_double, ctypes.c_int
        p = ctypes.c_void_p
        L.oq_num_threads.restype = i32
        L.oq_round_bf16_f64.restype = dbl
        L.oq_round_bf16_f64.argtypes = [dbl]
        L.oq_round_operand.restype = None
        L.oq_round_operand.argtypes = [p, p, u64, i32]
        L.oq_step_batch.restype = i32
        L.oq_step_batch.argtypes = [p, u64, u64, u64, u64, p, p, p, p, p, p, p]
        L.oq_jacobi_svd.restype = i32
        L.oq_jacobi_svd.argtypes = [p, u64, p, p, p]
        L.oq_procrustes.restype = i32
        L.oq_procrustes.argtypes = [p, p, u64, dbl, p, p]
        L.oq_quant_error.restype = i32
        L.oq_quant_error.argtypes = [p, u64, u64, u64, u64, p, i32, i32, p, p, p, p]
        L.oq_rotate.restype = i32
        L.oq_rotate.argtypes = [p, u64, u64, u64, u64, p, i32, p]
        L.oq_row_diagnostics.restype = i32
        L.oq_row_diagnostics.argtypes = [p, u64, u64, u64, u64, p, i32, p, p]
        L.oq_fake_quant.restype = i32
        L.oq_fake_quant.argtypes = [p, u64, u64, u64, u64, p, i32, i32, i32, ctypes.c_float, p]
        L.oq_quant_error_zp.restype = i32
        L.oq_quant_error_zp.argtypes = [p, u64, u64, u64, u64, p, i32, i32, ctypes.c_float, p, p, p, p]
        _lib = L
    return _lib


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def num_threads() -> int:
    return int(lib().oq_num_threads())


def round_bf16(y: float) -> float:
    return float(lib().oq_round_bf16_f64(float(y)))


def round_operand(R: np.ndarray, dtype: str) -> np.ndarray:
    R = np.ascontiguousarray(R, dtype=np.float32)
    out = np.empty_like(R)
    lib().oq_round_operand(_ptr(R), _ptr(out), R.size, 1 if dtype == "bf16" else 0)
    return out


def jacobi_svd(A: np.ndarray):
    A = np.ascontiguousarray(A, dtype=np.float64)
    d = A.shape[0]
    assert A.shape == (d, d)
    U = np.empty((d, d)); V = np.empty((d, d)); s = np.empty(d)
    sweeps = lib().oq_jacobi_svd(_ptr(A), d, _ptr(U), _ptr(s), _ptr(V))
    if sweeps < 0:
        raise RuntimeError("oq_jacobi_svd failed")
    return U, s, V, sweeps


def procrustes(M: np.ndarray, R_prev: Optional[np.ndarray] = None, prox_lambda: float = 0.0):
    """R = U V^T of A = M + lambda * tau * R_prev (Sec. 3.3). Returns (R fp64, stats dict)."""
    M = np.ascontiguousarray(M, dtype=np.float64)
    d = M.shape[0]
    Rp = None if R_prev is None else np.ascontiguousarray(R_prev, dtype=np.float64)
    R = np.empty((d, d)); st = np.zeros(5)
    if lib().oq_procrustes(_ptr(M), _ptr(Rp), d, float(prox_lambda), _ptr(R), _ptr(st)) != 0:
        raise RuntimeError("oq_procrustes failed")
    return R, dict(inner=st[0], nuclear=st[1], orth_err=st[2], tau=st[3], sweeps=int(st[4]))


class OracleCalibrator:
    """State of one rotation (or `heads` block rotations) across the stream (Alg. 1)."""

    def __init__(self, d: int, heads: int, dtype: str, R0: np.ndarray, prox_lambda: float = 0.0):
        assert d % heads == 0 and dtype in ("f32", "bf16")
        self.d, self.heads, self.dh, self.dtype = d, heads, d // heads, dtype
        self.prox_lambda = float(prox_lambda)
        self.R = np.ascontiguousarray(R0, dtype=np.float32).reshape(heads, self.dh, self.dh).copy()
        self.reset_stats()

    def reset_stats(self):
        self.M = np.zeros((self.heads, self.dh, self.dh), dtype=np.float64)
        self.L = np.zeros(self.heads, dtype=np.float64)
        self.n = np.zeros(self.heads, dtype=np.uint64)
        self.skipped = np.zeros(self.heads, dtype=np.uint64)

    @property
    def R_op(self) -> np.ndarray:
        return round_operand(self.R, self.dtype)

    def step_batch(self, X: np.ndarray, want_Y: bool = False, want_S: bool = False):
        X = np.ascontiguousarray(X, dtype=np.float32)
        T, stride = X.shape
        assert stride >= self.d
        Y = np.empty((T, self.d), dtype=np.float64) if want_Y else None
        S = np.empty((T, self.d), dtype=np.int8) if want_S else None
        Rop = self.R_op
        rc = lib().oq_step_batch(_ptr(X), T, self.d, self.heads, stride, _ptr(Rop), _ptr(self.M),
                                 _ptr(self.L), _ptr(self.n), _ptr(self.skipped), _ptr(Y), _ptr(S))
        if rc != 0:
            raise RuntimeError("oq_step_batch failed")
        return Y, S

    def objective(self) -> np.ndarray:
        """Eq. 1 via the l1 identity of Sec. 3.2: 2 n - (2 / sqrt(d)) L, per head."""
        return 2.0 * self.n.astype(np.float64) - 2.0 * self.L / np.sqrt(float(self.dh))

    def update_rotation(self):
        """R <- U V^T per head, then the statistics are cleared (Alg. 1 re-initialises them)."""
        stats = []
        for h in range(self.heads):
            Rn, st = procrustes(self.M[h], self.R[h].astype(np.float64), self.prox_lambda)
            self.R[h] = Rn.astype(np.float32)
            stats.append(st)
        self.reset_stats()
        return stats

    def quant_error(self, X: np.ndarray, bits: int = 4, want_rows: bool = False, want_codes: bool = False):
        X = np.ascontiguousarray(X, dtype=np.float32)
        T, stride = X.shape
        sse = ctypes.c_double(0.0); en = ctypes.c_double(0.0)
        rows = np.empty(T, dtype=np.float64) if want_rows else None
        codes = np.empty((T, self.d), dtype=np.int8) if want_codes else None
        Rop = self.R_op
        rc = lib().oq_quant_error(_ptr(X), T, self.d, self.heads, stride, _ptr(Rop),
                                  1 if self.dtype == "bf16" else 0, bits,
                                  ctypes.byref(sse), ctypes.byref(en), _ptr(rows), _ptr(codes))
        if rc != 0:
            raise RuntimeError("oq_quant_error failed")
        return sse.value, en.value, rows, codes

    def rotate(self, X: np.ndarray) -> np.ndarray:
        """Y = X R_op per head, stored in the activation dtype (returned as float32)."""
        X = np.ascontiguousarray(X, dtype=np.float32)
        T, stride = X.shape
        Y = np.empty((T, self.d), dtype=np.float32)
        rc = lib().oq_rotate(_ptr(X), T, self.d, self.heads, stride, _ptr(self.R_op), 1 if self.dtype == "bf16" else 0, _ptr(Y))
        if rc != 0:
            raise RuntimeError("oq_rotate failed")
        return Y

    def fake_quant(self, X: np.ndarray, bits: int = 4, zero_point: bool = True, clip: float = 1.0) -> np.ndarray:
        """Q(X R_op): the fake-quantised rotated rows a quantised linear layer receives (Sec. 3.4), as float32."""
        X = np.ascontiguousarray(X, dtype=np.float32)
        T, stride = X.shape
        Yq = np.empty((T, self.d), dtype=np.float32)
        rc = lib().oq_fake_quant(_ptr(X), T, self.d, self.heads, stride, _ptr(self.R_op), 1 if self.dtype == "bf16" else 0,
                                 bits, 1 if zero_point else 0, ctypes.c_float(clip), _ptr(Yq))
        if rc != 0:
            raise RuntimeError("oq_fake_quant failed")
        return Yq

    def row_diagnostics(self, X: np.ndarray):
        """Per row of Y = X R_op: normalised participation ratio PR/d (Sec. 4.2) and ||y||_inf^2/||y||_2^2 (App. B)."""
        X = np.ascontiguousarray(X, dtype=np.float32)
        T, stride = X.shape
        pr = np.empty(T, dtype=np.float64); rho = np.empty(T, dtype=np.float64)
        rc = lib().oq_row_diagnostics(_ptr(X), T, self.d, self.heads, stride, _ptr(self.R_op),
                                      1 if self.dtype == "bf16" else 0, _ptr(pr), _ptr(rho))
        if rc != 0:
            raise RuntimeError("oq_row_diagnostics failed")
        return pr, rho

    def quant_error_zp(self, X: np.ndarray, bits: int = 4, clip: float = 1.0, want_rows: bool = False,
                       want_codes: bool = False):
        """Asymmetric (zero-point) per-token quantiser of App. B with the clipping ratio of App. C."""
        X = np.ascontiguousarray(X, dtype=np.float32)
        T, stride = X.shape
        sse = ctypes.c_double(0.0); en = ctypes.c_double(0.0)
        rows = np.empty(T, dtype=np.float64) if want_rows else None
        codes = np.empty((T, self.d), dtype=np.uint8) if want_codes else None
        Rop = self.R_op
        rc = lib().oq_quant_error_zp(_ptr(X), T, self.d, self.heads, stride, _ptr(Rop),
                                     1 if self.dtype == "bf16" else 0, bits, ctypes.c_float(clip),
                                     ctypes.byref(sse), ctypes.byref(en), _ptr(rows), _ptr(codes))
        if rc != 0:
            raise RuntimeError("oq_quant_error_zp failed")
        return sse.value, en.value, rows, codes
