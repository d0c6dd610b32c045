"""Seeded synthetic calibration-activation streams.

This module only *draws inputs*: it holds none of the method's arithmetic (no
rotation, no normalisation, no corner assignment, no Procrustes, no quantiser)
and imports neither the HIP binding nor the CPU oracle.  Both sides are handed
the arrays produced here, so the same seed gives bit-identical inputs to each.

The streams stand in for the activations of the Llama-family models the paper
calibrates on (Sec. 4, experimental setup: 128 sequences of 2048 tokens); the
widths 3072 / 4096 / 8192 and 32 heads x 128 mirror the residual-stream and
per-head o_proj sites of those models (App. A).  No item of any dataset is
reproduced: every value is drawn from a counter-based generator (Philox), keyed
by (seed, batch index), so any batch can be regenerated independently.

Value recipe (per workload, see WORKLOADS):
  x_ij = s_j * z_ij                 z ~ N(0,1), s_j = exp(sigma * g_j), g ~ N(0,1)
  outlier channels                  s_j multiplied by a fixed factor (or U(lo,hi))
  heavy-tailed token magnitudes     row i multiplied by |t_i|, t ~ Student-t(nu=4)
  massive-activation rows           a fraction of rows gets x1000 on 2 fixed channels
  bf16 workloads                    every value rounded once to bf16 (nearest-even)
"""
from __future__ import annotations

import dataclasses
from typing import Optional, Tuple

import numpy as np


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    d: int                      # row width of X
    heads: int                  # 1 = one d x d rotation, h > 1 = h blocks of (d/h)
    dtype: str                  # "f32" or "bf16" (activation dtype)
    tokens_per_batch: int
    n_batches: int
    sigma: float                # log-normal channel-scale spread
    n_outliers: int             # outlier channels (per head when heads > 1)
    outlier_lo: float
    outlier_hi: float           # == lo -> fixed factor
    student_t: bool             # per-token |t_4| magnitude
    massive_frac: float         # fraction of rows with x1000 on 2 fixed channels
    prox_lambda: float          # proximal weight used for this workload
    seed: int

    @property
    def dh(self) -> int:
        return self.d // self.heads


# The five workloads (names c1..c5).  prox_lambda: 0 where tokens per update
# >= 8 * block width (the paper's own regime, unique polar factor); 0.1 where a
# 2048/4096-token batch leaves the d x d cross-covariance rank deficient.
WORKLOADS = {
    "c1": Workload("c1", 256, 1, "f32", 2048, 4, 0.5, 3, 40.0, 40.0, False, 0.0, 0.0, 1001),
    "c2": Workload("c2", 3072, 1, "bf16", 2048, 128, 0.5, 6, 50.0, 100.0, True, 0.0, 0.1, 1002),
    "c3": Workload("c3", 4096, 1, "bf16", 2048, 128, 0.5, 8, 100.0, 100.0, True, 0.001, 0.1, 1003),
    "c4": Workload("c4", 4096, 32, "bf16", 2048, 128, 0.7, 2, 30.0, 30.0, False, 0.0, 0.0, 1004),
    "c5": Workload("c5", 8192, 1, "bf16", 4096, 32, 0.5, 12, 100.0, 100.0, True, 0.0, 0.1, 1005),
}


def small_workload(d: int, tokens: int, n_batches: int = 2, heads: int = 1,
                   dtype: str = "bf16", seed: int = 7, student_t: bool = True,
                   n_outliers: int = 2, massive_frac: float = 0.0,
                   prox_lambda: float = 0.0) -> Workload:
    """A reduced-size workload with the same value recipe (for parity tests)."""
    return Workload(f"small_d{d}_h{heads}_{dtype}", d, heads, dtype, tokens, n_batches,
                    0.5, n_outliers, 50.0, 100.0, student_t, massive_frac, prox_lambda, seed)


def _rng(seed: int, stream: int, index: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[np.uint64(seed), np.uint64((stream << 32) | index)]))


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even); result stays fp32."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of an fp32 array whose values are bf16-representable."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    assert not np.any(u & np.uint32(0xFFFF)), "values are not bf16-representable"
    return (u >> np.uint32(16)).astype(np.uint16)


def channel_scales(w: Workload) -> np.ndarray:
    """Per-channel standard deviations s_j (length d), outlier channels included."""
    g = _rng(w.seed, 1)
    s = np.exp(w.sigma * g.standard_normal(w.d))
    dh = w.dh
    for h in range(w.heads):
        idx = g.choice(dh, size=w.n_outliers, replace=False) + h * dh
        if w.outlier_hi > w.outlier_lo:
            f = g.uniform(w.outlier_lo, w.outlier_hi, size=w.n_outliers)
        else:
            f = np.full(w.n_outliers, w.outlier_lo)
        s[idx] *= f
    return s


def massive_channels(w: Workload) -> np.ndarray:
    return _rng(w.seed, 2).choice(w.d, size=2, replace=False)


def batch(w: Workload, b: int, tokens: Optional[int] = None) -> np.ndarray:
    """Batch b of the stream: float32 [tokens, d]; bf16-representable for bf16 workloads."""
    T = w.tokens_per_batch if tokens is None else tokens
    g = _rng(w.seed, 3, b)
    x = g.standard_normal((T, w.d), dtype=np.float32)
    x *= channel_scales(w).astype(np.float32)[None, :]
    if w.student_t:
        z = g.standard_normal(T)
        chi2 = g.chisquare(4.0, size=T)
        x *= np.abs(z / np.sqrt(chi2 / 4.0)).astype(np.float32)[:, None]
    if w.massive_frac > 0.0:
        rows = np.nonzero(g.random(T) < w.massive_frac)[0]
        ch = massive_channels(w)
        x[np.ix_(rows, ch)] *= np.float32(1000.0)
    if w.dtype == "bf16":
        x = round_to_bf16(x)
    return x


def iid_row_indices(seed: int, update: int, n_pool: int, n_rows: int) -> np.ndarray:
    """Row indices (int64, with replacement) of the stored activations that update number `update` of the offline
    variant draws (Sec. 4.4: the stored activations are sampled i.i.d. during optimisation)."""
    return _rng(seed, 6, update).integers(0, n_pool, size=n_rows, dtype=np.int64)


def initial_rotation(w: Workload) -> np.ndarray:
    """R0: [heads, dh, dh] float32, Haar-distributed per head.

    Q of the QR factorisation of a seeded Gaussian, with the columns' signs
    fixed by the diagonal of the triangular factor (so the law is Haar)."""
    g = _rng(w.seed, 4)
    dh = w.dh
    out = np.empty((w.heads, dh, dh), dtype=np.float32)
    for h in range(w.heads):
        a = g.standard_normal((dh, dh))
        q, r = np.linalg.qr(a)
        q = q * np.sign(np.diag(r))[None, :]
        out[h] = q.astype(np.float32)
    return out


def random_orthogonal(d: int, seed: int) -> np.ndarray:
    """A Haar orthogonal d x d matrix in float64 (test helper; an input, not the method)."""
    g = _rng(seed, 5)
    q, r = np.linalg.qr(g.standard_normal((d, d)))
    return q * np.sign(np.diag(r))[None, :]


def spd_with_spectrum(d: int, sigma: np.ndarray, seed: int) -> Tuple[np.ndarray, np.ndarray]:
    """(P, W): P = W diag(sigma) W^T symmetric positive definite with a prescribed spectrum."""
    w = random_orthogonal(d, seed + 101)
    p = (w * np.asarray(sigma, dtype=np.float64)[None, :]) @ w.T
    return 0.5 * (p + p.T), w


def hadamard_rotation(d: int, heads: int = 1, seed: int = 0) -> np.ndarray:
    """Randomised Hadamard initial rotation [heads, dh, dh] (dh a power of two): Sylvester's H / sqrt(dh) with a seeded
    random sign per row, the fixed-rotation baseline the paper compares against."""
    dh = d // heads
    if dh & (dh - 1):
        raise ValueError("dh must be a power of two")
    H = np.ones((1, 1), dtype=np.float32)
    while H.shape[0] < dh:
        H = np.block([[H, H], [H, -H]])
    out = np.empty((heads, dh, dh), dtype=np.float32)
    for h in range(heads):
        sgn = np.where(_rng(seed, 9000 + h).random(dh) < 0.5, -1.0, 1.0).astype(np.float32)
        out[h] = (sgn[:, None] * H) / np.float32(np.sqrt(dh))
    return out

