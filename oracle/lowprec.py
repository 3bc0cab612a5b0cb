"""Emulation of the mixed-precision recipe of the paper's Appendix A.3 (operands of each
matmul rounded to half precision, accumulation and everything else in single precision),
with bf16 as the half format, applied to Newton-DB (Section 3.3) and to Clenshaw.

TEST INFRASTRUCTURE (see oracle/__init__.py).

PARITY UNPINNED for the Newton-DB part beyond what follows: the paper gives no numbers
for low-precision Newton-DB (it reports it unstable and leaves it to future work), so the
only pins are (i) the rounding function against exact bf16 facts and torch's conversion,
(ii) the emulation with rounding switched off equals the float64 iteration, (iii) on
inputs whose iterates are exactly representable in bf16 it equals the exact iteration.
The GPU path is compared with this emulation for few iterations (where the two cannot
have drifted apart) and otherwise only reported against the eigendecomposition root.

Products are evaluated in float64 on the rounded operands and then rounded to float32;
this differs from a float32 accumulation by at most a few float32 ulps per element.
"""
from __future__ import annotations

import numpy as np

from .newton_db import block_scale


def round_bf16(x) -> np.ndarray:
    """Round-to-nearest-even from float32 to bfloat16 (8 significand bits), returned as
    float32 values.  NaN stays NaN, overflow goes to infinity."""
    x32 = np.ascontiguousarray(x, dtype=np.float32)
    bits = x32.view(np.uint32).astype(np.uint64)
    lsb = (bits >> np.uint64(16)) & np.uint64(1)
    rounded = (bits + np.uint64(0x7FFF) + lsb) & np.uint64(0xFFFF0000)
    out = rounded.astype(np.uint32).view(np.float32).copy()
    nan = np.isnan(x32)
    if nan.any():
        out[nan] = np.nan
    return out.reshape(x32.shape)


def _f32(x):
    return np.asarray(x, dtype=np.float32)


def matmul_bf16(A, B, rounding: bool = True) -> np.ndarray:
    """float32( bf16(A) @ bf16(B) ) with the product summed in float64."""
    a = round_bf16(A) if rounding else _f32(A)
    b = round_bf16(B) if rounding else _f32(B)
    return _f32(a.astype(np.float64) @ b.astype(np.float64))


def ndb_call_lowprec(M32, iters: int, rounding: bool = True):
    """One Newton-DB call on a float32 matrix M (first update in closed form), every product
    through matmul_bf16, every linear combination in float32.  Returns float32 (Y, Z)."""
    n = M32.shape[0]
    I = np.eye(n, dtype=np.float32)
    E = _f32(np.float32(1.5) * I - np.float32(0.5) * M32)
    Y, Z = matmul_bf16(M32, E, rounding), E
    for _ in range(iters - 1):
        E = _f32(np.float32(1.5) * I - np.float32(0.5) * matmul_bf16(Z, Y, rounding))
        Y, Z = matmul_bf16(Y, E, rounding), matmul_bf16(E, Z, rounding)
    return Y, Z


def inverse_root_ndb_lowprec(A, p: int, iters: int, eps: float = 0.0, scaling: str = "frobenius",
                             rounding: bool = True) -> np.ndarray:
    """(A + eps I)^(-1/p) by Newton-DB with bf16-rounded matmul operands; same damping,
    scaling, chaining and un-scaling as oracle.newton_db.inverse_root_ndb."""
    A = np.asarray(A, dtype=np.float32)
    single = A.ndim == 2
    if single:
        A = A[None]
    X = np.empty(A.shape, dtype=np.float32)
    n = A.shape[1]
    I = np.eye(n, dtype=np.float32)
    for i in range(A.shape[0]):
        Ad = _f32(A[i] + np.float32(eps) * I)
        s = np.float32(block_scale(Ad.astype(np.float64), scaling))
        As = _f32(Ad * (np.float32(1.0) / s))
        with np.errstate(over="ignore", invalid="ignore"):
            Y, Z = ndb_call_lowprec(As, iters, rounding)
            if p == 4:
                _, Z = ndb_call_lowprec(Y, iters, rounding)
        X[i] = _f32(Z * np.float32(float(s) ** (-1.0 / p)))
    return X[0] if single else X
