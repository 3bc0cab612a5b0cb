"""Emulation of the mixed-precision recipe of the paper's Appendix A.3 (operands of each
matmul rounded to half precision, accumulation and everything else in single precision),
with fp16 (the paper's format), bf16, or split bf16 operands (two bf16 planes per operand
and three products, or three planes and six products), applied to Newton-DB (Section 3.3) and Coupled-Newton (Section 3.2).

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


def round_fp16(x) -> np.ndarray:
    """Round-to-nearest-even from float32 to IEEE half precision (11 significand bits, with
    subnormals, overflow to infinity), returned as float32 values."""
    with np.errstate(over="ignore"):
        return np.asarray(x, dtype=np.float32).astype(np.float16).astype(np.float32)


def round_half(x, fmt: str) -> np.ndarray:
    if fmt == "bf16":
        return round_bf16(x)
    if fmt == "fp16":
        return round_fp16(x)
    if fmt == "none":
        return _f32(x)
    raise ValueError(fmt)


def _f32(x):
    return np.asarray(x, dtype=np.float32)


def split_bf16(x):
    """x ~ hi + lo with hi = bf16(x), lo = bf16(x - hi) (both as float32 values)."""
    hi = round_bf16(x)
    with np.errstate(invalid="ignore"):
        lo = round_bf16(_f32(x) - hi)
    return hi, lo


FP16_LO_SCALE = np.float32(2048.0)   # 2^11: the low fp16 plane is stored times this, so that it does not go subnormal


def split_fp16(x):
    """x ~ hi + lo with hi = fp16(x) and lo = fp16((x - hi) 2^11) 2^-11 (as float32 values): 22 significand bits.
    The low plane is rounded after scaling by 2^11 -- it is 2^-11 of x or less, and unscaled it would fall into
    fp16's subnormal range for |x| < 0.125."""
    hi = round_fp16(x)
    with np.errstate(invalid="ignore", over="ignore"):
        lo = round_fp16((_f32(x) - hi) * FP16_LO_SCALE) / FP16_LO_SCALE
    return hi, _f32(lo)


def split3_bf16(x):
    """x ~ hi + mid + lo, three bf16 planes: hi = bf16(x), mid = bf16(x - hi), lo = bf16(x - hi - mid)
    (as float32 values; the differences are exact in float32)."""
    hi, mid = split_bf16(x)
    with np.errstate(invalid="ignore"):
        lo = round_bf16(_f32(_f32(x) - hi) - mid)
    return hi, mid, lo


def matmul_lowprec(A, B, fmt: str = "bf16") -> np.ndarray:
    """float32( half(A) @ half(B) ) with the product summed in float64.  fmt = 'bf16x3': both operands
    split into two bf16 planes, product = A_lo B_hi + A_hi B_lo + A_hi B_hi (lo*lo dropped).  fmt = 'bf16x6':
    three planes each, the six plane products of weight 2^-16 and above:
    A_lo B_hi + A_hi B_lo + A_mid B_mid + A_mid B_hi + A_hi B_mid + A_hi B_hi.  fmt = 'fp16x3': two fp16 planes
    (split_fp16: 22 significand bits), the same three products as 'bf16x3'."""
    if fmt == "bf16x6":
        ah, am, al = (t.astype(np.float64) for t in split3_bf16(A))
        bh, bm, bl = (t.astype(np.float64) for t in split3_bf16(B))
        with np.errstate(over="ignore", invalid="ignore"):
            return _f32(al @ bh + ah @ bl + am @ bm + am @ bh + ah @ bm + ah @ bh)
    if fmt == "fp16x3":
        ah, al = (t.astype(np.float64) for t in split_fp16(A))
        bh, bl = (t.astype(np.float64) for t in split_fp16(B))
        with np.errstate(over="ignore", invalid="ignore"):
            return _f32((al @ bh + ah @ bl) + ah @ bh)
    if fmt == "bf16x3":
        ah, al = (t.astype(np.float64) for t in split_bf16(A))
        bh, bl = (t.astype(np.float64) for t in split_bf16(B))
        with np.errstate(over="ignore", invalid="ignore"):
            return _f32(al @ bh + ah @ bl + ah @ bh)
    a, b = round_half(A, fmt), round_half(B, fmt)
    with np.errstate(over="ignore", invalid="ignore"):
        return _f32(a.astype(np.float64) @ b.astype(np.float64))


def matmul_bf16(A, B, rounding: bool = True) -> np.ndarray:
    return matmul_lowprec(A, B, "bf16" if rounding else "none")


def ndb_call_lowprec(M32, iters: int, rounding=True):
    """One Newton-DB call on a float32 matrix M (first update in closed form), every product
    through matmul_lowprec, every linear combination in float32.  `rounding` is True (bf16),
    False (no rounding) or a format name.  Returns float32 (Y, Z)."""
    fmt = rounding if isinstance(rounding, str) else ("bf16" if rounding else "none")
    n = M32.shape[0]
    I = np.eye(n, dtype=np.float32)
    E = _f32(np.float32(1.5) * I - np.float32(0.5) * M32)
    Y, Z = matmul_lowprec(M32, E, fmt), E
    for _ in range(iters - 1):
        E = _f32(np.float32(1.5) * I - np.float32(0.5) * matmul_lowprec(Z, Y, fmt))
        Y, Z = matmul_lowprec(Y, E, fmt), matmul_lowprec(E, Z, fmt)
    return Y, Z


def inverse_root_cn_lowprec(A, p: int, iters: int, eps: float = 0.0, scaling: str = "frobenius",
                            fmt: str = "fp16") -> np.ndarray:
    """(A + eps I)^(-1/p) by Coupled-Newton (Section 3.2, c = (1+p)^(-1/p)) with half-rounded matmul
    operands: M_0 = (p+1) A_s, C_k = (1+1/p) I - M_k/p in float32, X_{k+1} = X_k C_k,
    M_{k+1} = C_k^p M_k (powers by repeated squaring), X un-scaled by s^(-1/p)."""
    A = np.asarray(A, dtype=np.float32)
    single = A.ndim == 2
    if single:
        A = A[None]
    X = np.empty(A.shape, dtype=np.float32)
    n = A.shape[1]
    I = np.eye(n, dtype=np.float32)
    a, ip = np.float32(1.0 + 1.0 / p), np.float32(1.0 / p)
    inv_c = np.float32((1.0 + p) ** (1.0 / p))
    for i in range(A.shape[0]):
        Ad = _f32(A[i] + np.float32(eps) * I)
        s = np.float32(block_scale(Ad.astype(np.float64), scaling))
        M = _f32(np.float32(p + 1) * (Ad * (np.float32(1.0) / s)))
        C = _f32(a * I - ip * M)
        # X_k = (1/c) C_0 C_1 ... C_{k-1}: the scalar 1/c is applied once at the end, so the first
        # update X_1 = C_0 / c needs no product and no rounding
        Xk = None
        for k in range(iters):
            Xk = C if k == 0 else matmul_lowprec(Xk, C, fmt)        # X_{k+1} = X_k C_k
            if k + 1 < iters:                                        # the last M is never read
                P = matmul_lowprec(C, C, fmt)
                if p == 4:
                    P = matmul_lowprec(P, P, fmt)
                M = matmul_lowprec(P, M, fmt)                        # M_{k+1} = C_k^p M_k
                C = _f32(a * I - ip * M)
        X[i] = _f32(Xk * (inv_c * np.float32(float(s) ** (-1.0 / p))))
    return X[0] if single else X


def inverse_root_cn_lowprec_as_printed(A, p: int, iters: int, eps: float = 0.0, scaling: str = "frobenius",
                                       fmt: str = "fp16") -> np.ndarray:
    """Coupled-Newton exactly in the order Section 3.2 prints it, every product through matmul_lowprec:
    X_0 = I/c, M_0 = A_s/c^p; for k = 0 .. iters-1: C_k = (1+1/p) I - M_k/p, X_{k+1} = X_k C_k,
    M_{k+1} = C_k^p M_k -- including the product X_0 C_0 with the rounded scalar matrix I/c and the last M that
    nobody reads.  inverse_root_cn_lowprec carries 1/c to the end instead (a reading that saves two products and
    one rounding); this function is what pins that reading: the two must agree to the precision of the operand
    format (tests/test_oracle_lowprec.py)."""
    A = np.asarray(A, dtype=np.float32)
    single = A.ndim == 2
    if single:
        A = A[None]
    X = np.empty(A.shape, dtype=np.float32)
    n = A.shape[1]
    I = np.eye(n, dtype=np.float32)
    c = (1.0 + p) ** (-1.0 / p)
    for i in range(A.shape[0]):
        Ad = _f32(A[i] + np.float32(eps) * I)
        s = np.float32(block_scale(Ad.astype(np.float64), scaling))
        Xk = _f32(I * np.float32(1.0 / c))
        M = _f32((Ad * (np.float32(1.0) / s)) * np.float32(c ** -p))
        for _ in range(iters):
            C = _f32(np.float32(1.0 + 1.0 / p) * I - np.float32(1.0 / p) * M)
            Xk = matmul_lowprec(Xk, C, fmt)
            P = matmul_lowprec(C, C, fmt)
            if p == 4:
                P = matmul_lowprec(P, P, fmt)
            M = matmul_lowprec(P, M, fmt)
        X[i] = _f32(Xk * np.float32(float(s) ** (-1.0 / p)))
    return X[0] if single else X


def inverse_root_ndb_lowprec(A, p: int, iters: int, eps: float = 0.0, scaling: str = "frobenius",
                             rounding=True) -> np.ndarray:
    """(A + eps I)^(-1/p) by Newton-DB with half-rounded matmul operands (bf16 when rounding is
    True, or the named format); same damping, scaling, chaining and un-scaling as
    oracle.newton_db.inverse_root_ndb."""
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
