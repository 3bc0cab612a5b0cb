"""Coupled-Newton iteration for A^(-1/p) (paper Section 3.2).

TEST INFRASTRUCTURE (see oracle/__init__.py).  float64, plain matmuls, the paper's order.

  X_0 = I / c,  M_0 = A / c^p
  C_k = (1 + 1/p) I - M_k / p
  X_{k+1} = X_k C_k,   M_{k+1} = C_k^p M_k
  X_k -> A^(-1/p),  M_k -> I        (needs eigenvalues of A in [0, (p+1) c^p])

With c = (1+p)^(-1/p) the admissible interval is [0, 1] (Section 3.4), so the block is
damped, scaled by s >= lambda_max as for Newton-DB, and the result un-scaled by s^(-1/p).
The right end is in fact excluded: at x = 1 the first C is exactly 0 and the iterate stays
0, so s must be strictly larger than lambda_max (the Frobenius norm is, for B > 1).
Matmuls per iteration as the paper counts them: one for X, one (p=2) or two (p=4) for
C^p by repeated squaring, one for M: 3 (p=2) or 4 (p=4).
"""
from __future__ import annotations

import numpy as np

from .newton_db import MatmulCounter, block_scale


def cn_constant(p: int) -> float:
    """c with (p+1) c^p = 1."""
    return (1.0 + p) ** (-1.0 / p)


def matrix_power_by_squaring(C: np.ndarray, p: int, counter: MatmulCounter):
    if p == 2:
        return counter.mm(C, C)
    if p == 4:
        C2 = counter.mm(C, C)
        return counter.mm(C2, C2)
    raise ValueError("p must be 2 or 4")


def cn_plain(A: np.ndarray, p: int, iters: int, c: float | None = None, counter: MatmulCounter | None = None):
    """The iteration exactly as the equations state it.  Returns (X_k, M_k)."""
    cnt = counter or MatmulCounter()
    if c is None:
        c = cn_constant(p)
    n = A.shape[0]
    I = np.eye(n)
    X, M = I / c, A / c ** p
    for _ in range(iters):
        C = (1.0 + 1.0 / p) * I - M / p
        X = cnt.mm(X, C)
        M = cnt.mm(matrix_power_by_squaring(C, p, cnt), M)
    return X, M


def cn_scalar(x, p: int, iters: int, c: float | None = None):
    """The iteration on an eigenvalue x.  Returns (x_k, m_k)."""
    if c is None:
        c = cn_constant(p)
    x = np.asarray(x, dtype=np.float64)
    xk, m = np.ones_like(x) / c, x / c ** p
    for _ in range(iters):
        ck = (1.0 + 1.0 / p) - m / p
        xk, m = xk * ck, ck ** p * m
    return xk, m


def cn_scalar_steps_to_tol(x: float, p: int = 2, tol: float = 1e-10, max_iters: int = 500) -> int:
    """Iterations until |x_k - x^(-1/p)| <= tol (the experiment of the paper's Figures 1-2)."""
    c = cn_constant(p)
    xk, m = 1.0 / c, x / c ** p
    target = x ** (-1.0 / p)
    for k in range(1, max_iters + 1):
        ck = (1.0 + 1.0 / p) - m / p
        xk, m = xk * ck, ck ** p * m
        if abs(xk - target) <= tol:
            return k
    return max_iters + 1


def inverse_root_cn(A, p: int, iters: int, eps: float = 0.0, scaling: str = "frobenius",
                    counter: MatmulCounter | None = None, pi=None):
    """X_i ~ (A_i + eps I)^(-1/p): damp, scale by s, iterate with c = (1+p)^(-1/p), un-scale."""
    A = np.asarray(A, dtype=np.float64)
    single = A.ndim == 2
    if single:
        A = A[None]
    X = np.empty_like(A)
    eye = np.eye(A.shape[1])
    for i in range(A.shape[0]):
        Ad = A[i] + eps * eye
        s = block_scale(Ad, scaling, pi)
        Xk, _ = cn_plain(Ad / s, p, iters, counter=counter)
        X[i] = Xk * s ** (-1.0 / p)
    return X[0] if single else X


def inverse_root_cn_model(A, p: int, iters: int, eps: float = 0.0, scaling: str = "frobenius", pi=None):
    """The same result through the spectrum (every iterate is a polynomial in A)."""
    A = np.asarray(A, dtype=np.float64)
    single = A.ndim == 2
    if single:
        A = A[None]
    X = np.empty_like(A)
    eye = np.eye(A.shape[1])
    for i in range(A.shape[0]):
        Ad = 0.5 * (A[i] + A[i].T) + eps * eye
        s = block_scale(Ad, scaling, pi)
        lam, Q = np.linalg.eigh(Ad)
        xk, _ = cn_scalar(lam / s, p, iters)
        X[i] = (Q * (xk * s ** (-1.0 / p))[None, :]) @ Q.T
    return X[0] if single else X
