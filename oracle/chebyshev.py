"""Chebyshev approximation of x^(-1/p) evaluated by Clenshaw's recurrence
(paper Appendix A: coefficient fit, scalar Clenshaw, matrix Clenshaw, and the
reduced form with d-1 matmuls).

TEST INFRASTRUCTURE (see oracle/__init__.py).  float64 throughout.

Readings of points the paper leaves open or prints inconsistently:
  * The recurrence variable is the point mapped to [-1, 1]: t = (2x - (a+b)) / (b-a).
    The scalar listing writes the recurrence with "x"; a cosine-series fit on nodes
    t = cos(theta) only makes sense with the mapped variable.
  * The matrix listing maps with S = 2 A/||A||_F - I (i.e. the map of [0,1]) while it
    fits on [eps, 1+eps]; that evaluates f(x + eps) on the scaled spectrum.  Here the
    map interval [a, b] is an explicit argument, so the listing's form is (a,b) = (0,1)
    with coefficients fitted on [eps, 1+eps].
  * In the derivation of the reduced form one line prints "- B_1" where the recurrence
    gives "- B_2"; the final expression (S B_1 - B_2 + c_0 I) is the consistent one.
  * The loop set printed as {d-2, d-1, ..., 1} is the descending range d-2, d-3, ..., 1.
"""
from __future__ import annotations

import numpy as np

from .newton_db import MatmulCounter, block_scale


def chebyshev_fit(p: int, degree: int, a: float, b: float, n_points: int = 10000,
                  f=None) -> np.ndarray:
    """Coefficients c_0..c_d of sum_k c_k T_k(t) ~ f(x(t)) on [a, b], f(x) = x^(-1/p) (Appendix A.1).

    Discrete orthogonality of the Chebyshev polynomials at the N roots t_v = cos(theta_v) of T_N,
    theta_v = (v + 1/2) pi / N:  c = w * (T f) with the (d+1) x N matrix T[k, v] = T_k(t_v) = cos(k theta_v),
    f[v] = f(x(t_v)) and weights w_0 = 1/N, w_k = 2/N."""
    if f is None:
        def f(x):
            return np.power(x, -1.0 / p)
    theta = (np.arange(n_points, dtype=np.float64) + 0.5) * (np.pi / n_points)
    x = a + 0.5 * (b - a) * (1.0 + np.cos(theta))          # [-1, 1] -> [a, b]
    T = np.cos(np.outer(np.arange(degree + 1, dtype=np.float64), theta))
    w = np.full(degree + 1, 2.0 / n_points)
    w[0] = 1.0 / n_points
    return w * (T @ f(x))


def to_unit_interval(x, a: float, b: float):
    """Affine map [a, b] -> [-1, 1]."""
    return (2.0 * np.asarray(x, dtype=np.float64) - (a + b)) / (b - a)


def clenshaw_scalar(t, c: np.ndarray):
    """b_{d+2} = b_{d+1} = 0; b_k = 2 t b_{k+1} - b_{k+2} + c_k for k = d..0;
    value = b_0 - t b_1.  t is the mapped variable in [-1, 1]."""
    t = np.asarray(t, dtype=np.float64)
    d = len(c) - 1
    b2 = np.zeros_like(t)
    b1 = np.zeros_like(t)
    for k in range(d, -1, -1):
        b0 = 2.0 * t * b1 - b2 + c[k]
        b2, b1 = b1, b0
    # after the loop b1 holds b_0 and b2 holds b_1
    return b1 - t * b2


def clenshaw_matrix_plain(S: np.ndarray, c: np.ndarray, counter: MatmulCounter | None = None):
    """Matrix Clenshaw as first listed: B_{d+2} = B_{d+1} = 0,
    B_k = 2 S B_{k+1} - B_{k+2} + c_k I for k = d..0, result B_0 - S B_1
    (d+1 loop matmuls + 1 = d+2 matmuls)."""
    cnt = counter or MatmulCounter()
    n = S.shape[0]
    I = np.eye(n)
    d = len(c) - 1
    Bk2 = np.zeros((n, n))
    Bk1 = np.zeros((n, n))
    for k in range(d, -1, -1):
        Bk = 2.0 * cnt.mm(S, Bk1) - Bk2 + c[k] * I
        Bk2, Bk1 = Bk1, Bk
    return Bk1 - cnt.mm(S, Bk2)


def clenshaw_matrix_reduced(S: np.ndarray, c: np.ndarray, counter: MatmulCounter | None = None):
    """Reduced form: B_d = c_d I, B_{d-1} = 2 c_d S + c_{d-1} I set directly,
    B_k = 2 S B_{k+1} - B_{k+2} + c_k I for k = d-2..1, result S B_1 - B_2 + c_0 I
    (d-2 loop matmuls + 1 = d-1 matmuls).  Needs d >= 2."""
    cnt = counter or MatmulCounter()
    n = S.shape[0]
    I = np.eye(n)
    d = len(c) - 1
    if d < 2:
        raise ValueError("degree >= 2")
    Bk2 = c[d] * I                          # B_d
    Bk1 = 2.0 * c[d] * S + c[d - 1] * I     # B_{d-1}
    for k in range(d - 2, 0, -1):
        Bk = 2.0 * cnt.mm(S, Bk1) - Bk2 + c[k] * I
        Bk2, Bk1 = Bk1, Bk
    # Bk1 = B_1, Bk2 = B_2
    return cnt.mm(S, Bk1) - Bk2 + c[0] * I


def inverse_root_chebyshev(A, p: int, coeffs: np.ndarray, a: float, b: float,
                           eps: float = 0.0, scaling: str = "frobenius",
                           counter: MatmulCounter | None = None):
    """X_i ~ (A_i + eps I)^(-1/p): damp, scale by s, map the scaled block with the
    affine map of [a, b], evaluate the fitted series, un-scale by s^(-1/p).
    The coefficients must approximate x^(-1/p) for x = the scaled eigenvalues as seen
    through the map of [a, b]."""
    A = np.asarray(A, dtype=np.float64)
    single = A.ndim == 2
    if single:
        A = A[None]
    X = np.empty_like(A)
    eye = np.eye(A.shape[1])
    for i in range(A.shape[0]):
        Ad = A[i] + eps * eye
        s = block_scale(Ad, scaling)
        As = Ad / s
        S = (2.0 * As - (a + b) * eye) / (b - a)
        X[i] = clenshaw_matrix_reduced(S, coeffs, counter) * s ** (-1.0 / p)
    return X[0] if single else X


def inverse_root_chebyshev_model(A, p: int, coeffs: np.ndarray, a: float, b: float,
                                 eps: float = 0.0, scaling: str = "frobenius"):
    """Same result through the spectrum: Q diag(series(t(lam/s))) Q^T s^(-1/p)."""
    A = np.asarray(A, dtype=np.float64)
    single = A.ndim == 2
    if single:
        A = A[None]
    X = np.empty_like(A)
    eye = np.eye(A.shape[1])
    for i in range(A.shape[0]):
        Ad = 0.5 * (A[i] + A[i].T) + eps * eye
        s = block_scale(Ad, scaling)
        lam, Q = np.linalg.eigh(Ad)
        val = clenshaw_scalar(to_unit_interval(lam / s, a, b), coeffs)
        X[i] = (Q * (val * s ** (-1.0 / p))[None, :]) @ Q.T
    return X[0] if single else X
