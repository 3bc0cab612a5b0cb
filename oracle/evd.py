"""Inverse p-th root by eigendecomposition (paper Section 3.1, "EVD").

TEST INFRASTRUCTURE (see oracle/__init__.py).

For symmetric A = Q diag(lam) Q^T the matrix power is A^r = Q diag(lam^r) Q^T.  With the
damping of Algorithm 1 the quantity wanted is (A + eps I)^(-1/p), the principal root,
which is unique for a symmetric positive definite argument.
"""
from __future__ import annotations

import numpy as np


def inverse_root_evd(A: np.ndarray, p: int, eps: float = 0.0) -> np.ndarray:
    """X_i = (sym(A_i) + eps I)^(-1/p) for one block (B,B) or a stack (N,B,B), float64.

    sym(A) = (A + A^T)/2 removes any rounding-level asymmetry of the input before the
    symmetric eigensolver sees it.  Raises if a damped block is not positive definite
    (the paper's remark that a single failed block ends training, Appendix B.1).
    """
    A = np.asarray(A, dtype=np.float64)
    single = A.ndim == 2
    if single:
        A = A[None]
    N, B, B2 = A.shape
    assert B == B2
    X = np.empty_like(A)
    eye = np.eye(B)
    for i in range(N):
        Ad = 0.5 * (A[i] + A[i].T) + eps * eye
        lam, Q = np.linalg.eigh(Ad)
        if not np.all(np.isfinite(lam)) or lam.min() <= 0.0:
            raise ValueError(f"block {i}: damped matrix is not positive definite "
                             f"(lambda_min={lam.min():.3e})")
        X[i] = (Q * np.power(lam, -1.0 / p)[None, :]) @ Q.T
    return X[0] if single else X


def rel_frobenius_error(X: np.ndarray, X_ref: np.ndarray) -> np.ndarray:
    """Per-block ||X - X_ref||_F / ||X_ref||_F (the parity metric the benchmark spec states)."""
    X = np.asarray(X, dtype=np.float64)
    X_ref = np.asarray(X_ref, dtype=np.float64)
    if X.ndim == 2:
        X, X_ref = X[None], X_ref[None]
    num = np.sqrt(((X - X_ref) ** 2).sum(axis=(1, 2)))
    den = np.sqrt((X_ref ** 2).sum(axis=(1, 2)))
    return num / den
