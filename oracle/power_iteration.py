"""Multi-Power-Iteration estimate of the largest eigenvalue (paper Sections 3.4 and 3.5).

TEST INFRASTRUCTURE (see oracle/__init__.py).  float64, numpy only.

The paper fixes: the estimate is the Rayleigh quotient R_A(v) = v^T A v / v^T v of the
Power-Iteration vector (Section 3.4); a pool of 16 or 32 start vectors is iterated in
parallel and the largest Rayleigh quotient is kept (Section 3.5); the block is then divided
by 2 * lambda_PI, because lambda_PI <= lambda_max (Section 3.4).  It does not fix the number
of iterations, the normalisation, or how the start vectors are drawn.  Reading used here
(listed in the design notes):

  V_0  = the given start vectors (B x m), each column scaled to unit length
  for t = 1 .. sweeps:        W = (A + eps I) V_{t-1}
                               q_j = v_j . w_j                (Rayleigh quotient, ||v_j|| = 1)
                               V_t = W with every column scaled to unit length
  lambda_PI = max_j q_j of the last sweep,    s = 2 * lambda_PI

so `sweeps` passes over A give the Rayleigh quotients of the vectors after sweeps-1
multiplications.  The start vectors are an input (random numbers are drawn by the caller).
"""
from __future__ import annotations

import numpy as np


def rayleigh_quotient(A: np.ndarray, v: np.ndarray) -> float:
    return float(v @ (A @ v) / (v @ v))


def multi_power_iteration(A: np.ndarray, V0: np.ndarray, sweeps: int, eps: float = 0.0):
    """Returns (lambda_PI, q) for one block: q holds the pool's Rayleigh quotients of the
    last sweep, lambda_PI = max(q)."""
    if sweeps < 1:
        raise ValueError("sweeps >= 1")
    A = np.asarray(A, dtype=np.float64)
    V = np.asarray(V0, dtype=np.float64).copy()
    V /= np.sqrt((V * V).sum(axis=0, keepdims=True))
    q = None
    for _ in range(sweeps):
        W = A @ V + eps * V
        q = (V * W).sum(axis=0)
        V = W / np.sqrt((W * W).sum(axis=0, keepdims=True))
    return float(q.max()), q


def power_iteration_scale(A, V0: np.ndarray, sweeps: int, eps: float = 0.0) -> np.ndarray:
    """s_i = 2 * lambda_PI(A_i + eps I) for a block (B,B) or a stack (N,B,B)."""
    A = np.asarray(A, dtype=np.float64)
    if A.ndim == 2:
        return np.array(2.0 * multi_power_iteration(A, V0, sweeps, eps)[0])
    return np.array([2.0 * multi_power_iteration(A[i], V0, sweeps, eps)[0] for i in range(A.shape[0])])
