"""Newton-Denman-Beavers coupled iteration (paper Section 3.3) and the scaling that
makes it converge (Section 3.4).

TEST INFRASTRUCTURE (see oracle/__init__.py).  float64 throughout, plain matmuls, the
paper's operand order, no blocking or fusion.

  Y_0 = A,  Z_0 = I
  E_{k-1} = (3 I - Z_{k-1} Y_{k-1}) / 2
  Y_k = Y_{k-1} E_{k-1},   Z_k = E_{k-1} Z_{k-1}
  Y_k -> A^{1/2},  Z_k -> A^{-1/2}     (needs ||I - A||_2 < 1)

Readings of points the paper leaves open (also listed in the design notes):
  * `iters` counts updates of (Y, Z); the closed-form first update counts as one.
  * for p = 4 the same `iters` is used for each of the two chained calls and the
    intermediate Y is not rescaled (for 0 < x <= 1 the scalar iterate y_k stays <= 1).
  * damping is applied before scaling: A_d = A + eps I, s = norm(A_d), A_s = A_d / s,
    and the result is un-scaled as X = s^{-1/p} (A_s)^{-1/p}.
"""
from __future__ import annotations

import numpy as np


class MatmulCounter:
    """Counts the B x B x B products an algorithm performs (for the paper's counts)."""

    def __init__(self):
        self.n = 0

    def mm(self, a, b):
        self.n += 1
        return a @ b


def ndb_plain(A: np.ndarray, iters: int, counter: MatmulCounter | None = None):
    """The iteration exactly as the three equations state it, from (Y_0, Z_0) = (A, I).
    3 matmuls per iteration.  Returns (Y_k, Z_k)."""
    c = counter or MatmulCounter()
    n = A.shape[0]
    I = np.eye(n)
    Y, Z = A.copy(), I.copy()
    for _ in range(iters):
        E = 0.5 * (3.0 * I - c.mm(Z, Y))
        Y, Z = c.mm(Y, E), c.mm(E, Z)
    return Y, Z


def ndb_shortcut(A: np.ndarray, iters: int, counter: MatmulCounter | None = None):
    """Same iterates, with the first iteration written in closed form (Section 3.3):
    E_1 = 3/2 I - 1/2 A, Y_1 = A E_1, Z_1 = E_1, i.e. 1 matmul instead of 3."""
    if iters < 1:
        raise ValueError("iters >= 1")
    c = counter or MatmulCounter()
    n = A.shape[0]
    I = np.eye(n)
    E = 1.5 * I - 0.5 * A
    Y, Z = c.mm(A, E), E
    for _ in range(iters - 1):
        E = 0.5 * (3.0 * I - c.mm(Z, Y))
        Y, Z = c.mm(Y, E), c.mm(E, Z)
    return Y, Z


def ndb_scalar(x, iters: int):
    """The iteration on scalars (every iterate is a polynomial in A, so on an
    eigenvalue x of A the matrices act as these numbers).  Returns (y_k, z_k)."""
    x = np.asarray(x, dtype=np.float64)
    y, z = x.copy(), np.ones_like(x)
    for _ in range(iters):
        e = 0.5 * (3.0 - z * y)
        y, z = y * e, e * z
    return y, z


def ndb_scalar_steps_to_tol(x: float, tol: float = 1e-10, max_iters: int = 200) -> int:
    """Number of iterations until |z_k - x^{-1/2}| <= tol and |y_k - x^{1/2}| <= tol
    (the experiment behind the paper's Figures 1 and 2)."""
    y, z = float(x), 1.0
    for k in range(1, max_iters + 1):
        e = 0.5 * (3.0 - z * y)
        y, z = y * e, e * z
        if abs(z - x ** -0.5) <= tol and abs(y - x ** 0.5) <= tol:
            return k
    return max_iters + 1


def block_scale(Ad: np.ndarray, scaling: str, pi=None) -> float:
    """s with lambda_max(A_d) <= s: Frobenius norm (Section 3.4) or trace (valid for SPD
    since lambda_max <= ||A||_F <= tr A); 'none' returns 1.  'power_iteration' is the
    paper's 2 * lambda_PI (Sections 3.4, 3.5) with pi = (V0, sweeps); it satisfies
    lambda_max < 2 s' only once lambda_PI > lambda_max / 2, which a few sweeps give."""
    if scaling == "frobenius":
        return float(np.sqrt((Ad * Ad).sum()))
    if scaling == "trace":
        return float(np.trace(Ad))
    if scaling == "none":
        return 1.0
    if scaling == "power_iteration":
        from .power_iteration import multi_power_iteration
        V0, sweeps = pi
        return 2.0 * multi_power_iteration(Ad, V0, sweeps)[0]
    raise ValueError(scaling)


def inverse_root_ndb(A, p: int, iters: int, eps: float = 0.0, scaling: str = "frobenius",
                     counter: MatmulCounter | None = None, pi=None):
    """X_i ~ (A_i + eps I)^(-1/p), p in {2,4}, by Newton-DB with `iters` updates per call.

    p=2: one call, keep Z.  p=4: first call keeps Y ~ A_s^{1/2}; a second call on that Y
    keeps Z ~ A_s^{-1/4} (Section 3.3, chaining).  Accepts (B,B) or (N,B,B)."""
    if p not in (2, 4):
        raise ValueError("Newton-DB gives only powers +-1/2^k; p must be 2 or 4")
    A = np.asarray(A, dtype=np.float64)
    single = A.ndim == 2
    if single:
        A = A[None]
    X = np.empty_like(A)
    eye = np.eye(A.shape[1])
    for i in range(A.shape[0]):
        Ad = A[i] + eps * eye
        s = block_scale(Ad, scaling, pi)
        As = Ad / s
        Y, Z = ndb_shortcut(As, iters, counter)
        if p == 4:
            _, Z = ndb_shortcut(Y, iters, counter)
        X[i] = Z * s ** (-1.0 / p)
    return X[0] if single else X


def inverse_root_ndb_model(A, p: int, iters: int, eps: float = 0.0, scaling: str = "frobenius", pi=None):
    """The same result predicted through the spectrum: with A_d = Q diag(lam) Q^T every
    iterate is Q diag(g(lam/s)) Q^T where g is the scalar recurrence.  Used to separate
    truncation error (finite `iters`) from rounding error."""
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
        y, z = ndb_scalar(lam / s, iters)
        if p == 4:
            _, z = ndb_scalar(y, iters)
        X[i] = (Q * (z * s ** (-1.0 / p))[None, :]) @ Q.T
    return X[0] if single else X


def ndb_truncation_error(lam, s: float, p: int, iters: int) -> float:
    """Relative Frobenius distance between the exact-arithmetic Newton-DB result and the
    true root, from the eigenvalues alone: both share Q, so the matrix error is the
    2-norm error over the eigenvalues."""
    lam = np.asarray(lam, dtype=np.float64)
    y, z = ndb_scalar(lam / s, iters)
    if p == 4:
        _, z = ndb_scalar(y, iters)
    approx = z * s ** (-1.0 / p)
    exact = lam ** (-1.0 / p)
    return float(np.linalg.norm(approx - exact) / np.linalg.norm(exact))
