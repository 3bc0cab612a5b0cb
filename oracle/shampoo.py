"""Shampoo step on stacked blocks (paper Algorithm 1, Section 4, Section 2.3 grafting).

TEST INFRASTRUCTURE (see oracle/__init__.py).  float64 throughout.

Every gradient block G_i (B x B) owns one left factor L_i and one right factor R_i
(Section 4.1: "block(G)", products taken with the last two dimensions transposed).
"""
from __future__ import annotations

import numpy as np

from .evd import inverse_root_evd


def accumulate_factors(G, L, R, beta: float, alpha: float | None = None):
    """Algorithm 1, the two EMA lines:
         L_i <- beta L_i + alpha G_i G_i^T ,   R_i <- beta R_i + alpha G_i^T G_i
    with alpha = 1 - beta unless given.  Returns new (L, R); inputs are not modified."""
    if alpha is None:
        alpha = 1.0 - beta
    G = np.asarray(G, dtype=np.float64)
    L = np.asarray(L, dtype=np.float64)
    R = np.asarray(R, dtype=np.float64)
    Gt = np.swapaxes(G, -1, -2)
    L_new = beta * L + alpha * np.matmul(G, Gt)
    R_new = beta * R + alpha * np.matmul(Gt, G)
    return L_new, R_new


def precondition(Linv, G, Rinv):
    """Algorithm 1, update direction: U_i = Linv_i G_i Rinv_i."""
    Linv = np.asarray(Linv, dtype=np.float64)
    G = np.asarray(G, dtype=np.float64)
    Rinv = np.asarray(Rinv, dtype=np.float64)
    return np.matmul(np.matmul(Linv, G), Rinv)


def adam_graft(G, U, Acc, beta_g: float, eps_g: float):
    """Block-wise Adam grafting (Section 2.3).

    Acc <- beta_g Acc + (1-beta_g) G*G (elementwise); P = G / (eps_g + sqrt(Acc));
    s_i = ||P_i||_F / ||U_i||_F per block.  Returns (Acc_new, s) with s of shape (N,).
    The parameter update is then theta <- theta - eta * s_i * U_i.
    Section 2.3 is silent on a block whose update U_i is all zero (a block that saw no gradient):
    reading s_i = 0 there -- the update is zero whatever s_i is, and 0/0 would poison theta.
    """
    G = np.asarray(G, dtype=np.float64)
    U = np.asarray(U, dtype=np.float64)
    Acc = np.asarray(Acc, dtype=np.float64)
    Acc_new = beta_g * Acc + (1.0 - beta_g) * G * G
    P = G / (eps_g + np.sqrt(Acc_new))
    nP = np.sqrt((P * P).sum(axis=(-1, -2)))
    nU = np.sqrt((U * U).sum(axis=(-1, -2)))
    s = np.divide(nP, nU, out=np.zeros_like(nP), where=nU > 0.0)
    return Acc_new, s


def step(G, L, R, beta: float, eps: float, p: int = 4, alpha: float | None = None,
         inverse_root=None, graft=None, theta=None, lr: float = 0.0):
    """One step of Algorithm 1 on a stack: accumulate -> roots of the damped factors ->
    precondition (-> grafted parameter update).

    inverse_root(S, p, eps) defaults to the eigendecomposition root.  It is applied once
    to the stack S = [L; R] of 2N blocks (Section 4.1, the stack operator).

    graft = dict(Acc=..., beta_g=..., eps_g=...) switches the grafted update on; then
    theta (N,B,B) is updated with learning rate lr.

    Returns dict(L, R, X_L, X_R, U, and with grafting: Acc, s, theta).
    """
    if inverse_root is None:
        inverse_root = inverse_root_evd
    L1, R1 = accumulate_factors(G, L, R, beta, alpha)
    N = L1.shape[0]
    S = np.concatenate([L1, R1], axis=0)
    X = inverse_root(S, p, eps)
    XL, XR = X[:N], X[N:]
    U = precondition(XL, G, XR)
    out = dict(L=L1, R=R1, X_L=XL, X_R=XR, U=U)
    if graft is not None:
        Acc_new, s = adam_graft(G, U, graft["Acc"], graft["beta_g"], graft["eps_g"])
        out["Acc"] = Acc_new
        out["s"] = s
        if theta is not None:
            out["theta"] = np.asarray(theta, dtype=np.float64) - lr * s[:, None, None] * U
    return out
