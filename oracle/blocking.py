"""block(), stack() and their inverses for one layer (paper Section 4.1), and the 1-D
(normalisation layer) variant of the Shampoo step.

TEST INFRASTRUCTURE (see oracle/__init__.py).

A layer W of shape (m, n) is cut by a grid of pitch B into full blocks (B, B) and, where m
or n is not a multiple of B, smaller "rest" blocks: the last m mod B rows give blocks of
shape (m mod B, B), the last n mod B columns blocks of shape (B, n mod B), and both at once
one corner block.  Within a group blocks are numbered row by row of the grid.  (The paper
fixes the shapes and counts -- pinned by its worked example -- but not the numbering; any
fixed numbering gives the same optimizer step because every block is treated alone.)

Written with explicit loops over the grid so that it can be checked by eye.
"""
from __future__ import annotations

import numpy as np

from .evd import inverse_root_evd


def block_layer(W, B: int) -> dict:
    W = np.asarray(W)
    m, n = W.shape
    Nm, Nn, rm, rn = m // B, n // B, m % B, n % B
    full = np.zeros((Nm * Nn, B, B), dtype=W.dtype)
    row_rest = np.zeros((Nn if rm else 0, rm, B), dtype=W.dtype)
    col_rest = np.zeros((Nm if rn else 0, B, rn), dtype=W.dtype)
    corner = np.zeros((1 if rm and rn else 0, rm, rn), dtype=W.dtype)
    for i in range(Nm):
        for j in range(Nn):
            full[i * Nn + j] = W[i * B:(i + 1) * B, j * B:(j + 1) * B]
    if rm:
        for j in range(Nn):
            row_rest[j] = W[Nm * B:, j * B:(j + 1) * B]
    if rn:
        for i in range(Nm):
            col_rest[i] = W[i * B:(i + 1) * B, Nn * B:]
    if rm and rn:
        corner[0] = W[Nm * B:, Nn * B:]
    return dict(full=full, row_rest=row_rest, col_rest=col_rest, corner=corner)


def unblock_layer(groups: dict, m: int, n: int, B: int) -> np.ndarray:
    Nm, Nn, rm, rn = m // B, n // B, m % B, n % B
    W = np.zeros((m, n), dtype=groups["full"].dtype)
    for i in range(Nm):
        for j in range(Nn):
            W[i * B:(i + 1) * B, j * B:(j + 1) * B] = groups["full"][i * Nn + j]
    if rm:
        for j in range(Nn):
            W[Nm * B:, j * B:(j + 1) * B] = groups["row_rest"][j]
    if rn:
        for i in range(Nm):
            W[i * B:(i + 1) * B, Nn * B:] = groups["col_rest"][i]
    if rm and rn:
        W[Nm * B:, Nn * B:] = groups["corner"][0]
    return W


def stack_shapes(m: int, n: int, B: int) -> dict:
    """Shapes of G, L, R per group and of the stacked factor tensors S_full (every B x B factor) and
    S_rest (the smaller ones), as in the worked example of Section 4.1."""
    Nm, Nn, rm, rn = m // B, n // B, m % B, n % B
    g = dict(G_full=(Nm * Nn, B, B), L_full=(Nm * Nn, B, B), R_full=(Nm * Nn, B, B))
    n_big = 2 * Nm * Nn
    rest = []
    if rm:
        g.update(G_row_rest=(Nn, rm, B), L_row_rest=(Nn, rm, rm), R_row_rest=(Nn, B, B))
        n_big += Nn
        rest.append((Nn, rm, rm))
    if rn:
        g.update(G_col_rest=(Nm, B, rn), L_col_rest=(Nm, B, B), R_col_rest=(Nm, rn, rn))
        n_big += Nm
        rest.append((Nm, rn, rn))
    if rm and rn:
        g.update(G_corner=(1, rm, rn), L_corner=(1, rm, rm), R_corner=(1, rn, rn))
        rest += [(1, rm, rm), (1, rn, rn)]
    g["S_full"] = (n_big, B, B)
    g["S_rest"] = rest
    return g


def layer_step(W_grad, factors: dict | None, B: int, beta: float, eps: float, p: int = 4,
               alpha: float | None = None, inverse_root=None):
    """One Shampoo step (Algorithm 1) of a whole (m, n) layer, block by block straight on slices of
    the layer gradient: for the block at rows r0:r1, columns c0:c1
        L <- beta L + alpha G G^T, R <- beta R + alpha G^T G, U = (L+eps I)^(-1/p) G (R+eps I)^(-1/p).
    factors maps (r0, c0) -> (L, R) (missing = zeros).  Returns (U of shape (m, n), new factors)."""
    if alpha is None:
        alpha = 1.0 - beta
    if inverse_root is None:
        inverse_root = inverse_root_evd
    G = np.asarray(W_grad, dtype=np.float64)
    m, n = G.shape
    U = np.zeros_like(G)
    new = {}
    for r0 in range(0, m, B):
        for c0 in range(0, n, B):
            Gb = G[r0:min(r0 + B, m), c0:min(c0 + B, n)]
            L, R = (factors or {}).get((r0, c0), (np.zeros((Gb.shape[0],) * 2), np.zeros((Gb.shape[1],) * 2)))
            L = beta * L + alpha * Gb @ Gb.T
            R = beta * R + alpha * Gb.T @ Gb
            new[(r0, c0)] = (L, R)
            U[r0:r0 + Gb.shape[0], c0:c0 + Gb.shape[1]] = inverse_root(L, p, eps) @ Gb @ inverse_root(R, p, eps)
    return U, new


def layer_step_cached(W_grad, factors, roots, B: int, beta: float, eps: float, p: int = 4, alpha: float | None = None,
                      refresh: bool = True, inverse_root=None):
    """layer_step with the paper's recomputation frequency (Section 4.1, f > 1): the factors are updated
    at every step, the inverse roots only when `refresh` is true; otherwise the roots of the last refresh
    (`roots`: (r0, c0) -> (X_L, X_R)) precondition the new gradient.  Returns (U, factors, roots)."""
    if alpha is None:
        alpha = 1.0 - beta
    if inverse_root is None:
        inverse_root = inverse_root_evd
    G = np.asarray(W_grad, dtype=np.float64)
    m, n = G.shape
    U = np.zeros_like(G)
    new_f, new_r = {}, {}
    for r0 in range(0, m, B):
        for c0 in range(0, n, B):
            Gb = G[r0:min(r0 + B, m), c0:min(c0 + B, n)]
            L, R = (factors or {}).get((r0, c0), (np.zeros((Gb.shape[0],) * 2), np.zeros((Gb.shape[1],) * 2)))
            L = beta * L + alpha * Gb @ Gb.T
            R = beta * R + alpha * Gb.T @ Gb
            new_f[(r0, c0)] = (L, R)
            new_r[(r0, c0)] = (inverse_root(L, p, eps), inverse_root(R, p, eps)) if refresh else roots[(r0, c0)]
            XL, XR = new_r[(r0, c0)]
            U[r0:r0 + Gb.shape[0], c0:c0 + Gb.shape[1]] = XL @ Gb @ XR
    return U, new_f, new_r


def vector_param_step_cached(grad, factors, roots, B: int, beta: float, eps: float, p: int = 2,
                             alpha: float | None = None, refresh: bool = True, inverse_root=None):
    """One 1-D parameter of E entries: pieces of B entries (and one of E mod B), each with a left factor
    only: L <- beta L + alpha g g^T, u = (L + eps I)^(-1/p) g (roots as in layer_step_cached).
    factors, roots: lists per piece (None = zeros / nothing cached).  Returns (u, factors, roots)."""
    if alpha is None:
        alpha = 1.0 - beta
    if inverse_root is None:
        inverse_root = inverse_root_evd
    g = np.asarray(grad, dtype=np.float64)
    E = g.shape[0]
    u = np.zeros_like(g)
    new_f, new_r = [], []
    for j, a in enumerate(range(0, E, B)):
        gj = g[a:min(a + B, E)]
        L = factors[j] if factors else np.zeros((gj.shape[0],) * 2)
        L = beta * L + alpha * np.outer(gj, gj)
        new_f.append(L)
        new_r.append(inverse_root(L, p, eps) if refresh else roots[j])
        u[a:a + gj.shape[0]] = new_r[j] @ gj
    return u, new_f, new_r


def graft_layer(G, U, Acc, B: int, beta_g: float, eps_g: float):
    """Block-wise Adam grafting (Section 2.3) of one layer (2-D, or 1-D cut into pieces of B): the
    second-moment accumulator is elementwise over the layer, Acc <- beta_g Acc + (1-beta_g) G*G,
    P = G / (eps_g + sqrt(Acc)), and every block b of the grid gets s_b = ||P_b||_F / ||U_b||_F and
    U_b <- s_b U_b.  Returns (U_grafted, Acc_new)."""
    G = np.asarray(G, dtype=np.float64)
    U = np.asarray(U, dtype=np.float64)
    Acc = beta_g * np.asarray(Acc, dtype=np.float64) + (1.0 - beta_g) * G * G
    P = G / (eps_g + np.sqrt(Acc))
    out = np.zeros_like(U)
    if G.ndim == 1:
        for a in range(0, G.shape[0], B):
            sl = slice(a, min(a + B, G.shape[0]))
            out[sl] = U[sl] * (np.linalg.norm(P[sl]) / np.linalg.norm(U[sl]))
        return out, Acc
    m, n = G.shape
    for r0 in range(0, m, B):
        for c0 in range(0, n, B):
            sl = (slice(r0, min(r0 + B, m)), slice(c0, min(c0 + B, n)))
            out[sl] = U[sl] * (np.linalg.norm(P[sl]) / np.linalg.norm(U[sl]))
    return out, Acc


# ---- normalisation layers (Section 4.1): vectors as B x 1 blocks, left factor only, p = 2 ----
def accumulate_vector(g, L, beta: float, alpha: float | None = None):
    """L_i <- beta L_i + alpha g_i g_i^T for g of shape (N, B)."""
    if alpha is None:
        alpha = 1.0 - beta
    g = np.asarray(g, dtype=np.float64)
    L = np.asarray(L, dtype=np.float64)
    out = np.empty_like(L)
    for i in range(g.shape[0]):
        out[i] = beta * L[i] + alpha * np.outer(g[i], g[i])
    return out


def precondition_vector(Linv, g):
    """u_i = Linv_i g_i."""
    Linv = np.asarray(Linv, dtype=np.float64)
    g = np.asarray(g, dtype=np.float64)
    return np.stack([Linv[i] @ g[i] for i in range(g.shape[0])]) if g.shape[0] else np.zeros_like(g)


def norm_layers_step(grads, L, B: int, beta: float, eps: float, alpha: float | None = None, inverse_root=None):
    """N normalisation layers of size E stacked to (N, E), cut into (N*E/B) vectors of B entries:
    L <- beta L + alpha g g^T, u = (L + eps I)^(-1/2) g, u reshaped back to (N, E).
    Returns (U (N, E), L_new (N*E/B, B, B))."""
    if inverse_root is None:
        inverse_root = inverse_root_evd
    grads = np.asarray(grads, dtype=np.float64)
    N, E = grads.shape
    assert E % B == 0
    g = grads.reshape(N * (E // B), B)
    L_new = accumulate_vector(g, L, beta, alpha)
    u = precondition_vector(inverse_root(L_new, 2, eps), g)
    return u.reshape(N, E), L_new
