"""Seeded synthetic inputs for the block-diagonal Shampoo hot path.

This module only *draws inputs*: random gradients and SPD blocks assembled from a
chosen orthogonal factor and a chosen spectrum.  It holds none of the optimizer's
arithmetic (no factor accumulation, no roots, no preconditioning) so that the CPU
oracle and the HIP path can both take their inputs from here without sharing any
code of the method itself.

Shapes follow the paper's stacked-block layout (Section 4, "Blocking Strategy in
DASH"): a gradient of shape (m, n) with m, n divisible by B becomes
block(G) of shape (N, B, B), N = (m/B)*(n/B), and every Kronecker factor is a
B x B block of an (N, B, B) stack.
"""
from __future__ import annotations

import numpy as np

# ---------------------------------------------------------------------------
# spectra and orthogonal factors
# ---------------------------------------------------------------------------


def log_uniform_spectrum(B: int, lo_exp: float, hi_exp: float, seed: int) -> np.ndarray:
    """B eigenvalues 10**u with u ~ U(lo_exp, hi_exp); the two extremes are forced to
    10**lo_exp and 10**hi_exp so the condition number is exactly 10**(hi_exp-lo_exp).
    Returned in float64, unsorted (position j belongs to column j of Q)."""
    rng = np.random.default_rng(seed)
    u = rng.uniform(lo_exp, hi_exp, size=B)
    if B >= 2:
        u[0] = lo_exp
        u[1] = hi_exp
    return np.power(10.0, u)


def orthogonal_factor(B: int, seed: int) -> np.ndarray:
    """Q factor of the QR decomposition of a seeded N(0,1) B x B matrix, with the
    column signs fixed so that diag(R) > 0 (which makes Q unique)."""
    rng = np.random.default_rng(seed)
    M = rng.standard_normal((B, B))
    Q, R = np.linalg.qr(M)
    sgn = np.sign(np.diag(R))
    sgn[sgn == 0] = 1.0
    return Q * sgn[None, :]


def spd_from_spectrum(Q: np.ndarray, lam: np.ndarray) -> np.ndarray:
    """A = Q diag(lam) Q^T in float64, symmetrised exactly."""
    A = (Q * lam[None, :]) @ Q.T
    return 0.5 * (A + A.T)


def spd_stack(N: int, B: int, lo_exp: float, hi_exp: float, seed: int,
              share_q: bool = False):
    """Stack of N SPD blocks with known eigen-structure.

    Block i uses Q from seed 1000+seed*100003+i (or one shared Q when share_q) and a
    log-uniform spectrum from seed 2000+seed*100003+i.

    Returns (A32, Q, lam): A32 is the float32 (N,B,B) stack the GPU receives, Q is
    (N,B,B) or (1,B,B) float64, lam is (N,B) float64.  The float32 rounding is applied
    to the already symmetric float64 matrix, so A32 is bit-symmetric.
    """
    base = seed * 100003
    A32 = np.empty((N, B, B), dtype=np.float32)
    lam = np.empty((N, B), dtype=np.float64)
    nq = 1 if share_q else N
    Qs = np.empty((nq, B, B), dtype=np.float64)
    for i in range(nq):
        Qs[i] = orthogonal_factor(B, 1000 + base + i)
    for i in range(N):
        lam[i] = log_uniform_spectrum(B, lo_exp, hi_exp, 2000 + base + i)
        A32[i] = spd_from_spectrum(Qs[0 if share_q else i], lam[i]).astype(np.float32)
    return A32, Qs, lam


# ---------------------------------------------------------------------------
# gradients
# ---------------------------------------------------------------------------


def gradient_stack(N: int, B: int, seed: int, std: float = 1e-2) -> np.ndarray:
    """block(G): (N,B,B) float32, entries N(0, std^2)."""
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((N, B, B)) * std).astype(np.float32)


def blocks_of_layer(m: int, n: int, B: int) -> int:
    """Number of full B x B gradient blocks of an (m, n) layer (m, n divisible by B)."""
    if m % B or n % B:
        raise ValueError("this helper counts the full B x B blocks of a layer whose dims are multiples of B; "
                         "ragged layers go through the library's block() (dash_block_layer)")
    return (m // B) * (n // B)


# ---------------------------------------------------------------------------
# the five benchmark configurations
# ---------------------------------------------------------------------------

CFG1 = dict(name="cfg1_small_root", N=16, B=128, lo_exp=-3.0, hi_exp=0.0, seed=1,
            p=4, ndb_iters=10, cheb_degree=16)

CFG2 = dict(name="cfg2_layer4096_step", m=4096, n=4096, B=1024, beta=0.95, eps=1e-6,
            p=4, ndb_iters=10, warm_steps=20, grad_std=1e-2, seed_base=3000)

CFG3 = dict(name="cfg3_decoder24_stack", layers=24, d=2048, ffn=8192, B=1024,
            beta=0.95, eps=1e-6, p=4, ndb_iters=10, grad_std=1e-2, seed_base=5000)

CFG4 = dict(name="cfg4_sweep", shapes=[(256, 256), (512, 64), (2048, 4)],
            lo_exp=-4.0, hi_exp=0.0, ndb_iters=[5, 10, 20], cheb_degrees=[8, 16, 32],
            ps=[2, 4], seed=4)

CFG5 = dict(name="cfg5_illcond_bf16", N=1024, B=1024, lo_exp=-8.0, hi_exp=0.0,
            eps=1e-6, p=4, iters=[5, 10, 15, 20, 25, 30, 40], seed=5)


def cfg2_num_blocks() -> int:
    return blocks_of_layer(CFG2["m"], CFG2["n"], CFG2["B"])


def cfg3_num_gradient_blocks() -> int:
    c = CFG3
    per_layer = 4 * blocks_of_layer(c["d"], c["d"], c["B"]) + 3 * blocks_of_layer(c["d"], c["ffn"], c["B"])
    return c["layers"] * per_layer


# ---------------------------------------------------------------------------
# start vectors of the multi-Power-Iteration pool (random numbers the method draws)
# ---------------------------------------------------------------------------


def start_vectors(B: int, m: int, seed: int) -> np.ndarray:
    """(B, m) float32 N(0,1) start vectors, one column per pool member."""
    rng = np.random.default_rng(seed)
    return rng.standard_normal((B, m)).astype(np.float32)
