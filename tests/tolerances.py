"""Stated tolerances of the fp32 path and the error metrics the parity tests share.

The rounding floor of fp32 Newton-DB (the distance between the fp32 iteration and the same iteration in
float64, once converged) is not fitted to the GPU kernel: tests/test_fp32_floor.py runs the iteration of
Section 3.3 on the CPU in float32 with every dot product accumulated strictly in k order (the order of one
matrix-core accumulator) and pins the law below on both sides.  The GPU tests import the bar from here."""
from __future__ import annotations

import numpy as np

FLOOR_MARGIN_FULL = 3.0        # bar / typical floor when every product is computed in full
FLOOR_MARGIN_SYMMETRIC = 4.0   # the mirrored residual product of symmetric mode costs up to 1.3x for kappa <= 1e4
# at kappa ~ 1e6 the mirrored residual doubles the floor of the inverse 4th root (CPU float32: 2.2x); tests that
# run such blocks hold symmetric mode to this multiple of the full-products error instead
SYMMETRIC_OVER_FULL_ILLCONDITIONED = 2.5


def fp32_floor_typical(kappa: float, p: int, B: int = 256) -> float:
    """Typical converged distance of fp32 Newton-DB (full products, Frobenius scaling) to the float64 iteration:
    0.085 kappa 2^-24 at B <= 256 -- the coupled iteration amplifies a rounding perturbation by about the
    condition number of the scaled block -- growing like (B/256)^0.75 with the length of the sequentially
    accumulated fp32 dot products, 2.5 times that for the inverse square root; never below 1e-6."""
    base = max(1e-6, 0.085 * kappa * 2.0 ** -24)
    return base * max(1.0, B / 256.0) ** 0.75 * (2.5 if p == 2 else 1.0)


def fp32_floor(kappa: float, p: int, B: int = 256, symmetric: bool = True) -> float:
    """The bar: typical floor times the stated margin (3 with full products, 4 in symmetric mode)."""
    return (FLOOR_MARGIN_SYMMETRIC if symmetric else FLOOR_MARGIN_FULL) * fp32_floor_typical(kappa, p, B)


def clenshaw_fp32_floor_typical(d: int, p: int, B: int = 256) -> float:
    """Typical distance of the fp32 Clenshaw recurrence (Appendix A.2, reduced form) to the same recurrence in
    float64 on spectra spread over four decades (interval [lambda_min/s, 1]): every step adds the rounding of
    one product and the recurrence carries it on, which measures as d^1.5; sqrt(B/256) for the dot products;
    1.7 times more for the inverse square root.  Better-conditioned blocks stay below it."""
    return 0.7e-7 * d ** 1.5 * max(1.0, B / 256.0) ** 0.5 * (1.7 if p == 2 else 1.0)


def clenshaw_fp32_floor(d: int, p: int, B: int = 256) -> float:
    """The bar: three times the typical value (pinned on the CPU in tests/test_fp32_floor.py)."""
    return 3.0 * clenshaw_fp32_floor_typical(d, p, B)


def max_abs_bar(frobenius_bar: float) -> float:
    """Bar for rel_max_abs_error that goes with a relative-Frobenius bar e.  The entries of a rounding-error matrix
    D are spread evenly, so the largest of the B^2 of them is about sqrt(2 ln B^2) = 4.4 .. 5.5 times their rms
    ||D||_F / B (B = 128 .. 2048); with ||X||_F <= B ||X||_max that gives max|D| / ||X||_max <= 5.5 e, and less
    when X is far from flat.  5 e is used: a deviation that is NOT spread evenly (one wrong entry, row or tile)
    exceeds it long before it shows in the Frobenius ratio."""
    return 5.0 * frobenius_bar


def rel_max_abs_error(X, X_ref) -> np.ndarray:
    """Per-block max_ij |X - X_ref| / max_ij |X_ref|: unlike the Frobenius ratio it sees a single wrong entry
    in a low-energy region of a block (an entry off by d moves it by d / ||X_ref||_max, the Frobenius ratio only
    by d / ||X_ref||_F, a factor sqrt(B) to B less)."""
    X = np.asarray(X, dtype=np.float64)
    X_ref = np.asarray(X_ref, dtype=np.float64)
    if X.ndim == 2:
        X, X_ref = X[None], X_ref[None]
    return np.abs(X - X_ref).max(axis=(1, 2)) / np.abs(X_ref).max(axis=(1, 2))
