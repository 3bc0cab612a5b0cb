"""Pins the fp32 rounding floor of Newton-DB (tests/tolerances.py) on the CPU, independently of the GPU kernel.

The iteration of Section 3.3 (closed-form first update, full products, the paper's operand order) runs in
float32 with every product done by tests/host/seq_sgemm.c: each output element is accumulated over k strictly in
order with one fused multiply-add per term, the summation order of a single matrix-core accumulator (a blocked
BLAS sgemm sums partial blocks and shows a weaker growth with B).  The result is compared with the same
iteration in float64 (oracle), so only rounding is measured."""
import ctypes
import os
import shutil
import subprocess

import numpy as np
import pytest

import workloads
from oracle import newton_db as ondb
from oracle import chebyshev as ocheb
from tolerances import (SYMMETRIC_OVER_FULL_ILLCONDITIONED, clenshaw_fp32_floor, clenshaw_fp32_floor_typical,
                        fp32_floor, fp32_floor_typical, max_abs_bar)

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def mm(tmp_path_factory):
    if shutil.which("gcc") is None:
        pytest.skip("gcc not available")
    so = tmp_path_factory.mktemp("seq") / "seq_sgemm.so"
    subprocess.run(["gcc", "-O3", "-march=native", "-fopenmp", "-shared", "-fPIC", "-o", str(so),
                    os.path.join(ROOT, "tests", "host", "seq_sgemm.c"), "-lm"], check=True)
    lib = ctypes.CDLL(str(so))
    lib.seq_sgemm.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int]

    def product(a, b, upper=False):
        a = np.ascontiguousarray(a, dtype=np.float32)
        b = np.ascontiguousarray(b, dtype=np.float32)
        c = np.empty_like(a)
        lib.seq_sgemm(a.shape[0], a.ctypes.data, b.ctypes.data, c.ctypes.data, 1 if upper else 0)
        return c
    return product


def test_sequential_product_is_a_product(mm):
    rng = np.random.default_rng(0)
    a, b = rng.standard_normal((96, 96)).astype(np.float32), rng.standard_normal((96, 96)).astype(np.float32)
    ref = a.astype(np.float64) @ b.astype(np.float64)
    assert np.abs(mm(a, b) - ref).max() < 1e-4
    s = (a + a.T).astype(np.float32)
    up = mm(s, s, upper=True)                       # S S is symmetric: mirrored upper triangle = full product
    assert np.array_equal(up, up.T) and np.abs(up - s.astype(np.float64) @ s.astype(np.float64)).max() < 1e-3


def _ndb_float32(mm, As, iters, symmetric):
    """Section 3.3 in float32: E_1 = 3/2 I - 1/2 A, Y_1 = A E_1, Z_1 = E_1, then E = 3/2 I - 1/2 Z Y,
    Y <- Y E, Z <- E Z.  symmetric: the residual Z Y is computed on its upper triangle and mirrored."""
    I = np.eye(As.shape[0], dtype=np.float32)
    E = np.float32(1.5) * I - np.float32(0.5) * As
    Y, Z = mm(As, E), E
    for _ in range(iters - 1):
        E = np.float32(1.5) * I - np.float32(0.5) * mm(Z, Y, upper=symmetric)
        Y, Z = mm(Y, E), mm(E, Z)
    return Y, Z


def _floors(mm, B, lo_exp, k, p, eps):
    """(full-products, symmetric-mode) distance of the float32 iteration to the float64 iteration of the oracle."""
    A32, _, _ = workloads.spd_stack(1, B, lo_exp, 0.0, seed=7, share_q=True)
    A = A32[0].astype(np.float64)
    X64 = ondb.inverse_root_ndb(A, p, k, eps=eps)
    Ad = A + eps * np.eye(B)
    s = np.sqrt((Ad * Ad).sum())
    As = (Ad / s).astype(np.float32)
    out = []
    for symmetric in (False, True):
        Y, Z = _ndb_float32(mm, As, k, symmetric)
        if p == 4:
            _, Z = _ndb_float32(mm, Y, k, symmetric)
        X32 = Z.astype(np.float64) * s ** (-1.0 / p)
        out.append(float(np.linalg.norm(X32 - X64) / np.linalg.norm(X64)))
    return out


# kappa = 1e4 at the block sizes of the sweep configuration, kappa = 1e3 at the small one; 20 (15) updates per
# call are past convergence, so what is left is rounding
@pytest.mark.parametrize("B,lo_exp,k,p", [(128, -3.0, 15, 4), (128, -3.0, 15, 2), (256, -4.0, 20, 4), (256, -4.0, 20, 2),
                                          (512, -4.0, 20, 4), (1024, -4.0, 20, 4), (1024, -4.0, 20, 2),
                                          (2048, -4.0, 20, 4)])
def test_floor_law_holds_on_the_cpu(mm, B, lo_exp, k, p):
    kappa = 10.0 ** (-lo_exp)
    full, sym = _floors(mm, B, lo_exp, k, p, 0.0)
    typ = fp32_floor_typical(kappa, p, B)
    print(f"B={B} kappa={kappa:.0e} p={p}: float32 floor full {full:.2e} symmetric {sym:.2e}; law {typ:.2e}, "
          f"bars {fp32_floor(kappa, p, B, False):.2e} / {fp32_floor(kappa, p, B, True):.2e}", flush=True)
    # the law is the typical value, on both sides: a law without the growth in B, or with linear growth, fails
    assert typ / 2.0 <= full <= 2.0 * typ
    # and the bars the GPU tests use keep a margin over what the arithmetic itself does
    assert full <= fp32_floor(kappa, p, B, symmetric=False) / 1.5
    assert sym <= fp32_floor(kappa, p, B, symmetric=True) / 1.5
    assert sym <= 1.4 * full          # mirroring the residual costs little on these spectra


def test_growth_with_block_size(mm):
    """The (B/256)^0.75 factor: measured growth from B = 256 to 1024 at kappa = 1e4 (p = 2: half the products)."""
    f256, _ = _floors(mm, 256, -4.0, 20, 2, 0.0)
    f1024, _ = _floors(mm, 1024, -4.0, 20, 2, 0.0)
    growth = f1024 / f256
    print(f"floor growth 256 -> 1024: {growth:.2f} (law {4 ** 0.75:.2f}, sqrt law 2.00, no growth 1.00)", flush=True)
    assert 2.2 <= growth <= 3.6


def test_illconditioned_floor_and_the_cost_of_symmetric_mode(mm):
    """The ill-conditioned configuration: spectrum in [1e-8, 1] plus 1e-6 damping (kappa 1e6), B = 1024, p = 4,
    30 updates per call.  Full products stay under their bar; mirroring the residual product about doubles the
    floor -- a stated, visible cost of symmetric mode that the GPU test of that configuration holds it to."""
    B, eps = 1024, 1e-6
    kappa = (1.0 + eps) / (1e-8 + eps)
    full, sym = _floors(mm, B, -8.0, 30, 4, eps)
    typ = fp32_floor_typical(kappa, 4, B)
    print(f"kappa={kappa:.2e} B={B}: float32 floor full {full:.2e} symmetric {sym:.2e} (ratio {sym / full:.2f}); "
          f"law {typ:.2e}, full-products bar {fp32_floor(kappa, 4, B, False):.2e}", flush=True)
    assert typ / 2.0 <= full <= 2.0 * typ
    assert full <= fp32_floor(kappa, 4, B, symmetric=False) / 1.5
    assert 1.5 * full <= sym <= SYMMETRIC_OVER_FULL_ILLCONDITIONED * full


# ---- the Clenshaw recurrence in float32 ------------------------------------------------------------------------

def _clenshaw_float32(mm, S, c, symmetric):
    """Appendix A.2, reduced form (d - 1 products), float32: B_{d-1} = 2 c_d S + c_{d-1} I,
    B_k = 2 S B_{k+1} - B_{k+2} + c_k I (B_d = c_d I enters only through c_{d-2} - c_d), result S B_1 - B_2 + c_0 I."""
    f = np.float32
    I = np.eye(S.shape[0], dtype=np.float32)
    d = len(c) - 1
    b1 = f(2.0 * c[d]) * S + f(c[d - 1]) * I
    b0 = f(2) * mm(S, b1, upper=symmetric) + f(c[d - 2] - c[d]) * I
    b2, b1 = b1, b0
    for k in range(d - 3, 0, -1):
        b0 = f(2) * mm(S, b1, upper=symmetric) - b2 + f(c[k]) * I
        b2, b1 = b1, b0
    return mm(S, b1, upper=symmetric) - b2 + f(c[0]) * I


@pytest.mark.parametrize("B,lo_exp", [(256, -4.0), (1024, -4.0), (1024, -1.0)])
@pytest.mark.parametrize("p", [2, 4])
@pytest.mark.parametrize("d", [8, 32])
def test_clenshaw_floor_law_holds_on_the_cpu(mm, B, lo_exp, p, d):
    A32, _, lam = workloads.spd_stack(1, B, lo_exp, 0.0, seed=7, share_q=True)
    A = A32[0].astype(np.float64)
    s = np.sqrt((A * A).sum())
    a, b = float(lam.min() / s) * 0.99, 1.0
    coef = ocheb.chebyshev_fit(p, d, a, b)
    X64 = ocheb.inverse_root_chebyshev(A, p, coef, a, b)
    S = np.float32(2.0 / (b - a)) * (A32[0] * np.float32(1.0 / s)) + np.float32(-(a + b) / (b - a)) * np.eye(B, dtype=np.float32)
    typ, bar = clenshaw_fp32_floor_typical(d, p, B), clenshaw_fp32_floor(d, p, B)
    for symmetric in (False, True):
        X32 = _clenshaw_float32(mm, S, coef, symmetric).astype(np.float64) * s ** (-1.0 / p)
        e = float(np.linalg.norm(X32 - X64) / np.linalg.norm(X64))
        m = float(np.abs(X32 - X64).max() / np.abs(X64).max())
        print(f"Clenshaw B={B} kappa=1e{-lo_exp:.0f} p={p} d={d} symmetric={symmetric}: float32 vs float64 {e:.2e} "
              f"(element-wise {m:.2e}); law {typ:.2e}, bar {bar:.2e}", flush=True)
        assert e <= bar / 1.5 and m <= max_abs_bar(bar) / 1.5
        if lo_exp == -4.0:          # the spectra the law describes: typical value on both sides
            assert typ / 2.0 <= e <= 2.0 * typ
