"""Pins for the Chebyshev / Clenshaw oracle (oracle/chebyshev.py)."""
import os

import numpy as np
import numpy.polynomial.chebyshev as npcheb
import pytest

import workloads
from oracle.evd import inverse_root_evd, rel_frobenius_error
from oracle import chebyshev as cb
from oracle.newton_db import MatmulCounter

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_matmul_counts.txt")


def _golden():
    out = {}
    for line in open(GOLDEN):
        line = line.split("#")[0].strip()
        if line:
            k, v = line.split("=")
            out[k.strip()] = int(v)
    return out


@pytest.mark.parametrize("p", [2, 4])
@pytest.mark.parametrize("d", [4, 9, 16])
def test_fit_with_d_plus_1_nodes_is_interpolation(p, d):
    # with N = d+1 nodes the cosine-sum fit is the Chebyshev interpolant (library routine)
    a, b = 0.05, 1.0
    c = cb.chebyshev_fit(p, d, a, b, n_points=d + 1)
    ref = npcheb.chebinterpolate(lambda t: (0.5 * (b - a) * t + 0.5 * (b + a)) ** (-1.0 / p), d)
    assert np.allclose(c, ref, atol=1e-12)


def test_fit_of_constant_and_linear():
    c = cb.chebyshev_fit(2, 6, 0.1, 1.0, 1000, f=lambda x: np.ones_like(x))
    assert np.allclose(c, [1, 0, 0, 0, 0, 0, 0], atol=1e-13)      # c_0 halved -> exactly 1
    a, b = 0.2, 1.4
    c = cb.chebyshev_fit(2, 4, a, b, 1000, f=lambda x: x)           # x = (b-a)/2 t + (a+b)/2
    assert np.allclose(c, [0.5 * (a + b), 0.5 * (b - a), 0, 0, 0], atol=1e-13)


def test_fit_of_a_chebyshev_polynomial():
    # f = T_3(t): orthogonality picks out c_3 = 1
    a, b = 0.0, 1.0
    c = cb.chebyshev_fit(2, 5, a, b, 64, f=lambda x: npcheb.chebval(2 * x - 1, [0, 0, 0, 1]))
    assert np.allclose(c, [0, 0, 0, 1, 0, 0], atol=1e-13)


def test_coefficients_decay_and_series_converges():
    a, b = 0.01, 1.0
    c = cb.chebyshev_fit(4, 60, a, b, 10000)
    assert abs(c[60]) < abs(c[30]) < abs(c[5])
    x = np.linspace(a, b, 501)
    err = np.abs(cb.clenshaw_scalar(cb.to_unit_interval(x, a, b), c) - x ** -0.25)
    assert err.max() < 2e-3
    c100 = cb.chebyshev_fit(4, 100, a, b, 10000)
    err100 = np.abs(cb.clenshaw_scalar(cb.to_unit_interval(x, a, b), c100) - x ** -0.25)
    assert err100.max() < err.max() / 20


def test_scalar_clenshaw_equals_library_chebval():
    rng = np.random.default_rng(2)
    c = rng.standard_normal(13)
    t = np.linspace(-1, 1, 41)
    assert np.allclose(cb.clenshaw_scalar(t, c), npcheb.chebval(t, c), atol=1e-13)


def test_scalar_clenshaw_low_degree_by_hand():
    # c0 + c1 t + c2 (2t^2 - 1)
    t = np.array([-0.3, 0.0, 0.8])
    assert np.allclose(cb.clenshaw_scalar(t, np.array([2.0, -1.0, 0.5])),
                       2.0 - t + 0.5 * (2 * t * t - 1), atol=1e-15)


@pytest.mark.parametrize("d", [2, 3, 8, 17])
def test_reduced_matrix_form_equals_plain_and_counts(d):
    g = _golden()
    rng = np.random.default_rng(d)
    M = rng.standard_normal((12, 12))
    S = (M + M.T) / 12.0
    c = rng.standard_normal(d + 1)
    c1, c2 = MatmulCounter(), MatmulCounter()
    P = cb.clenshaw_matrix_plain(S, c, c1)
    Rm = cb.clenshaw_matrix_reduced(S, c, c2)
    assert np.allclose(P, Rm, atol=1e-12)
    assert c1.n == d + g["clenshaw_plain_offset"]
    assert c2.n == d + g["clenshaw_reduced_offset"]


def test_matrix_clenshaw_is_the_matrix_polynomial():
    # explicit sum_k c_k T_k(S) with T_k from the three-term recurrence
    rng = np.random.default_rng(4)
    M = rng.standard_normal((10, 10))
    S = (M + M.T) / 10.0
    c = rng.standard_normal(7)
    T_prev, T_cur = np.eye(10), S.copy()
    acc = c[0] * T_prev + c[1] * T_cur
    for k in range(2, 7):
        T_prev, T_cur = T_cur, 2 * S @ T_cur - T_prev
        acc += c[k] * T_cur
    assert np.allclose(cb.clenshaw_matrix_plain(S, c), acc, atol=1e-12)


@pytest.mark.parametrize("p", [2, 4])
def test_inverse_root_matches_spectral_model_and_converges(p):
    B = 32
    Q = workloads.orthogonal_factor(B, 31)
    lam = workloads.log_uniform_spectrum(B, -1.0, 0.0, 32)
    A = workloads.spd_from_spectrum(Q, lam)
    s = np.sqrt((lam ** 2).sum())
    a, b = lam.min() / s, lam.max() / s
    c = cb.chebyshev_fit(p, 40, a, b)
    X = cb.inverse_root_chebyshev(A, p, c, a, b)
    Xm = cb.inverse_root_chebyshev_model(A, p, c, a, b)
    assert rel_frobenius_error(X, Xm)[0] < 1e-11
    X_true = (Q * lam ** (-1.0 / p)) @ Q.T
    assert rel_frobenius_error(X, X_true)[0] < 1e-9


def test_paper_form_evaluates_shifted_function():
    # map of [0,1] (S = 2 A/||A||_F - I) with coefficients fitted on [e, 1+e]:
    # the series then approximates (x + e)^(-1/p) at the scaled eigenvalues x
    B, e, p = 24, 0.05, 2
    Q = workloads.orthogonal_factor(B, 41)
    lam = workloads.log_uniform_spectrum(B, -1.0, 0.0, 42)
    A = workloads.spd_from_spectrum(Q, lam)
    s = np.sqrt((lam ** 2).sum())
    c = cb.chebyshev_fit(p, 60, e, 1.0 + e)
    X = cb.inverse_root_chebyshev(A, p, c, 0.0, 1.0)
    X_true = inverse_root_evd(A / s + e * np.eye(B), p) * s ** (-1.0 / p)
    assert rel_frobenius_error(X, X_true)[0] < 1e-6


def test_identity_block():
    # A = I: s = sqrt(B), scaled eigenvalue 1/sqrt(B); result must be I
    B, p = 16, 4
    a, b = 0.1, 1.0
    c = cb.chebyshev_fit(p, 30, a, b)
    X = cb.inverse_root_chebyshev(np.eye(B), p, c, a, b)
    assert np.allclose(X, np.eye(B), atol=1e-6)
