"""Pins for the Coupled-Newton oracle (oracle/coupled_newton.py)."""
import os

import numpy as np
import pytest

import workloads
from oracle import coupled_newton as ocn
from oracle import newton_db as ondb
from oracle.evd import inverse_root_evd, rel_frobenius_error

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_matmul_counts.txt")


def _golden():
    out = {}
    for line in open(GOLDEN):
        line = line.split("#")[0].strip()
        if line:
            k, v = line.split("=")
            out[k.strip()] = int(v)
    return out


def _spd(B, lo, seed):
    Q = workloads.orthogonal_factor(B, seed)
    lam = workloads.log_uniform_spectrum(B, lo, 0.0, seed + 1)
    return workloads.spd_from_spectrum(Q, lam), Q, lam


def test_constant():
    # Section 3.4: (p+1) c^p = 1
    for p in (2, 4):
        assert (p + 1) * ocn.cn_constant(p) ** p == pytest.approx(1.0)


@pytest.mark.parametrize("p", [2, 4])
def test_converges_to_known_root_and_m_to_identity(p):
    A, Q, lam = _spd(24, -1.0, 3)
    A, lam = 0.9 * A, 0.9 * lam              # strictly inside the admissible interval (0, 1)
    X, M = ocn.cn_plain(A, p, 80)
    assert np.allclose(X, (Q * lam ** (-1.0 / p)) @ Q.T, atol=1e-10)
    assert np.allclose(M, np.eye(24), atol=1e-10)


@pytest.mark.parametrize("p", [2, 4])
def test_right_end_of_the_interval_is_a_dead_point(p):
    # at x = (p+1) c^p = 1 exactly: m_0 = p+1, C_0 = 0, and the iterate is stuck at 0 -- the
    # admissible interval is half open, so the scale must be strictly above lambda_max
    xk, _ = ocn.cn_scalar(1.0, p, 30)
    assert abs(xk) < 1e-12
    xk, _ = ocn.cn_scalar(0.999, p, 200)
    assert xk == pytest.approx(0.999 ** (-1.0 / p), rel=1e-9)


@pytest.mark.parametrize("p", [2, 4])
def test_coupling_invariant(p):
    # M_k = X_k^p A at every step (M tracks how far X^p A is from the identity)
    A, _, _ = _spd(12, -2.0, 5)
    for k in (1, 3, 7):
        X, M = ocn.cn_plain(A, p, k)
        assert np.allclose(M, np.linalg.matrix_power(X, p) @ A, atol=1e-11)


def test_matmul_counts_match_paper():
    g = _golden()
    A, _, _ = _spd(6, -1.0, 7)
    for p, key in ((2, "cn_per_iteration_p2"), (4, "cn_per_iteration_p4")):
        for k in (1, 4, 9):
            c = ondb.MatmulCounter()
            ocn.cn_plain(A, p, k, counter=c)
            assert c.n == g[key] * k


@pytest.mark.parametrize("p", [2, 4])
def test_scalar_recurrence_and_one_step_by_hand(p):
    A, Q, lam = _spd(16, -2.0, 9)
    for k in (1, 2, 5):
        X, M = ocn.cn_plain(A, p, k)
        xk, mk = ocn.cn_scalar(lam, p, k)
        assert np.allclose(Q.T @ X @ Q, np.diag(xk), atol=1e-11)
        assert np.allclose(Q.T @ M @ Q, np.diag(mk), atol=1e-11)
    # one step from x: m0 = (p+1) x, c0 = (1 + 1/p) - (p+1) x / p, x1 = c0 / c
    x = 0.3
    c = ocn.cn_constant(p)
    x1, m1 = ocn.cn_scalar(x, p, 1)
    c0 = (1 + 1 / p) - (p + 1) * x / p
    assert x1 == pytest.approx(c0 / c) and m1 == pytest.approx(c0 ** p * (p + 1) * x)


def test_steps_to_tolerance_shape_of_the_paper_figures():
    # Figures 1-2: small x needs more steps; near x -> 1 Coupled-Newton needs many more steps than
    # Newton-DB (which needs very few there), the reason the paper prefers Newton-DB
    cn = [ocn.cn_scalar_steps_to_tol(x, 2) for x in (1e-4, 1e-2, 0.3)]
    assert cn[0] > cn[1] > cn[2]
    assert ocn.cn_scalar_steps_to_tol(0.99, 2) > 2 * ondb.ndb_scalar_steps_to_tol(0.99)
    assert ocn.cn_scalar_steps_to_tol(0.99, 2) > ocn.cn_scalar_steps_to_tol(0.3, 2)


@pytest.mark.parametrize("p", [2, 4])
@pytest.mark.parametrize("scaling", ["frobenius", "trace"])
def test_inverse_root_reaches_evd_and_model(p, scaling):
    A, Q, lam = _spd(32, -2.0, 11)
    X_true = (Q * lam ** (-1.0 / p)) @ Q.T
    assert rel_frobenius_error(ocn.inverse_root_cn(A, p, 80, scaling=scaling), X_true)[0] < 1e-9
    for k in (3, 10):
        X = ocn.inverse_root_cn(A, p, k, eps=1e-6, scaling=scaling)
        Xm = ocn.inverse_root_cn_model(A, p, k, eps=1e-6, scaling=scaling)
        assert rel_frobenius_error(X, Xm)[0] < 1e-10


def test_identity_scaled():
    # A = a I: s = a sqrt(B); the result must be a^(-1/p) I once converged
    for p in (2, 4):
        X = ocn.inverse_root_cn(0.7 * np.eye(9), p, 60)
        assert np.allclose(X, 0.7 ** (-1 / p) * np.eye(9), atol=1e-10)
