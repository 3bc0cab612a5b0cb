"""Pins for the eigendecomposition root (oracle/evd.py): each compares the oracle with
something that is not the oracle -- a spectrum chosen by construction, a closed form,
a defining identity, brute force on tiny matrices, a library routine."""
import numpy as np
import pytest
import scipy.linalg

import workloads
from oracle.evd import inverse_root_evd, rel_frobenius_error


@pytest.mark.parametrize("p", [2, 4])
@pytest.mark.parametrize("B,lo", [(16, -3.0), (64, -4.0), (128, -3.0)])
def test_known_q_lambda(p, B, lo):
    # A = Q diag(lam) Q^T  =>  A^{-1/p} = Q diag(lam^{-1/p}) Q^T without any eigensolver
    Q = workloads.orthogonal_factor(B, 11 + B)
    lam = workloads.log_uniform_spectrum(B, lo, 0.0, 17 + B)
    A = workloads.spd_from_spectrum(Q, lam)
    X_true = (Q * lam[None, :] ** (-1.0 / p)) @ Q.T
    X = inverse_root_evd(A, p)
    assert rel_frobenius_error(X, X_true)[0] < 1e-9 * 10 ** (-lo - 3)


@pytest.mark.parametrize("p", [2, 4])
def test_defining_identities(p):
    # X^p A = I, X A = A X, X = X^T, X positive definite
    rng = np.random.default_rng(5)
    M = rng.standard_normal((48, 60))
    A = M @ M.T / 60.0
    X = inverse_root_evd(A, p, eps=1e-3)
    Ad = A + 1e-3 * np.eye(48)
    assert np.allclose(np.linalg.matrix_power(X, p) @ Ad, np.eye(48), atol=1e-9)
    assert np.allclose(X @ Ad, Ad @ X, atol=1e-10)
    assert np.allclose(X, X.T, atol=1e-12)
    assert np.linalg.eigvalsh(X).min() > 0


@pytest.mark.parametrize("p", [2, 4])
def test_2x2_closed_form(p):
    # [[a,b],[b,c]]: eigenpairs from the quadratic formula and a rotation angle
    a, b, c = 2.0, 0.7, 1.1
    A = np.array([[a, b], [b, c]])
    mean, diff = 0.5 * (a + c), 0.5 * (a - c)
    rad = np.hypot(diff, b)
    l1, l2 = mean + rad, mean - rad
    th = 0.5 * np.arctan2(2 * b, a - c)
    v1 = np.array([np.cos(th), np.sin(th)])
    v2 = np.array([-np.sin(th), np.cos(th)])
    X_true = l1 ** (-1 / p) * np.outer(v1, v1) + l2 ** (-1 / p) * np.outer(v2, v2)
    assert np.allclose(inverse_root_evd(A, p), X_true, atol=1e-13)


@pytest.mark.parametrize("p", [2, 4])
def test_4x4_kronecker_and_diagonal(p):
    # diag: elementwise power; kron(A1, A2)^{-1/p} = kron(A1^{-1/p}, A2^{-1/p})
    d = np.array([0.5, 2.0, 3.0, 0.01])
    assert np.allclose(inverse_root_evd(np.diag(d), p), np.diag(d ** (-1 / p)), atol=1e-13)
    A1 = np.array([[2.0, 0.3], [0.3, 1.0]])
    A2 = np.array([[1.5, -0.4], [-0.4, 0.9]])
    lhs = inverse_root_evd(np.kron(A1, A2), p)
    rhs = np.kron(inverse_root_evd(A1, p), inverse_root_evd(A2, p))
    assert np.allclose(lhs, rhs, atol=1e-12)


@pytest.mark.parametrize("p", [2, 4])
def test_scalar_multiple_of_identity_and_damping(p):
    X = inverse_root_evd(3.0 * np.eye(7), p, eps=1.0)   # (3+1) I
    assert np.allclose(X, 4.0 ** (-1 / p) * np.eye(7), atol=1e-14)
    # zero matrix + eps I: only the damping term remains
    X0 = inverse_root_evd(np.zeros((5, 5)), p, eps=1e-6)
    assert np.allclose(X0, (1e-6) ** (-1 / p) * np.eye(5), rtol=1e-12)


@pytest.mark.parametrize("p", [2, 4])
def test_rank_one_update_closed_form(p):
    # (I + u u^T)^{-1/p} = I + ((1 + u^T u)^{-1/p} - 1) u u^T / (u^T u)
    rng = np.random.default_rng(9)
    u = rng.standard_normal(40)
    uu = u @ u
    A = np.eye(40) + np.outer(u, u)
    X_true = np.eye(40) + ((1 + uu) ** (-1 / p) - 1) * np.outer(u, u) / uu
    assert np.allclose(inverse_root_evd(A, p), X_true, atol=1e-12)


@pytest.mark.parametrize("p", [2, 4])
def test_against_scipy_fractional_power(p):
    rng = np.random.default_rng(21)
    M = rng.standard_normal((24, 24))
    A = M @ M.T + 0.5 * np.eye(24)
    X_lib = scipy.linalg.fractional_matrix_power(A, -1.0 / p)
    assert np.allclose(inverse_root_evd(A, p), np.real(X_lib), atol=1e-9)
    if p == 2:
        assert np.allclose(inverse_root_evd(A, 2), np.linalg.inv(np.real(scipy.linalg.sqrtm(A))), atol=1e-9)


def test_stack_matches_per_block_and_symmetrises():
    A32, Q, lam = workloads.spd_stack(3, 32, -2.0, 0.0, seed=3)
    X = inverse_root_evd(A32, 4, eps=1e-6)
    for i in range(3):
        assert np.array_equal(X[i], inverse_root_evd(A32[i], 4, eps=1e-6))
    # asymmetric rounding noise is averaged away, not picked from one triangle
    A = A32[0].astype(np.float64)
    noise = 1e-9 * np.triu(np.ones_like(A), 1)
    assert np.allclose(inverse_root_evd(A + noise, 4), inverse_root_evd(A + 0.5 * (noise + noise.T), 4), atol=1e-13)


def test_rejects_indefinite():
    with pytest.raises(ValueError):
        inverse_root_evd(np.diag([1.0, -0.5]), 2)


def test_rel_error_metric():
    X = np.eye(3)
    assert rel_frobenius_error(1.1 * X, X)[0] == pytest.approx(0.1)
