"""Pins for the Newton-DB oracle (oracle/newton_db.py)."""
import os

import numpy as np
import pytest

import workloads
from oracle.evd import inverse_root_evd, rel_frobenius_error
from oracle import newton_db as ndb

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


def test_converges_to_sqrt_and_inverse_sqrt():
    # limit of the iteration: Y -> A^{1/2}, Z -> A^{-1/2} (Section 3.3), known by construction
    A, Q, lam = _spd(24, -1.0, 3)
    Y, Z = ndb.ndb_plain(A, 40)
    assert np.allclose(Y, (Q * np.sqrt(lam)) @ Q.T, atol=1e-12)
    assert np.allclose(Z, (Q / np.sqrt(lam)) @ Q.T, atol=1e-11)
    assert np.allclose(Y @ Z, np.eye(24), atol=1e-11)


@pytest.mark.parametrize("iters", [1, 2, 3, 7])
def test_shortcut_equals_plain(iters):
    # Section 3.3: the closed-form first iteration does not change the result
    A, _, _ = _spd(20, -2.0, 5)
    Yp, Zp = ndb.ndb_plain(A, iters)
    Ys, Zs = ndb.ndb_shortcut(A, iters)
    assert np.allclose(Yp, Ys, atol=1e-13) and np.allclose(Zp, Zs, atol=1e-13)


def test_first_iteration_closed_form():
    A, _, _ = _spd(8, -1.0, 7)
    Y, Z = ndb.ndb_plain(A, 1)
    E1 = 1.5 * np.eye(8) - 0.5 * A
    assert np.allclose(Z, E1, atol=1e-15) and np.allclose(Y, A @ E1, atol=1e-15)


def test_matmul_counts_match_paper():
    g = _golden()
    A, _, _ = _spd(6, -1.0, 9)
    for k in (1, 2, 5, 10):
        c = ndb.MatmulCounter()
        ndb.ndb_plain(A, k, c)
        assert c.n == g["ndb_per_iteration"] * k
        c = ndb.MatmulCounter()
        ndb.ndb_shortcut(A, k, c)
        assert c.n == g["ndb_per_iteration"] * k - g["ndb_first_iteration_saved"]
        for p, calls in ((2, g["ndb_calls_p2"]), (4, g["ndb_calls_p4"])):
            c = ndb.MatmulCounter()
            ndb.inverse_root_ndb(A, p, k, counter=c)
            assert c.n == calls * (3 * k - 2)


def test_scalar_recurrence_is_what_matrices_do():
    # every iterate is a polynomial in A: Q^T Z_k Q = diag(z_k(lam))
    A, Q, lam = _spd(16, -2.0, 11)
    for k in (1, 3, 6):
        Y, Z = ndb.ndb_plain(A, k)
        y, z = ndb.ndb_scalar(lam, k)
        assert np.allclose(Q.T @ Y @ Q, np.diag(y), atol=1e-12)
        assert np.allclose(Q.T @ Z @ Q, np.diag(z), atol=1e-11)


def test_scalar_one_step_by_hand():
    # x = 1/4: e = (3 - 1/4)/2 = 11/8, y1 = 11/32, z1 = 11/8
    y, z = ndb.ndb_scalar(0.25, 1)
    assert y == pytest.approx(11 / 32) and z == pytest.approx(11 / 8)
    # second step: e = (3 - 121/256)/2 = 647/512
    y, z = ndb.ndb_scalar(0.25, 2)
    assert y == pytest.approx(11 / 32 * 647 / 512) and z == pytest.approx(11 / 8 * 647 / 512)


def test_scalar_invariants():
    # y_k = x z_k at every step (Y = A Z), fixed point at x = 1, y_k <= sqrt(x) <= 1 on (0, 1]
    x = np.array([1e-6, 1e-3, 0.1, 0.5, 0.99, 1.0])
    for k in range(1, 30):
        y, z = ndb.ndb_scalar(x, k)
        assert np.allclose(y, x * z, rtol=1e-12)
        assert np.all(y <= np.sqrt(x) * (1 + 1e-12))
    y, z = ndb.ndb_scalar(1.0, 5)
    assert y == 1.0 and z == 1.0


def test_steps_grow_as_eigenvalue_shrinks():
    # Figures 1-2: smaller x needs more steps; close to 1 very few
    steps = [ndb.ndb_scalar_steps_to_tol(x) for x in (0.99, 0.5, 1e-1, 1e-2, 2e-4, 1e-6)]
    assert steps == sorted(steps)
    assert steps[0] <= 4
    assert ndb.ndb_scalar_steps_to_tol(2e-4) > ndb.ndb_scalar_steps_to_tol(1e-2)


@pytest.mark.parametrize("p", [2, 4])
@pytest.mark.parametrize("scaling", ["frobenius", "trace"])
def test_inverse_root_reaches_evd(p, scaling):
    A, Q, lam = _spd(32, -2.0, 13)
    X_true = (Q * lam ** (-1.0 / p)) @ Q.T
    X = ndb.inverse_root_ndb(A, p, 40, scaling=scaling)
    assert rel_frobenius_error(X, X_true)[0] < 1e-10


@pytest.mark.parametrize("p", [2, 4])
@pytest.mark.parametrize("k", [3, 8, 12])
def test_matrix_equals_spectral_model_when_unconverged(p, k):
    A, Q, lam = _spd(32, -3.0, 15)
    X = ndb.inverse_root_ndb(A, p, k, eps=1e-6)
    Xm = ndb.inverse_root_ndb_model(A, p, k, eps=1e-6)
    assert rel_frobenius_error(X, Xm)[0] < 1e-10
    # and the closed-form truncation error agrees with the measured distance to the true root
    s = ndb.block_scale(A + 1e-6 * np.eye(32), "frobenius")
    pred = ndb.ndb_truncation_error(lam + 1e-6, s, p, k)
    meas = rel_frobenius_error(X, inverse_root_evd(A, p, eps=1e-6))[0]
    assert meas == pytest.approx(pred, rel=1e-6, abs=1e-12)


def test_scaling_bounds():
    # lambda_max <= ||A||_F <= tr A for SPD; identity: ||I||_F = sqrt(B)
    A, _, lam = _spd(40, -3.0, 17)
    fro, tr = ndb.block_scale(A, "frobenius"), ndb.block_scale(A, "trace")
    assert lam.max() <= fro * (1 + 1e-12) <= tr * (1 + 1e-12)
    assert fro == pytest.approx(np.sqrt((lam ** 2).sum()))
    assert tr == pytest.approx(lam.sum())
    assert ndb.block_scale(np.eye(9), "frobenius") == pytest.approx(3.0)


def test_damping_and_unscaling():
    # A = c I: s = (c+eps) sqrt(B); result must still be (c+eps)^{-1/p} I
    B, c, eps = 9, 0.3, 0.2
    for p in (2, 4):
        X = ndb.inverse_root_ndb(c * np.eye(B), p, 30, eps=eps)
        assert np.allclose(X, (c + eps) ** (-1 / p) * np.eye(B), atol=1e-12)


def test_config1_prediction_table():
    # k = 10 is not converged for kappa = 1e3 under Frobenius scaling, k = 15 is
    A32, Q, lam = workloads.spd_stack(1, 128, -3.0, 0.0, seed=1)
    A = A32[0].astype(np.float64)
    Xe = inverse_root_evd(A, 4)
    e10 = rel_frobenius_error(ndb.inverse_root_ndb_model(A, 4, 10), Xe)[0]
    e15 = rel_frobenius_error(ndb.inverse_root_ndb_model(A, 4, 15), Xe)[0]
    assert 1e-3 < e10 < 0.3
    assert e15 < 1e-6
