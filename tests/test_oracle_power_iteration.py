"""Pins for the multi-Power-Iteration oracle (oracle/power_iteration.py)."""
import numpy as np
import pytest

import workloads
from oracle import newton_db as ondb
from oracle import power_iteration as opi
from oracle.evd import inverse_root_evd, rel_frobenius_error


def _spd(B, lo, seed):
    Q = workloads.orthogonal_factor(B, seed)
    lam = workloads.log_uniform_spectrum(B, lo, 0.0, seed + 1)
    return workloads.spd_from_spectrum(Q, lam), Q, lam


def _pool(B, m, seed):
    return workloads.start_vectors(B, m, seed).astype(np.float64)


def test_rayleigh_quotient_bounds_and_eigenvector():
    # R_A(x) <= lambda_max for every x, with equality at the top eigenvector (Section 3.4)
    A, Q, lam = _spd(24, -2.0, 3)
    rng = np.random.default_rng(0)
    for _ in range(20):
        assert opi.rayleigh_quotient(A, rng.standard_normal(24)) <= lam.max() * (1 + 1e-12)
    top = Q[:, np.argmax(lam)]
    assert opi.rayleigh_quotient(A, top) == pytest.approx(lam.max(), rel=1e-12)


def test_single_vector_is_textbook_power_iteration():
    A, _, lam = _spd(16, -1.0, 5)
    v0 = _pool(16, 1, 7)
    lam_pi, q = opi.multi_power_iteration(A, v0, 6)
    v = v0[:, 0] / np.linalg.norm(v0[:, 0])
    for _ in range(5):                       # five multiplications, then the quotient of that vector
        v = A @ v
        v /= np.linalg.norm(v)
    assert lam_pi == pytest.approx(v @ A @ v, rel=1e-12) and q.shape == (1,)


def test_never_exceeds_and_converges_to_lambda_max():
    A, _, lam = _spd(32, -3.0, 9)
    V0 = _pool(32, 16, 11)
    prev = 0.0
    for sweeps in (1, 2, 4, 8, 16, 64, 400):
        l, _ = opi.multi_power_iteration(A, V0, sweeps)
        assert l <= lam.max() * (1 + 1e-12)
        assert l >= prev * (1 - 1e-12)       # Rayleigh quotients of power iterates do not decrease (SPD)
        prev = l
    assert prev == pytest.approx(np.linalg.eigvalsh(A).max(), rel=1e-6)


def test_pool_keeps_the_largest_quotient():
    A, _, _ = _spd(20, -2.0, 13)
    V0 = _pool(20, 16, 15)
    l, q = opi.multi_power_iteration(A, V0, 3)
    singles = [opi.multi_power_iteration(A, V0[:, j:j + 1], 3)[0] for j in range(16)]
    assert np.allclose(q, singles, rtol=1e-12) and l == pytest.approx(max(singles))


def test_start_vector_orthogonal_to_top_is_rescued_by_the_pool():
    # Section 3.5: a single start vector can converge to a smaller eigenvalue; a pool avoids it
    lam = np.array([1.0, 0.5, 0.1, 0.05])
    A = np.diag(lam)
    bad = np.array([[0.0], [1.0], [0.3], [0.2]])              # no component along e_1
    assert opi.multi_power_iteration(A, bad, 50)[0] == pytest.approx(0.5, rel=1e-6)
    pool = np.concatenate([bad, np.array([[0.1], [1.0], [0.0], [0.0]])], axis=1)
    assert opi.multi_power_iteration(A, pool, 50)[0] == pytest.approx(1.0, rel=1e-6)


def test_scaling_damping_and_homogeneity():
    A, _, lam = _spd(16, -1.0, 17)
    V0 = _pool(16, 16, 19)
    l, _ = opi.multi_power_iteration(A, V0, 5)
    assert opi.multi_power_iteration(3.0 * A, V0, 5)[0] == pytest.approx(3.0 * l, rel=1e-12)
    assert opi.multi_power_iteration(A, 7.0 * V0, 5)[0] == pytest.approx(l, rel=1e-12)
    # damping: (A + eps I) has the same eigenvectors, eigenvalues shifted by eps
    le, _ = opi.multi_power_iteration(A, V0, 5, eps=0.25)
    ls, _ = opi.multi_power_iteration(A + 0.25 * np.eye(16), V0, 5)
    assert le == pytest.approx(ls, rel=1e-12)
    s = opi.power_iteration_scale(np.stack([A, 2 * A]), V0, 5)
    assert np.allclose(s, [2 * l, 4 * l], rtol=1e-12)


def test_ndb_with_power_iteration_scaling_needs_fewer_iterations():
    # Section 3.4: 2*lambda_PI is much closer to lambda_max than ||A||_F, so a fixed iteration
    # count gets closer to the root
    # flat spectrum in [0.5, 1]: ||A||_F ~ 0.76 sqrt(B) is ~9x lambda_max at B = 128
    B = 128
    Q = workloads.orthogonal_factor(B, 21)
    lam = np.linspace(0.5, 1.0, B)
    A = workloads.spd_from_spectrum(Q, lam)
    V0 = _pool(B, 16, 23)
    s_pi = ondb.block_scale(A, "power_iteration", (V0, 8))
    s_fro = ondb.block_scale(A, "frobenius")
    assert lam.max() <= s_pi <= 2 * lam.max() * (1 + 1e-12) and s_pi < s_fro / 4
    X_true = inverse_root_evd(A, 4)
    e_pi = rel_frobenius_error(ondb.inverse_root_ndb(A, 4, 5, scaling="power_iteration", pi=(V0, 8)), X_true)[0]
    e_fro = rel_frobenius_error(ondb.inverse_root_ndb(A, 4, 5, scaling="frobenius"), X_true)[0]
    assert e_pi < e_fro / 5
    # and both converge to the same root
    X = ondb.inverse_root_ndb(A, 4, 40, scaling="power_iteration", pi=(V0, 8))
    assert rel_frobenius_error(X, X_true)[0] < 1e-9
