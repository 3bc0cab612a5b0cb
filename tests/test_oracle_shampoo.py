"""Pins for the Shampoo-step oracle (oracle/shampoo.py)."""
import numpy as np
import pytest

import workloads
from oracle import shampoo
from oracle.evd import inverse_root_evd


def _G(N=3, B=12, seed=0, std=1.0):
    return workloads.gradient_stack(N, B, seed, std).astype(np.float64)


def test_accumulate_elementwise_brute_force():
    G = _G(2, 5, 1)
    L0 = np.arange(50, dtype=np.float64).reshape(2, 5, 5)
    R0 = -L0
    L, R = shampoo.accumulate_factors(G, L0, R0, beta=0.9, alpha=0.25)
    for n in range(2):
        for i in range(5):
            for j in range(5):
                l = sum(G[n, i, k] * G[n, j, k] for k in range(5))
                r = sum(G[n, k, i] * G[n, k, j] for k in range(5))
                assert L[n, i, j] == pytest.approx(0.9 * L0[n, i, j] + 0.25 * l, abs=1e-12)
                assert R[n, i, j] == pytest.approx(0.9 * R0[n, i, j] + 0.25 * r, abs=1e-12)


def test_accumulate_default_alpha_and_invariants():
    G = _G(4, 16, 2)
    Z = np.zeros_like(G)
    L, R = shampoo.accumulate_factors(G, Z, Z, beta=0.0)          # alpha = 1: L = G G^T
    assert np.allclose(L, G @ np.swapaxes(G, 1, 2)) and np.allclose(R, np.swapaxes(G, 1, 2) @ G)
    # tr L = tr R = ||G||_F^2, symmetric, PSD -- and preserved along an EMA from equal traces
    L, R = Z, Z
    for t in range(5):
        L, R = shampoo.accumulate_factors(_G(4, 16, 10 + t), L, R, beta=0.95)
        assert np.allclose(np.trace(L, axis1=1, axis2=2), np.trace(R, axis1=1, axis2=2))
        assert np.allclose(L, np.swapaxes(L, 1, 2)) and np.allclose(R, np.swapaxes(R, 1, 2))
        assert np.linalg.eigvalsh(L).min() > -1e-12
    Lb, _ = shampoo.accumulate_factors(G, Z, Z, beta=0.95)
    assert np.allclose(np.trace(Lb, axis1=1, axis2=2), 0.05 * (G ** 2).sum(axis=(1, 2)))


def test_accumulate_does_not_modify_inputs():
    G = _G(1, 4, 3)
    L0 = np.ones((1, 4, 4))
    shampoo.accumulate_factors(G, L0, L0, 0.5)
    assert np.all(L0 == 1.0)


def test_precondition_identity_and_order():
    G = _G(2, 6, 4)
    I = np.broadcast_to(np.eye(6), (2, 6, 6))
    assert np.allclose(shampoo.precondition(I, G, I), G)
    rng = np.random.default_rng(0)
    Lm, Rm = rng.standard_normal((2, 6, 6)), rng.standard_normal((2, 6, 6))
    U = shampoo.precondition(Lm, G, Rm)
    for n in range(2):
        assert np.allclose(U[n], Lm[n] @ G[n] @ Rm[n])
        assert not np.allclose(U[n], Rm[n] @ G[n] @ Lm[n])


def test_single_gradient_step_gives_orthogonal_factor():
    # beta = 0, alpha = 1, eps -> 0, G = Q_L Sigma Q_R^T full rank:
    # L^{-1/4} G R^{-1/4} = Q_L Sigma^{-1/2} Sigma Sigma^{-1/2} Q_R^T = Q_L Q_R^T
    B = 10
    QL, QR = workloads.orthogonal_factor(B, 1), workloads.orthogonal_factor(B, 2)
    sig = np.linspace(0.5, 2.0, B)
    G = ((QL * sig) @ QR.T)[None]
    Z = np.zeros_like(G)
    out = shampoo.step(G, Z, Z, beta=0.0, eps=0.0, p=4, alpha=1.0)
    assert np.allclose(out["U"][0], QL @ QR.T, atol=1e-10)
    assert np.allclose(np.linalg.svd(out["U"][0], compute_uv=False), 1.0, atol=1e-10)
    # scale invariance of that case: U(cG) = U(G)
    out3 = shampoo.step(3.0 * G, Z, Z, beta=0.0, eps=0.0, p=4, alpha=1.0)
    assert np.allclose(out3["U"], out["U"], atol=1e-10)


def test_step_composition_and_stacking():
    G = _G(3, 8, 6)
    L0 = np.broadcast_to(np.eye(8), (3, 8, 8)) * 0.1
    out = shampoo.step(G, L0, L0, beta=0.9, eps=1e-3, p=4)
    L, R = shampoo.accumulate_factors(G, L0, L0, 0.9)
    assert np.allclose(out["L"], L) and np.allclose(out["R"], R)
    assert np.allclose(out["X_L"], inverse_root_evd(L, 4, 1e-3))
    assert np.allclose(out["X_R"], inverse_root_evd(R, 4, 1e-3))
    assert np.allclose(out["U"], out["X_L"] @ G @ out["X_R"])


def test_grafting_norm_and_adam_direction():
    G = _G(2, 8, 7)
    U = _G(2, 8, 8)
    Acc0 = np.zeros_like(G)
    Acc, s = shampoo.adam_graft(G, U, Acc0, beta_g=0.999, eps_g=1e-8)
    assert np.allclose(Acc, 0.001 * G * G)
    P = G / (1e-8 + np.sqrt(Acc))
    for n in range(2):
        assert np.linalg.norm(s[n] * U[n]) == pytest.approx(np.linalg.norm(P[n]))
    # first step from zero state: |P| ~ 1/sqrt(1-beta_g) elementwise, so ||P||_F ~ B/sqrt(1e-3)
    assert np.linalg.norm(P[0]) == pytest.approx(8 / np.sqrt(1e-3), rel=1e-4)


def test_step_with_grafted_update():
    G = _G(2, 6, 9)
    Z = np.zeros_like(G)
    theta = _G(2, 6, 10)
    out = shampoo.step(G, Z, Z, beta=0.95, eps=1e-6, p=4,
                       graft=dict(Acc=Z, beta_g=0.999, eps_g=1e-8), theta=theta, lr=1e-3)
    for n in range(2):
        assert np.allclose(out["theta"][n], theta[n] - 1e-3 * out["s"][n] * out["U"][n])


def test_blocking_example_shapes():
    # Section 4.1 worked example (full blocks only are built; this checks the counting)
    import os
    vals = {}
    for line in open(os.path.join(os.path.dirname(__file__), "golden", "paper_blocking_example.txt")):
        line = line.split("#")[0].strip()
        if line:
            k, v = line.split("=")
            vals[k.strip()] = v.strip()
    V, E, B = int(vals["V"]), int(vals["E"]), int(vals["B"])
    n_m, n_n = V // B, E // B
    assert n_m == int(vals["N_m_full"]) and n_n == int(vals["N_n"])
    assert n_m * n_n == int(vals["N_full"]) and V % B == int(vals["rest_rows"])
    assert workloads.blocks_of_layer(n_m * B, E, B) == int(vals["N_full"])
    # S_full = L_full + R_full + R_rest blocks
    assert 2 * n_m * n_n + n_n == int(vals["S_full"].split(",")[0])
    assert workloads.cfg2_num_blocks() == 16 and workloads.cfg3_num_gradient_blocks() == 1536


def test_adam_graft_zero_block_has_zero_scale():
    """Reading of Section 2.3 for a block whose update is all zero: s = 0 (not 0/0); other blocks unchanged."""
    rng = np.random.default_rng(5)
    G = rng.standard_normal((3, 8, 8))
    U = rng.standard_normal((3, 8, 8))
    G[1] = 0.0
    U[1] = 0.0
    Acc, s = shampoo.adam_graft(G, U, np.zeros((3, 8, 8)), 0.999, 1e-8)
    assert s[1] == 0.0 and np.all(np.isfinite(s)) and s[0] > 0 and s[2] > 0
    P0 = G[0] / (1e-8 + np.sqrt(Acc[0]))
    assert s[0] == pytest.approx(np.linalg.norm(P0) / np.linalg.norm(U[0]), rel=1e-12)
