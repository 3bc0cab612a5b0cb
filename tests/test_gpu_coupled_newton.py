"""Coupled-Newton inverse roots (paper Section 3.2) through the C ABI against the float64 oracle."""
import numpy as np
import pytest

import workloads
from oracle import coupled_newton as ocn
from oracle.evd import inverse_root_evd, rel_frobenius_error

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dash():
    from paper_2602_02016_amd import Dash
    d = Dash(0)
    yield d
    d.close()


def cn_floor(kappa: float, B: int) -> float:
    """fp32 floor of Coupled-Newton.  X is a running product of the C_k that nothing corrects (M steers
    C towards I whatever X has accumulated), so the floor sits above Newton-DB's and keeps growing slowly
    with the iteration count.  Empirical bound: measured 2e-5 (kappa 10, B 1024, k 25), 7.5e-5 (kappa 1e2,
    B 512, k 30), 1.5e-4 (kappa 1e3, B 128, k 30), 9.4e-5 (kappa 1e4, B 256, k 80) -- all below
    4e-5 sqrt(kappa) max(1, sqrt(B/256)) with a factor >= 8 to spare."""
    return 4e-5 * kappa ** 0.5 * max(1.0, (B / 256.0) ** 0.5)


def _to_gpu(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


@pytest.mark.parametrize("p", [2, 4])
@pytest.mark.parametrize("k", [1, 2, 3, 4, 7])
def test_few_iterations_match_float64_iteration(dash, p, k):
    N, B = 3, 128
    A32, _, _ = workloads.spd_stack(N, B, -2.0, 0.0, seed=111)
    dash.reset_stats()
    X = dash.inverse_root(_to_gpu(A32), method="coupled_newton", p=p, iters=k, eps=1e-4).cpu().numpy()
    st = dash.get_stats()
    X_same = ocn.inverse_root_cn(A32.astype(np.float64), p, k, eps=1e-4)
    assert rel_frobenius_error(X, X_same).max() < 1e-5
    # products: the first X update is free, the last iteration updates only X:
    # (k-1) * (3 or 4) against the paper's k * (3 or 4)
    assert st["matmul_products"] == (k - 1) * (3 if p == 2 else 4)


@pytest.mark.parametrize("p", [2, 4])
@pytest.mark.parametrize("N,B,lo,k", [(16, 128, -3.0, 30), (5, 256, -1.0, 25), (3, 512, -2.0, 30), (9, 1024, -1.0, 25)])
def test_converged_and_unconverged_against_evd_and_model(dash, N, B, lo, k, p):
    print(f"cn N={N} B={B} kappa=1e{-lo:.0f} p={p}", flush=True)
    A32, _, _ = workloads.spd_stack(N, B, lo, 0.0, seed=113 + B, share_q=B >= 512)
    sample = [0, N - 1]
    A64 = A32[sample].astype(np.float64)
    X_evd = inverse_root_evd(A64, p, eps=1e-6)
    floor = cn_floor(10 ** (-lo), B)
    for kk in (8, k):
        nf = _to_gpu(np.zeros(N, dtype=np.int32))
        X = dash.inverse_root(_to_gpu(A32), method="cn", p=p, iters=kk, eps=1e-6, nonfinite_out=nf).cpu().numpy()
        X_mod = ocn.inverse_root_cn_model(A64, p, kk, eps=1e-6)
        e_gpu = rel_frobenius_error(X[sample], X_evd)
        e_mod = rel_frobenius_error(X_mod, X_evd)
        print(f"   k={kk}: vs EVD {e_gpu.max():.2e} (float64 model {e_mod.max():.2e})", flush=True)
        assert np.all(np.abs(e_gpu - e_mod) <= 0.1 * e_mod + floor)
        assert int(nf.sum().item()) == 0
    assert e_gpu.max() < max(1e-4, floor)


def test_stability_and_no_mirroring(dash):
    """Long after convergence the iteration must stay put; Coupled-Newton never mirrors a product
    (doing so, even only for C^2 and C^4, makes X drift), so symmetric mode changes nothing."""
    from paper_2602_02016_amd import Dash
    full = Dash(0)
    full.set_symmetric(False)
    N, B = 4, 256
    A32, _, _ = workloads.spd_stack(N, B, -4.0, 0.0, seed=115, share_q=True)
    for p in (2, 4):
        X_evd = inverse_root_evd(A32.astype(np.float64), p)
        floor = cn_floor(1e4, B)
        for k in (40, 80):
            dash.reset_stats(); full.reset_stats()
            es = rel_frobenius_error(dash.inverse_root(_to_gpu(A32), method="cn", p=p, iters=k).cpu().numpy(), X_evd).max()
            ef = rel_frobenius_error(full.inverse_root(_to_gpu(A32), method="cn", p=p, iters=k).cpu().numpy(), X_evd).max()
            print(f"cn stability p={p} k={k}: sym {es:.2e} full {ef:.2e}", flush=True)
            assert es < floor and ef < floor and es == ef
            assert dash.get_stats()["matmul_flops"] == full.get_stats()["matmul_flops"]
    full.close()


def test_half_precision_one_iteration_and_workspace(dash):
    """iters = 1 needs no product in any precision (X = s^(-1/p) C_0 / c), and the half-precision
    workspace (nine 16-bit buffers per block) is smaller than the fp32 one (nine fp32 buffers)."""
    from oracle import lowprec
    N, B = 2, 128
    A32, _, _ = workloads.spd_stack(N, B, -1.0, 0.0, seed=117)
    for prec in ("fp16", "bf16"):
        dash.reset_stats()
        X = dash.inverse_root(_to_gpu(A32), method="cn", p=4, iters=1, eps=1e-6, precision=prec).cpu().numpy()
        assert dash.get_stats()["matmul_products"] == 0
        X_ref = lowprec.inverse_root_cn_lowprec(A32, 4, 1, eps=1e-6, fmt=prec)
        assert rel_frobenius_error(X, X_ref).max() < 1e-6
    assert dash.workspace_bytes(8, 1024, "cn", 4, "fp16") < 0.6 * dash.workspace_bytes(8, 1024, "cn", 4, "fp32")


def test_step_with_coupled_newton(dash):
    import torch
    from oracle import shampoo as oshampoo
    N, B = 3, 256
    beta, eps = 0.95, 1e-6
    S = torch.zeros(2 * N, B, B, device="cuda")
    L64, R64 = np.zeros((N, B, B)), np.zeros((N, B, B))
    for t in range(5):
        G = workloads.gradient_stack(N, B, 9300 + t)
        dash.accumulate_factors(_to_gpu(G), S[:N], S[N:], beta)
        L64, R64 = oshampoo.accumulate_factors(G, L64, R64, beta)
    G = workloads.gradient_stack(N, B, 9400)
    X = torch.zeros_like(S); U = torch.zeros(N, B, B, device="cuda")
    dash.step(_to_gpu(G), S, X, U, beta=beta, eps=eps, method="coupled_newton", p=4, iters=25)
    ref = oshampoo.step(G, L64, R64, beta=beta, eps=eps, p=4)
    assert rel_frobenius_error(X.cpu().numpy(), np.concatenate([ref["X_L"], ref["X_R"]])).max() < 1e-4
    assert rel_frobenius_error(U.cpu().numpy(), ref["U"]).max() < 1e-4
