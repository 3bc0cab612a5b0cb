"""Parity of dash_step and dash_graft_update (HIP, through the C ABI) with the float64
oracle step of Algorithm 1 (eigendecomposition roots)."""
import numpy as np
import pytest

import workloads
from oracle import shampoo as oshampoo
from oracle.evd import rel_frobenius_error
from tolerances import max_abs_bar, rel_max_abs_error

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dash():
    from paper_2602_02016_amd import Dash
    d = Dash(0)
    yield d
    d.close()


def _to_gpu(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


@pytest.mark.parametrize("precision", ["fp32", "bf16x6", "fp16x3"])
@pytest.mark.parametrize("N,B,warm", [(4, 128, 6), (3, 256, 4), (2, 512, 3)])
def test_step_against_oracle(dash, N, B, warm, precision):
    """Factors are EMAs of seeded N(0, 1e-2^2) gradients (Wishart-like, well conditioned once
    a few gradients are in); Newton-DB p=4 with k=12 is converged there, so the GPU step
    must agree with the EVD-based oracle step to fp32 accuracy -- with fp32 MFMA operands and with
    three-plane split bf16 operands, to the same bar."""
    import torch
    print(f"step N={N} B={B} {precision}", flush=True)
    beta, eps = 0.95, 1e-6
    S = torch.zeros(2 * N, B, B, device="cuda")
    X = torch.zeros_like(S)
    U = torch.zeros(N, B, B, device="cuda")
    nf = torch.ones(2 * N, dtype=torch.int32, device="cuda")
    L64, R64 = np.zeros((N, B, B)), np.zeros((N, B, B))
    for t in range(warm):
        G = workloads.gradient_stack(N, B, 3000 + t)
        dash.accumulate_factors(_to_gpu(G), S[:N], S[N:], beta)
        L64, R64 = oshampoo.accumulate_factors(G, L64, R64, beta)
    G = workloads.gradient_stack(N, B, 3000 + warm)
    dash.step(_to_gpu(G), S, X, U, beta=beta, eps=eps, p=4, iters=12, nonfinite_out=nf, precision=precision)
    ref = oshampoo.step(G, L64, R64, beta=beta, eps=eps, p=4)
    torch.cuda.synchronize()
    eS = rel_frobenius_error(S.cpu().numpy(), np.concatenate([ref["L"], ref["R"]])).max()
    eX = rel_frobenius_error(X.cpu().numpy(), np.concatenate([ref["X_L"], ref["X_R"]])).max()
    eU = rel_frobenius_error(U.cpu().numpy(), ref["U"]).max()
    # the same comparisons element by element, scaled by the largest entry of the reference block
    mS = rel_max_abs_error(S.cpu().numpy(), np.concatenate([ref["L"], ref["R"]])).max()
    mX = rel_max_abs_error(X.cpu().numpy(), np.concatenate([ref["X_L"], ref["X_R"]])).max()
    mU = rel_max_abs_error(U.cpu().numpy(), ref["U"]).max()
    print(f"   factors {eS:.2e} roots {eX:.2e} update {eU:.2e}; element-wise {mS:.2e} {mX:.2e} {mU:.2e}", flush=True)
    assert eS < 1e-5
    assert eX < 1e-4
    assert eU < 1e-4
    assert mS < max_abs_bar(1e-5) and mX < max_abs_bar(1e-4) and mU < max_abs_bar(1e-4)
    assert np.all(nf.cpu().numpy() == 0)

    # non-refresh step (cached roots, Section 4.1): factors move on, X untouched, U uses old X
    X_before = X.clone()
    G2 = workloads.gradient_stack(N, B, 3900)
    dash.step(_to_gpu(G2), S, X, U, beta=beta, eps=eps, p=4, iters=12, refresh=False)
    L2, R2 = oshampoo.accumulate_factors(G2, ref["L"], ref["R"], beta)
    assert torch.equal(X, X_before)
    assert rel_frobenius_error(S.cpu().numpy(), np.concatenate([L2, R2])).max() < 1e-5
    U_ref = oshampoo.precondition(ref["X_L"], G2, ref["X_R"])
    assert rel_frobenius_error(U.cpu().numpy(), U_ref).max() < 1e-4
    assert rel_max_abs_error(U.cpu().numpy(), U_ref).max() < max_abs_bar(1e-4)


def test_step_with_grafting_and_chunked_workspace(dash):
    import torch
    N, B = 5, 128
    # scalar parameters cross the C ABI as float: the oracle gets the same rounded values
    beta, eps, lr, beta_g, eps_g = 0.95, 1e-6, 1e-3, float(np.float32(0.999)), float(np.float32(1e-8))
    S = torch.zeros(2 * N, B, B, device="cuda")
    L64, R64 = np.zeros((N, B, B)), np.zeros((N, B, B))
    for t in range(5):
        G = workloads.gradient_stack(N, B, 3100 + t)
        dash.accumulate_factors(_to_gpu(G), S[:N], S[N:], beta)
        L64, R64 = oshampoo.accumulate_factors(G, L64, R64, beta)
    G = workloads.gradient_stack(N, B, 3200)
    theta0 = workloads.gradient_stack(N, B, 3300, std=1.0)
    acc0 = (workloads.gradient_stack(N, B, 3400, std=1e-2) ** 2).astype(np.float32)
    X = torch.zeros_like(S)
    U = torch.zeros(N, B, B, device="cuda")
    theta, acc = _to_gpu(theta0), _to_gpu(acc0)
    S2, X2, U2, theta2, acc2 = S.clone(), X.clone(), U.clone(), theta.clone(), acc.clone()
    dash.step(_to_gpu(G), S, X, U, beta=beta, eps=eps, p=4, iters=12, graft_acc=acc, theta=theta,
              beta_g=beta_g, eps_g=eps_g, lr=lr)
    ref = oshampoo.step(G, L64, R64, beta=beta, eps=eps, p=4,
                        graft=dict(Acc=acc0, beta_g=beta_g, eps_g=eps_g), theta=theta0, lr=lr)
    assert rel_frobenius_error(acc.cpu().numpy(), ref["Acc"]).max() < 1e-6
    assert rel_frobenius_error(U.cpu().numpy(), ref["U"]).max() < 1e-4
    assert rel_max_abs_error(U.cpu().numpy(), ref["U"]).max() < max_abs_bar(1e-4)
    # theta moved by lr * s * U: compare the movement, not theta itself
    moved = theta0.astype(np.float64) - theta.cpu().numpy().astype(np.float64)
    assert rel_frobenius_error(moved, lr * ref["s"][:, None, None] * ref["U"]).max() < 1e-3
    # by construction ||s U||_F = ||P||_F per block
    P = G.astype(np.float64) / (eps_g + np.sqrt(ref["Acc"]))
    for i in range(N):
        assert np.linalg.norm(moved[i]) / lr == pytest.approx(np.linalg.norm(P[i]), rel=1e-3)

    # same step through a workspace that holds 3 of the 10 factor blocks: same bits
    from paper_2602_02016_amd import Dash
    d2 = Dash(0)
    d2.step(_to_gpu(G), S2, X2, U2, beta=beta, eps=eps, p=4, iters=12, graft_acc=acc2, theta=theta2,
            beta_g=beta_g, eps_g=eps_g, lr=lr, workspace_max_bytes=d2.workspace_bytes(3, B))
    torch.cuda.synchronize()
    assert torch.equal(X, X2) and torch.equal(U, U2) and torch.equal(theta, theta2) and torch.equal(acc, acc2)
    d2.close()


def test_graft_update_alone(dash):
    import torch
    N, B = 3, 256
    G = workloads.gradient_stack(N, B, 3500)
    Uh = workloads.gradient_stack(N, B, 3501, std=1.0)
    acc0 = np.zeros((N, B, B), dtype=np.float32)
    acc = _to_gpu(acc0)
    s_out = torch.zeros(N, device="cuda")
    beta_g, eps_g = float(np.float32(0.999)), float(np.float32(1e-8))   # as the float ABI receives them
    dash.graft_update(_to_gpu(G), _to_gpu(Uh), acc, theta=None, beta_g=beta_g, eps_g=eps_g, s_out=s_out)
    Acc_ref, s_ref = oshampoo.adam_graft(G, Uh, acc0, beta_g, eps_g)
    assert np.allclose(acc.cpu().numpy(), Acc_ref, rtol=1e-6, atol=0)
    assert np.allclose(s_out.cpu().numpy(), s_ref, rtol=1e-5)


def test_graft_block_without_gradient_stays_finite(dash):
    """A gradient block that is all zero (rows of an embedding that saw no token) has U = 0 and P = 0: the grafting
    scale is taken as 0 there (Section 2.3 is silent), theta of that block does not move and nothing turns NaN."""
    import torch
    N, B = 3, 128
    G = workloads.gradient_stack(N, B, 3550)
    Uh = workloads.gradient_stack(N, B, 3551, std=1.0)
    G[1] = 0.0
    Uh[1] = 0.0
    theta0 = workloads.gradient_stack(N, B, 3552, std=1.0)
    acc0 = np.zeros((N, B, B), dtype=np.float32)
    acc, theta = _to_gpu(acc0), _to_gpu(theta0)
    s_out = torch.full((N,), -1.0, device="cuda")
    beta_g, eps_g, lr = float(np.float32(0.999)), float(np.float32(1e-8)), 1e-2
    dash.graft_update(_to_gpu(G), _to_gpu(Uh), acc, theta=theta, beta_g=beta_g, eps_g=eps_g, lr=lr, s_out=s_out)
    Acc_ref, s_ref = oshampoo.adam_graft(G, Uh, acc0, beta_g, eps_g)
    assert s_ref[1] == 0.0 and float(s_out[1]) == 0.0
    assert np.allclose(s_out.cpu().numpy(), s_ref, rtol=1e-5)
    th = theta.cpu().numpy()
    assert np.isfinite(th).all() and np.array_equal(th[1], theta0[1])
    assert not np.array_equal(th[0], theta0[0])
    scaled = dash.graft_scale(_to_gpu(G), _to_gpu(Uh), _to_gpu(acc0), beta_g=beta_g, eps_g=eps_g)
    assert bool(torch.isfinite(scaled).all()) and float(scaled[1].abs().max()) == 0.0


def test_step_chebyshev(dash):
    """The step with the Chebyshev root: compared with the oracle step that uses the float64
    Clenshaw evaluation of the same coefficients."""
    import torch
    from oracle import chebyshev as ocheb
    from paper_2602_02016_amd import chebyshev_fit
    N, B = 3, 128
    beta, eps, d = 0.95, 1e-6, 24
    S = torch.zeros(2 * N, B, B, device="cuda")
    L64, R64 = np.zeros((N, B, B)), np.zeros((N, B, B))
    for t in range(6):
        G = workloads.gradient_stack(N, B, 3600 + t)
        dash.accumulate_factors(_to_gpu(G), S[:N], S[N:], beta)
        L64, R64 = oshampoo.accumulate_factors(G, L64, R64, beta)
    G = workloads.gradient_stack(N, B, 3700)
    a, b = 0.005, 0.2          # scaled Wishart-EMA spectra sit around 0.02 .. 0.15 at B = 128
    coef = chebyshev_fit(4, d, a, b)
    X = torch.zeros_like(S)
    U = torch.zeros(N, B, B, device="cuda")
    dash.step(_to_gpu(G), S, X, U, beta=beta, eps=eps, method="chebyshev", p=4, iters=d, cheb_coeffs=coef,
              cheb_a=a, cheb_b=b)
    ref = oshampoo.step(G, L64, R64, beta=beta, eps=eps, p=4,
                        inverse_root=lambda S_, p_, e_: ocheb.inverse_root_chebyshev(S_, p_, np.array(coef), a, b, eps=e_))
    assert rel_frobenius_error(X.cpu().numpy(), np.concatenate([ref["X_L"], ref["X_R"]])).max() < 1e-4
    assert rel_frobenius_error(U.cpu().numpy(), ref["U"]).max() < 1e-4
    assert rel_max_abs_error(X.cpu().numpy(), np.concatenate([ref["X_L"], ref["X_R"]])).max() < max_abs_bar(1e-4)
    assert rel_max_abs_error(U.cpu().numpy(), ref["U"]).max() < max_abs_bar(1e-4)


def test_streaming_kernels_on_arrays_larger_than_the_caches(dash):
    """Calls that touch more than the last-level cache holds take a second form of the HBM-bound kernels
    (contiguous ranges per workgroup, non-temporal accesses).  80 blocks of 1024 x 1000 (ragged against the
    range length) and of 1024 x 1024: grafting, parameter update of a length that is not a multiple of four,
    Frobenius norms; against the float64 oracle on sampled blocks, the update bit for bit."""
    import torch
    N, B = 80, 1024
    beta_g, eps_g = float(np.float32(0.999)), float(np.float32(1e-8))
    rng = np.random.default_rng(3900)
    sample = [0, 37, N - 1]
    print("streaming forms: grafting", flush=True)
    for cols in (1000, 1024):
        G = (rng.standard_normal((N, B, cols)) * 1e-2).astype(np.float32)
        U = rng.standard_normal((N, B, cols)).astype(np.float32)
        A0 = (rng.random((N, B, cols)) * 1e-4).astype(np.float32)
        Gd, Ud, Ad = _to_gpu(G), _to_gpu(U), _to_gpu(A0)
        s_out = torch.zeros(N, device="cuda")
        out = torch.empty_like(Ud)
        dash.graft_scale(Gd, Ud, Ad, U_scaled=out, beta_g=beta_g, eps_g=eps_g, s_out=s_out)
        torch.cuda.synchronize()
        Acc_ref, s_ref = oshampoo.adam_graft(G[sample], U[sample], A0[sample], beta_g, eps_g)
        assert np.allclose(Ad[sample].cpu().numpy(), Acc_ref, rtol=1e-6, atol=0)
        assert np.allclose(s_out[sample].cpu().numpy(), s_ref, rtol=1e-5)
        got = out[sample].cpu().numpy()
        assert np.allclose(got, s_ref[:, None, None] * U[sample].astype(np.float64), rtol=2e-5, atol=0)
        del Gd, Ud, Ad, out
    print("streaming forms: parameter update", flush=True)
    n = N * B * B - 5
    t = rng.standard_normal(n).astype(np.float32)
    tg = torch.from_numpy(t).cuda()
    ug = _to_gpu(U).reshape(-1)[:n]
    dash.apply_update(tg, ug, 0.25)
    assert np.array_equal(tg.cpu().numpy(), t - np.float32(0.25) * U.reshape(-1)[:n])
    print("streaming forms: norms", flush=True)
    fro = dash.block_norms(_to_gpu(U), eps=1e-3, scaling="frobenius").cpu().numpy()
    for b in sample:
        ref = np.linalg.norm(U[b].astype(np.float64) + 1e-3 * np.eye(B))
        assert abs(fro[b] - ref) <= 2e-6 * ref
