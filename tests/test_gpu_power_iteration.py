"""Multi-Power-Iteration scaling (paper Sections 3.4, 3.5) through the C ABI against the
float64 oracle: the scale s = 2 lambda_PI itself, and Newton-DB run with it."""
import numpy as np
import pytest

import workloads
from oracle import newton_db as ondb
from oracle import power_iteration as opi
from oracle.evd import inverse_root_evd, rel_frobenius_error

pytestmark = pytest.mark.gpu


@pytest.fixture()
def dash():
    from paper_2602_02016_amd import Dash
    d = Dash(0)
    yield d
    d.close()


def _to_gpu(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


@pytest.mark.parametrize("N,B", [(3, 64), (5, 128), (4, 256), (3, 512), (33, 1024), (2, 2048)])
@pytest.mark.parametrize("pool,sweeps", [(16, 1), (16, 4), (32, 8), (5, 3)])
def test_scale_matches_oracle(dash, N, B, pool, sweeps):
    print(f"pi scale N={N} B={B} pool={pool} sweeps={sweeps}", flush=True)
    A32, _, lam = workloads.spd_stack(N, B, -3.0, 0.0, seed=91 + B, share_q=True)
    V0 = workloads.start_vectors(B, pool, 93)
    eps = 1e-3
    dash.set_power_iteration(_to_gpu(V0), sweeps)
    s = dash.block_norms(_to_gpu(A32), eps=eps, scaling="power_iteration").cpu().numpy()
    sample = sorted(set([0, N // 2, N - 1]))
    s_ref = opi.power_iteration_scale(A32[sample].astype(np.float64), V0.astype(np.float64), sweeps, eps)
    assert np.allclose(s[sample], s_ref, rtol=2e-5)
    # Rayleigh quotients never exceed lambda_max: s <= 2 (lambda_max + eps), for every block
    assert np.all(s <= 2 * (lam.max(axis=1) + eps) * (1 + 1e-5))
    assert np.all(s > 0)


@pytest.mark.parametrize("pool", [16, 32])
def test_scale_on_a_stack_larger_than_the_cache(dash, pool):
    """From 256 MiB on the sweep reads the blocks with the non-temporal hint (second instances of the 16-wide and
    of the 32-wide kernel)."""
    N, B, sweeps, eps = 65, 1024, 4, 1e-3
    print(f"pi scale N={N} B={B} (streaming form)", flush=True)
    A32, _, lam = workloads.spd_stack(N, B, -3.0, 0.0, seed=98, share_q=True)
    V0 = workloads.start_vectors(B, pool, 99)
    dash.set_power_iteration(_to_gpu(V0), sweeps)
    s = dash.block_norms(_to_gpu(A32), eps=eps, scaling="power_iteration").cpu().numpy()
    sample = [0, 31, N - 1]
    s_ref = opi.power_iteration_scale(A32[sample].astype(np.float64), V0.astype(np.float64), sweeps, eps)
    assert np.allclose(s[sample], s_ref, rtol=2e-5)
    assert np.all(s <= 2 * (lam.max(axis=1) + eps) * (1 + 1e-5)) and np.all(s > 0)


def test_scale_converges_to_twice_lambda_max(dash):
    N, B = 4, 256
    A32, _, lam = workloads.spd_stack(N, B, -2.0, 0.0, seed=95)
    dash.set_power_iteration(_to_gpu(workloads.start_vectors(B, 32, 96)), 200)
    s = dash.block_norms(_to_gpu(A32), scaling="pi").cpu().numpy()
    lam_max = np.array([np.linalg.eigvalsh(A32[i].astype(np.float64)).max() for i in range(N)])
    assert np.allclose(s, 2 * lam_max, rtol=1e-4)


def test_larger_rows_of_start_vectors_and_errors(dash):
    import torch
    from paper_2602_02016_amd import DashError
    A32, _, _ = workloads.spd_stack(2, 128, -1.0, 0.0, seed=97)
    A = _to_gpu(A32)
    with pytest.raises(DashError) as ei:                      # not configured yet
        dash.block_norms(A, scaling="pi")
    assert ei.value.status == 1
    V0 = workloads.start_vectors(256, 16, 98)                  # more rows than B: the first B rows are used
    dash.set_power_iteration(_to_gpu(V0), 3)
    s = dash.block_norms(A, scaling="pi").cpu().numpy()
    s_ref = opi.power_iteration_scale(A32.astype(np.float64), V0[:128].astype(np.float64), 3)
    assert np.allclose(s, s_ref, rtol=2e-5)
    dash.set_power_iteration(_to_gpu(workloads.start_vectors(64, 16, 99)), 3)
    with pytest.raises(DashError):                             # fewer rows than B
        dash.block_norms(A, scaling="pi")
    for bad in (dict(pool=0), dict(pool=33), dict(sweeps=0)):
        kw = dict(pool=16, sweeps=2); kw.update(bad)
        v = torch.zeros(128, max(kw["pool"], 1), device="cuda")
        st = dash.lib.dash_set_power_iteration(dash.h, kw["pool"], kw["sweeps"], v.data_ptr(), 128)
        assert st == 1


@pytest.mark.parametrize("p", [2, 4])
@pytest.mark.parametrize("N,B", [(4, 128), (3, 512), (5, 1024)])
def test_ndb_with_power_iteration_scaling(dash, N, B, p):
    """Flat spectrum in [0.5, 1] (||A||_F ~ 0.76 sqrt(B) lambda_max): with s = 2 lambda_PI six
    iterations reach the root, with Frobenius scaling they do not (the paper's Section 3.4 point)."""
    Q = workloads.orthogonal_factor(B, 101)
    A64 = np.stack([workloads.spd_from_spectrum(Q, np.linspace(0.5, 1.0, B) * (1 + 0.1 * i)) for i in range(N)])
    A32 = A64.astype(np.float32)
    V0 = workloads.start_vectors(B, 16, 102)
    k, sweeps = 6, 5
    dash.set_power_iteration(_to_gpu(V0), sweeps)
    s_out = _to_gpu(np.zeros(N, dtype=np.float32))
    X_pi = dash.inverse_root(_to_gpu(A32), p=p, iters=k, eps=1e-6, scaling="power_iteration", scale_out=s_out)
    X_fro = dash.inverse_root(_to_gpu(A32), p=p, iters=k, eps=1e-6, scaling="frobenius")
    X_pi, X_fro = X_pi.cpu().numpy(), X_fro.cpu().numpy()
    sample = [0, N - 1]
    A_s = A32[sample].astype(np.float64)
    X_same = ondb.inverse_root_ndb(A_s, p, k, eps=1e-6, scaling="power_iteration", pi=(V0.astype(np.float64), sweeps))
    X_evd = inverse_root_evd(A_s, p, eps=1e-6)
    e_same = rel_frobenius_error(X_pi[sample], X_same).max()
    e_pi = rel_frobenius_error(X_pi[sample], X_evd).max()
    e_fro = rel_frobenius_error(X_fro[sample], X_evd).max()
    print(f"ndb+pi N={N} B={B} p={p}: vs float64 same method {e_same:.2e}; vs EVD: pi {e_pi:.2e}, frobenius {e_fro:.2e}",
          flush=True)
    assert e_same < 2e-5
    assert e_pi < 1e-4 and e_fro > 20 * e_pi
    s_ref = opi.power_iteration_scale(A_s + 1e-6 * np.eye(B), V0.astype(np.float64), sweeps)
    assert np.allclose(s_out.cpu().numpy()[sample], s_ref, rtol=2e-5)


def test_step_with_power_iteration_scaling(dash):
    import torch
    from oracle import shampoo as oshampoo
    N, B = 3, 256
    beta, eps = 0.95, 1e-6
    S = torch.zeros(2 * N, B, B, device="cuda")
    L64, R64 = np.zeros((N, B, B)), np.zeros((N, B, B))
    for t in range(5):
        G = workloads.gradient_stack(N, B, 9100 + t)
        dash.accumulate_factors(_to_gpu(G), S[:N], S[N:], beta)
        L64, R64 = oshampoo.accumulate_factors(G, L64, R64, beta)
    G = workloads.gradient_stack(N, B, 9200)
    dash.set_power_iteration(_to_gpu(workloads.start_vectors(B, 16, 103)), 6)
    X = torch.zeros_like(S); U = torch.zeros(N, B, B, device="cuda")
    dash.step(_to_gpu(G), S, X, U, beta=beta, eps=eps, p=4, iters=8, scaling="power_iteration")
    ref = oshampoo.step(G, L64, R64, beta=beta, eps=eps, p=4)
    assert rel_frobenius_error(X.cpu().numpy(), np.concatenate([ref["X_L"], ref["X_R"]])).max() < 1e-4
    assert rel_frobenius_error(U.cpu().numpy(), ref["U"]).max() < 1e-4


def test_power_iteration_scaling_saves_iterations_on_wishart_factors(dash):
    """The paper's Section 3.4 argument on the benchmark's kind of factor (EMA of G G^T, eigenvalues near
    ||L||_F / sqrt(B)): scaled by 2 lambda_PI, Newton-DB with five updates per call is converged to the fp32
    floor, scaled by the Frobenius norm it is still far off and needs eight."""
    import torch
    N, B, eps = 4, 512, 1e-6
    S = torch.zeros(2 * N, B, B, device="cuda")
    for t in range(20):
        G = torch.from_numpy(workloads.gradient_stack(N, B, 3000 + t)).cuda()
        dash.accumulate_factors(G, S[:N], S[N:], 0.95)
    X_evd = inverse_root_evd(S.cpu().numpy().astype(np.float64), 4, eps)
    V0 = torch.from_numpy(workloads.start_vectors(B, 16, 77)).cuda()
    dash.set_power_iteration(V0, 4)
    err = {}
    for scaling in ("frobenius", "pi"):
        for k in (5, 8):
            X = dash.inverse_root(S, p=4, iters=k, eps=eps, scaling=scaling).cpu().numpy()
            err[scaling, k] = rel_frobenius_error(X, X_evd).max()
    print({f"{a} k={k}": f"{e:.1e}" for (a, k), e in err.items()}, flush=True)
    assert err["pi", 5] < 1e-4 and err["frobenius", 5] > 1e-2 and err["frobenius", 8] < 1e-4
