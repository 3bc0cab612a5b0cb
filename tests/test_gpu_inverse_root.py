"""Parity of dash_inverse_root / dash_block_norms (HIP, through the C ABI) with the float64
oracle: element-by-element against the same method in float64 (same iteration count, so
the comparison isolates fp32 rounding) and against the eigendecomposition root."""
import numpy as np
import pytest

import workloads
from oracle import chebyshev as ocheb
from oracle import newton_db as ondb
from oracle.evd import inverse_root_evd, rel_frobenius_error
from tolerances import fp32_floor, max_abs_bar, rel_max_abs_error

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


# ---- scaling ------------------------------------------------------------------------------

@pytest.mark.parametrize("N,B", [(3, 64), (5, 128), (2, 512), (3, 1024)])
def test_block_norms(dash, N, B):
    A32, _, lam = workloads.spd_stack(N, B, -3.0, 0.0, seed=20 + B, share_q=True)
    A = A32.astype(np.float64)
    eps = 1e-3
    Ad = A + eps * np.eye(B)
    fro = dash.block_norms(_to_gpu(A32), eps=eps, scaling="frobenius").cpu().numpy()
    tr = dash.block_norms(_to_gpu(A32), eps=eps, scaling="trace").cpu().numpy()
    one = dash.block_norms(_to_gpu(A32), eps=eps, scaling="none").cpu().numpy()
    assert np.allclose(fro, np.sqrt((Ad ** 2).sum(axis=(1, 2))), rtol=2e-6)
    assert np.allclose(tr, np.trace(Ad, axis1=1, axis2=2), rtol=2e-6)
    assert np.all(one == 1.0)
    assert np.all(lam.max(axis=1) + eps <= fro * (1 + 1e-6)) and np.all(fro <= tr * (1 + 1e-6))


# ---- Newton-DB ------------------------------------------------------------------------------

@pytest.mark.parametrize("p", [2, 4])
@pytest.mark.parametrize("k", [10, 12, 15])
def test_ndb_config1(dash, p, k):
    """N=16, B=128, spectrum log-uniform in [1e-3, 1] (kappa = 1e3)."""
    c = workloads.CFG1
    A32, Q, lam = workloads.spd_stack(c["N"], c["B"], c["lo_exp"], c["hi_exp"], c["seed"])
    X = dash.inverse_root(_to_gpu(A32), p=p, iters=k).cpu().numpy()
    A = A32.astype(np.float64)
    X_same = ondb.inverse_root_ndb(A, p, k)
    X_evd = inverse_root_evd(A, p)
    e_same = rel_frobenius_error(X, X_same)
    e_evd = rel_frobenius_error(X, X_evd)
    e_model = rel_frobenius_error(X_same, X_evd)
    print(f"cfg1 p={p} k={k}: vs f64 same-k max {e_same.max():.2e}; vs EVD max {e_evd.max():.2e} "
          f"(f64 model {e_model.max():.2e})", flush=True)
    floor = fp32_floor(1e3, p, c["B"])          # derived on the CPU: tests/test_fp32_floor.py
    assert e_same.max() < floor
    # element by element, scaled by the largest entry of the reference block: the same bar
    m_same = rel_max_abs_error(X, X_same)
    print(f"   largest element-wise deviation / max|X_ref|: {m_same.max():.2e} (bar {max_abs_bar(floor):.2e})", flush=True)
    assert m_same.max() < max_abs_bar(floor)
    # distance to the true root = truncation error of the method, up to the fp32 floor
    assert np.all(np.abs(e_evd - e_model) <= 0.1 * e_model + floor)
    # the closed form known by construction (no eigensolver): same statement
    X_true = np.stack([(Q[i] * lam[i] ** (-1.0 / p)) @ Q[i].T for i in range(c["N"])])
    assert np.all(np.abs(rel_frobenius_error(X, X_true) - e_model) <= 0.1 * e_model + 2 * floor)


@pytest.mark.parametrize("p", [2, 4])
@pytest.mark.parametrize("N,B", [(5, 64), (16, 128), (5, 256), (3, 512), (2, 1024)])
def test_ndb_well_conditioned_meets_1e4(dash, N, B, p):
    """Spectra in [0.1, 1]: k = 10 converges and the fp32 result is within 1e-4 of the EVD root."""
    print(f"ndb well-conditioned N={N} B={B} p={p}", flush=True)
    A32, Q, lam = workloads.spd_stack(N, B, -1.0, 0.0, seed=30 + B, share_q=B >= 512)
    nf = _to_gpu(np.full(N, 7, dtype=np.int32))
    X = dash.inverse_root(_to_gpu(A32), p=p, iters=10, eps=1e-6, nonfinite_out=nf).cpu().numpy()
    X_evd = inverse_root_evd(A32.astype(np.float64), p, eps=1e-6)
    e = rel_frobenius_error(X, X_evd)
    m = rel_max_abs_error(X, X_evd)
    print(f"   max rel err vs EVD {e.max():.2e}, largest element-wise deviation / max|X_ref| {m.max():.2e}", flush=True)
    assert e.max() < 1e-4
    assert m.max() < max_abs_bar(1e-4)
    assert np.all(nf.cpu().numpy() == 0)
    # defining identity X^p (A + eps I) = I, computed in float64 from the GPU result
    Xd = X.astype(np.float64)
    Ad = A32.astype(np.float64) + 1e-6 * np.eye(B)
    res = np.linalg.matrix_power(Xd[0], p) @ Ad[0] - np.eye(B)
    assert np.linalg.norm(res) / np.sqrt(B) < 1e-3
    assert np.linalg.norm(Xd[0] - Xd[0].T) / np.linalg.norm(Xd[0]) < 1e-5


@pytest.mark.parametrize("k", [1, 2, 3])
@pytest.mark.parametrize("p", [2, 4])
def test_ndb_few_iterations_match_float64_iteration(dash, p, k):
    """k = 1 uses no product for p = 2 (closed-form Z_1) -- all small k must match the same
    iteration in float64 even though they are far from the root."""
    N, B = 3, 128
    A32, _, _ = workloads.spd_stack(N, B, -2.0, 0.0, seed=41)
    X = dash.inverse_root(_to_gpu(A32), p=p, iters=k, eps=1e-4).cpu().numpy()
    X_same = ondb.inverse_root_ndb(A32.astype(np.float64), p, k, eps=1e-4)
    assert rel_frobenius_error(X, X_same).max() < 1e-5
    assert rel_max_abs_error(X, X_same).max() < max_abs_bar(1e-5)


@pytest.mark.parametrize("scaling", ["trace", "none"])
def test_ndb_other_scalings(dash, scaling):
    N, B, p, k = 4, 128, 4, 14
    A32, _, _ = workloads.spd_stack(N, B, -1.0, 0.0, seed=43)
    if scaling == "none":
        A32 = (A32 * 0.9).astype(np.float32)          # spectrum already inside (0, 1]
    s_out = _to_gpu(np.zeros(N, dtype=np.float32))
    X = dash.inverse_root(_to_gpu(A32), p=p, iters=k, scaling=scaling, scale_out=s_out).cpu().numpy()
    X_same = ondb.inverse_root_ndb(A32.astype(np.float64), p, k, scaling=scaling)
    assert rel_frobenius_error(X, X_same).max() < 1e-5
    assert rel_max_abs_error(X, X_same).max() < max_abs_bar(1e-5)
    s_ref = [ondb.block_scale(A32[i].astype(np.float64), scaling) for i in range(N)]
    assert np.allclose(s_out.cpu().numpy(), s_ref, rtol=2e-6)


def test_ndb_matmul_counts_and_chunking(dash):
    """Products per block: each call spends 1 (closed-form start) + 3 per further iteration,
    minus the one iterate of the last iteration that is never used: 3k-3 for k >= 2.
    The paper's count for the unoptimised tail is 3k-2 per call (Section 3.3)."""
    import torch
    from paper_2602_02016_amd import Dash
    N, B = 7, 128
    A32, _, _ = workloads.spd_stack(N, B, -1.0, 0.0, seed=47)
    A = _to_gpu(A32)
    for p, calls in ((2, 1), (4, 2)):
        for k in (2, 5, 10):
            dash.reset_stats()
            X = dash.inverse_root(A, p=p, iters=k)
            st = dash.get_stats()
            assert st["matmul_products"] == calls * (3 * k - 3)
            assert st["matmul_block_products"] == calls * (3 * k - 3) * N
    dash.reset_stats()
    dash.inverse_root(A, p=2, iters=1)
    assert dash.get_stats()["matmul_products"] == 0
    dash.reset_stats()
    dash.inverse_root(A, p=4, iters=1)
    assert dash.get_stats()["matmul_products"] == 1
    # a workspace that holds 3 blocks: chunks of 3, 3, 1 -- same bits as one chunk
    X_full = dash.inverse_root(A, p=4, iters=6)
    d2 = Dash(0)
    X_chunk = d2.inverse_root(A, p=4, iters=6, workspace_max_bytes=d2.workspace_bytes(3, B))
    torch.cuda.synchronize()
    assert torch.equal(X_full, X_chunk)
    # too small for one block: clean error, no launch
    d3 = Dash(0)
    d3.set_workspace_bytes(1024)
    from paper_2602_02016_amd import DashError
    with pytest.raises(DashError) as ei:
        d3._check(d3.lib.dash_inverse_root(d3.h, d3._stack(A, "A"), d3._stack(X_chunk, "X"), N, B, 0, 4, 5, 0.0, 0, 0,
                                           None, 0.0, 1.0, None, None))
    assert ei.value.status == 3
    d2.close(); d3.close()


def test_invalid_arguments_are_rejected(dash):
    import torch
    from paper_2602_02016_amd import DashError
    A = torch.zeros(2, 128, 128, device="cuda")
    X = torch.zeros_like(A)
    for kw in (dict(p=3), dict(iters=0), dict(method="chebyshev", iters=1, cheb_coeffs=[1.0, 0.0]),
               dict(method="chebyshev", iters=4), dict(eps=-1.0)):
        with pytest.raises(DashError) as ei:
            dash.inverse_root(A, X, **kw)
        assert ei.value.status == 1
    with pytest.raises(DashError):
        dash.inverse_root(A, A)                                  # output aliases input
    with pytest.raises(DashError):
        dash.inverse_root(torch.zeros(2, 100, 100, device="cuda"))   # B not a multiple of 64


def test_nonfinite_blocks_are_flagged_not_hidden(dash):
    N, B = 5, 128
    A32, _, _ = workloads.spd_stack(N, B, -1.0, 0.0, seed=53)
    A32[1, 3, 3] = np.nan
    A32[3, 0, 5] = np.inf
    nf = _to_gpu(np.zeros(N, dtype=np.int32))
    X = dash.inverse_root(_to_gpu(A32), p=4, iters=6, nonfinite_out=nf).cpu().numpy()
    assert list(nf.cpu().numpy()) == [0, 1, 0, 1, 0]
    assert np.isfinite(X[[0, 2, 4]]).all() and not np.isfinite(X[1]).all()
    with pytest.raises(ValueError):
        inverse_root_evd(np.nan_to_num(A32[1].astype(np.float64), nan=-5.0) - 10 * np.eye(B), 4)


# ---- Chebyshev / Clenshaw -------------------------------------------------------------------

@pytest.mark.parametrize("p", [2, 4])
@pytest.mark.parametrize("d", [2, 3, 8, 16, 32])
def test_chebyshev_matches_float64_clenshaw(dash, p, d):
    from paper_2602_02016_amd import chebyshev_fit
    N, B = 5, 128
    A32, Q, lam = workloads.spd_stack(N, B, -1.0, 0.0, seed=61)
    A = A32.astype(np.float64)
    s = np.sqrt((A ** 2).sum(axis=(1, 2)))
    a, b = float((lam.min(axis=1) / s).min()) * 0.99, 1.0
    c_lib = chebyshev_fit(p, d, a, b)
    c_ref = ocheb.chebyshev_fit(p, d, a, b)
    assert np.allclose(c_lib, c_ref, rtol=0, atol=1e-12)
    dash.reset_stats()
    X = dash.inverse_root(_to_gpu(A32), method="chebyshev", p=p, iters=d, cheb_coeffs=c_lib, cheb_a=a, cheb_b=b)
    assert dash.get_stats()["matmul_products"] == d - 1
    X = X.cpu().numpy()
    X_same = ocheb.inverse_root_chebyshev(A, p, c_ref, a, b)
    e_same = rel_frobenius_error(X, X_same)
    e_evd = rel_frobenius_error(X, inverse_root_evd(A, p))
    e_model = rel_frobenius_error(X_same, inverse_root_evd(A, p))
    print(f"cheb p={p} d={d}: vs f64 Clenshaw {e_same.max():.2e}; vs EVD {e_evd.max():.2e} (model {e_model.max():.2e})",
          flush=True)
    assert e_same.max() < 1e-5
    assert rel_max_abs_error(X, X_same).max() < max_abs_bar(1e-5)
    assert np.all(np.abs(e_evd - e_model) <= 0.1 * e_model + 1e-5)


def test_chebyshev_config1_and_paper_interval(dash):
    """cfg 1 with degree 16, in the paper's own form: map of [0,1] with coefficients fitted
    on [eps, 1+eps] (Appendix A.2), and with an interval that hugs the spectrum."""
    from paper_2602_02016_amd import chebyshev_fit
    c = workloads.CFG1
    A32, Q, lam = workloads.spd_stack(c["N"], c["B"], c["lo_exp"], c["hi_exp"], c["seed"])
    A = A32.astype(np.float64)
    d, p, e = c["cheb_degree"], 4, 1e-3
    coef = chebyshev_fit(p, d, e, 1.0 + e)
    X = dash.inverse_root(_to_gpu(A32), method="chebyshev", p=p, iters=d, cheb_coeffs=coef, cheb_a=0.0, cheb_b=1.0)
    X_same = ocheb.inverse_root_chebyshev(A, p, np.array(coef), 0.0, 1.0)
    assert rel_frobenius_error(X.cpu().numpy(), X_same).max() < 1e-5
    assert rel_max_abs_error(X.cpu().numpy(), X_same).max() < max_abs_bar(1e-5)
    s = np.sqrt((A ** 2).sum(axis=(1, 2)))
    a = float((lam.min(axis=1) / s).min())
    coef2 = chebyshev_fit(p, d, a, 1.0)
    X2 = dash.inverse_root(_to_gpu(A32), method="chebyshev", p=p, iters=d, cheb_coeffs=coef2, cheb_a=a, cheb_b=1.0)
    X2_same = ocheb.inverse_root_chebyshev(A, p, np.array(coef2), a, 1.0)
    assert rel_frobenius_error(X2.cpu().numpy(), X2_same).max() < 1e-5
    assert rel_max_abs_error(X2.cpu().numpy(), X2_same).max() < max_abs_bar(1e-5)
    e2 = rel_frobenius_error(X2.cpu().numpy(), inverse_root_evd(A, p)).max()
    print(f"cfg1 chebyshev d=16: err vs EVD with [lmin/s,1] = {e2:.2e}", flush=True)
