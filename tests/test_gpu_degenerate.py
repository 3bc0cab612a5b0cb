"""Degenerate inputs with closed-form inverse roots, through the C ABI: multiples of the identity, the zero
matrix with damping, diagonal blocks, rank-one plus damping (the factor after the first Shampoo step), and
blocks of wildly different magnitude in one stack (the scaling is per block)."""
import numpy as np
import pytest

from oracle.evd import rel_frobenius_error

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dash():
    from paper_2602_02016_amd import Dash
    d = Dash(0)
    yield d
    d.close()


def _to_gpu(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


@pytest.mark.parametrize("method,iters", [("newton_db", 25), ("coupled_newton", 40)])
@pytest.mark.parametrize("p", [2, 4])
def test_identity_multiples_zero_and_mixed_magnitudes(dash, method, iters, p):
    B = 256
    I = np.eye(B)
    scales = [1.0, 1e-6, 1e6, 3.7e-3, 0.0]                    # the last block is the zero matrix
    eps = 1e-4
    A = np.stack([c * I for c in scales])
    nf = _to_gpu(np.zeros(len(scales))).int()
    X = dash.inverse_root(_to_gpu(A), method=method, p=p, iters=iters, eps=eps, nonfinite_out=nf).cpu().numpy()
    for i, c in enumerate(scales):
        want = (np.float64(np.float32(c) + np.float32(eps))) ** (-1.0 / p)
        off = X[i] - np.diag(np.diag(X[i]))
        assert np.abs(off).max() <= 1e-6 * want, (i, c)
        assert np.allclose(np.diag(X[i]), want, rtol=2e-5), (i, c, np.diag(X[i])[:3], want)
    assert int(nf.sum().item()) == 0


@pytest.mark.parametrize("p", [2, 4])
def test_diagonal_blocks(dash, p):
    B, N = 128, 3
    rng = np.random.default_rng(5)
    lam = 10.0 ** rng.uniform(-2, 0, size=(N, B))
    A = np.stack([np.diag(l) for l in lam])
    X = dash.inverse_root(_to_gpu(A), method="newton_db", p=p, iters=20).cpu().numpy()
    for i in range(N):
        want = np.float32(lam[i]).astype(np.float64) ** (-1.0 / p)
        assert np.abs(X[i] - np.diag(np.diag(X[i]))).max() <= 1e-6 * want.max()
        assert np.allclose(np.diag(X[i]), want, rtol=1e-4)


def test_rank_one_plus_damping(dash):
    """(a g g^T + eps I)^(-1/4) = eps^(-1/4) (I - u u^T) + (a |g|^2 + eps)^(-1/4) u u^T with u = g / |g|."""
    B, N = 256, 4
    rng = np.random.default_rng(11)
    a, eps = 0.05, 1e-3
    g = rng.standard_normal((N, B)) * 0.1
    A = a * g[:, :, None] * g[:, None, :]
    A32 = A.astype(np.float32)
    X = dash.inverse_root(_to_gpu(A32), method="newton_db", p=4, iters=30, eps=eps).cpu().numpy()
    eps32 = float(np.float32(eps))
    for i in range(N):
        # closed form on the matrix the GPU received: its rank-one part is fp32-rounded, so take u and the
        # top eigenvalue from it in float64 (one eigenvector; the rest of the spectrum is numerically eps)
        w, V = np.linalg.eigh(A32[i].astype(np.float64))
        u, top = V[:, -1], w[-1]
        want = eps32 ** -0.25 * (np.eye(B) - np.outer(u, u)) + (top + eps32) ** -0.25 * np.outer(u, u)
        assert rel_frobenius_error(X[i][None], want[None]).max() < 2e-4


def test_chebyshev_on_identity_multiple(dash):
    from paper_2602_02016_amd import chebyshev_fit
    B = 128
    A = np.stack([0.5 * np.eye(B), 2.0 * np.eye(B)])
    # after Frobenius scaling every eigenvalue is 1 / sqrt(B); fit on an interval around it
    x = 1.0 / np.sqrt(B)
    c = chebyshev_fit(4, 24, 0.5 * x, 2.0 * x)
    X = dash.inverse_root(_to_gpu(A), method="chebyshev", p=4, iters=24, cheb_coeffs=c, cheb_a=0.5 * x, cheb_b=2.0 * x).cpu().numpy()
    for i, cst in enumerate((0.5, 2.0)):
        assert np.allclose(np.diag(X[i]), cst ** -0.25, rtol=1e-4)
        assert np.abs(X[i] - np.diag(np.diag(X[i]))).max() < 1e-6
