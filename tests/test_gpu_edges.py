"""Edges of the argument space: empty stacks, a single smallest block, stacks longer than one grid dimension
(more than 65535 blocks), one very large block."""
import ctypes as C

import numpy as np
import pytest

import workloads
from oracle import newton_db as ondb
from oracle import shampoo as oshampoo
from oracle.evd import rel_frobenius_error
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


def test_empty_stacks_are_no_ops(dash):
    """N = 0 returns DASH_OK from every stack entry point and touches nothing (null pointers are accepted)."""
    null = C.c_void_p(None)
    lib, h = dash.lib, dash.h
    assert lib.dash_gemm_batched(h, 0, 0, null, null, null, null, 0, 128, 1.0, 0.0, 0.0, 0) == 0
    assert lib.dash_accumulate_factors(h, null, null, null, 0, 128, 0.95, 0.05) == 0
    assert lib.dash_accumulate_factors_rect(h, null, null, null, 0, 128, 64, 0.95, 0.05) == 0
    assert lib.dash_precondition(h, null, null, null, null, 0, 128) == 0
    assert lib.dash_precondition_rect(h, null, null, null, null, 0, 128, 64) == 0
    assert lib.dash_accumulate_vector(h, null, null, 0, 128, 0.95, 0.05) == 0
    assert lib.dash_precondition_vector(h, null, null, null, 0, 128) == 0
    assert lib.dash_block_norms(h, null, 0, 128, 0.0, 0, null) == 0
    assert lib.dash_block_norms_static(h, null, 0, 128, 0.0, 0, null) == 0
    assert lib.dash_inverse_root(h, null, null, 0, 128, 0, 4, 10, 0.0, 0, 0, None, 0.0, 1.0, null, null) == 0
    assert lib.dash_graft_update(h, null, null, null, null, 0, 128, 0.999, 1e-8, 0.0, null) == 0
    assert lib.dash_graft_scale(h, null, null, null, 0, 4096, 0.999, 1e-8, null, null) == 0
    assert lib.dash_apply_update(h, null, null, 0, 0.1) == 0


def test_one_smallest_block_through_the_step(dash):
    import torch
    N, B, beta, eps = 1, 64, 0.9, 1e-6
    S = torch.zeros(2, B, B, device="cuda")
    L64, R64 = np.zeros((1, B, B)), np.zeros((1, B, B))
    for t in range(8):
        G = workloads.gradient_stack(N, B, 9100 + t)
        dash.accumulate_factors(_to_gpu(G), S[:1], S[1:], beta)
        L64, R64 = oshampoo.accumulate_factors(G, L64, R64, beta)
    G = workloads.gradient_stack(N, B, 9200)
    X = torch.zeros_like(S); U = torch.zeros(1, B, B, device="cuda")
    dash.step(_to_gpu(G), S, X, U, beta=beta, eps=eps, p=4, iters=14)
    ref = oshampoo.step(G, L64, R64, beta=beta, eps=eps, p=4)
    assert rel_frobenius_error(X.cpu().numpy(), np.concatenate([ref["X_L"], ref["X_R"]])).max() < 1e-4
    assert rel_frobenius_error(U.cpu().numpy(), ref["U"]).max() < 1e-4
    assert rel_max_abs_error(U.cpu().numpy(), ref["U"]).max() < max_abs_bar(1e-4)


def test_more_blocks_than_one_grid_dimension(dash):
    """70 000 blocks of 64 x 64: the elementwise kernels walk the stack in slices of 65535 blocks (one grid
    dimension) and the matmul grid has millions of workgroups.  Blocks on both sides of the slice boundary and the
    last block against the float64 iteration; every block finite, no block flagged."""
    import torch
    N, B, p, k = 70000, 64, 2, 4
    base, _, _ = workloads.spd_stack(8, B, -1.0, 0.0, seed=77)
    A = _to_gpu(base).repeat(N // 8, 1, 1).contiguous()
    shift = (torch.arange(N, device="cuda", dtype=torch.float32) % 97) * 1e-3
    A += shift[:, None, None] * torch.eye(B, device="cuda")
    nf = torch.ones(N, dtype=torch.int32, device="cuda")
    s_out = torch.zeros(N, device="cuda")
    X = dash.inverse_root(A, p=p, iters=k, eps=1e-6, nonfinite_out=nf, scale_out=s_out)
    torch.cuda.synchronize()
    assert int(nf.sum().item()) == 0 and bool(torch.isfinite(X).all())
    sample = [0, 65534, 65535, 65536, N - 1]
    A_s = A[sample].cpu().numpy().astype(np.float64)
    X_ref = ondb.inverse_root_ndb(A_s, p, k, eps=1e-6)
    assert rel_frobenius_error(X[sample].cpu().numpy(), X_ref).max() < 1e-5
    s_ref = np.sqrt(((A_s + 1e-6 * np.eye(B)) ** 2).sum(axis=(1, 2)))
    assert np.allclose(s_out[sample].cpu().numpy(), s_ref, rtol=2e-6)
    norms = dash.block_norms(A, eps=1e-6)
    assert torch.equal(norms, s_out)


def test_one_very_large_block(dash):
    """A single 4096 x 4096 block (K loop of 256 slabs, 1024 tiles per product): few Newton-DB updates against the
    same iteration in float64."""
    import torch
    B, p, k = 4096, 2, 3
    A32, _, _ = workloads.spd_stack(1, B, -1.0, 0.0, seed=78, share_q=True)
    X = dash.inverse_root(_to_gpu(A32), p=p, iters=k, eps=1e-6).cpu().numpy()
    X_ref = ondb.inverse_root_ndb(A32.astype(np.float64), p, k, eps=1e-6)
    bar = fp32_floor(10.0, p, B)            # dot products of 4096 terms: the floor law's (B/256)^0.75 factor is 8
    e, m = rel_frobenius_error(X, X_ref).max(), rel_max_abs_error(X, X_ref).max()
    print(f"B={B}: vs float64 same-k {e:.2e} (element-wise {m:.2e}), bar {bar:.2e}", flush=True)
    assert e < bar and m < max_abs_bar(bar)
