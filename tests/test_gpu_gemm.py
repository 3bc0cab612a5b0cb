"""Parity of the batched matmul primitive and of the calls that are a single product
with an epilogue (accumulate, precondition) against float64 numpy, through the C ABI."""
import numpy as np
import pytest

import workloads
from oracle import shampoo as oracle_shampoo
from oracle.evd import rel_frobenius_error

pytestmark = pytest.mark.gpu

# fp32 products with fp32 accumulation over K = B terms: relative Frobenius error of a
# product of random matrices grows like sqrt(B) * 2^-24 at worst; 1e-5 covers B <= 2048.
TOL_MM = 1e-5


@pytest.fixture(scope="module")
def dash():
    from paper_2602_02016_amd import Dash
    d = Dash(0)
    yield d
    d.close()


def _rand(N, B, seed):
    rng = np.random.default_rng(seed)
    return rng.standard_normal((N, B, B)).astype(np.float32)


@pytest.mark.parametrize("N,B", [(1, 64), (3, 128), (5, 192), (2, 256), (9, 512), (3, 1024)])
@pytest.mark.parametrize("ta,tb", [(0, 0), (0, 1), (1, 0), (1, 1)])
def test_gemm_all_transposes(dash, N, B, ta, tb):
    import torch
    print(f"gemm N={N} B={B} ta={ta} tb={tb}", flush=True)
    A, Bm, D = _rand(N, B, 1), _rand(N, B, 2), _rand(N, B, 3)
    alpha, beta, gamma = 0.75, -1.25, 2.5
    opA = np.swapaxes(A, 1, 2) if ta else A
    opB = np.swapaxes(Bm, 1, 2) if tb else Bm
    ref = alpha * (opA.astype(np.float64) @ opB.astype(np.float64)) + beta * D.astype(np.float64) \
        + gamma * np.eye(B)
    Cd = torch.empty(N, B, B, device="cuda")
    dash.gemm_batched(torch.from_numpy(A).cuda(), torch.from_numpy(Bm).cuda(), Cd, D=torch.from_numpy(D).cuda(),
                      transA=bool(ta), transB=bool(tb), alpha=alpha, beta=beta, gamma=gamma)
    torch.cuda.synchronize()
    err = rel_frobenius_error(Cd.cpu().numpy(), ref)
    assert err.max() < TOL_MM, err
    # element-wise as well: no element may be off by more than a few ulps of the row scale
    assert np.abs(Cd.cpu().numpy() - ref).max() < 1e-4 * np.sqrt(B)


def test_gemm_in_place_addend_and_no_addend(dash):
    import torch
    N, B = 4, 256
    A, Bm, D = _rand(N, B, 4), _rand(N, B, 5), _rand(N, B, 6)
    Cd = torch.from_numpy(D).cuda()
    dash.gemm_batched(torch.from_numpy(A).cuda(), torch.from_numpy(Bm).cuda(), Cd, D=Cd, alpha=1.0, beta=0.5)
    ref = A.astype(np.float64) @ Bm.astype(np.float64) + 0.5 * D
    assert rel_frobenius_error(Cd.cpu().numpy(), ref).max() < TOL_MM
    C2 = torch.full((N, B, B), float("nan"), device="cuda")       # output is overwritten, never read
    dash.gemm_batched(torch.from_numpy(A).cuda(), torch.from_numpy(Bm).cuda(), C2)
    assert rel_frobenius_error(C2.cpu().numpy(), A.astype(np.float64) @ Bm.astype(np.float64)).max() < TOL_MM


def test_gemm_identity_and_blocks_are_independent(dash):
    import torch
    N, B = 6, 128
    A = _rand(N, B, 7)
    I = np.broadcast_to(np.eye(B, dtype=np.float32), (N, B, B)).copy()
    Cd = torch.empty(N, B, B, device="cuda")
    dash.gemm_batched(torch.from_numpy(A).cuda(), torch.from_numpy(I).cuda(), Cd)
    assert np.array_equal(Cd.cpu().numpy(), A)                     # exact: products with 0 and 1
    dash.gemm_batched(torch.from_numpy(I).cuda(), torch.from_numpy(A).cuda(), Cd, transB=True)
    assert np.array_equal(Cd.cpu().numpy(), np.swapaxes(A, 1, 2))


def test_empty_stack_is_a_no_op(dash):
    import torch
    E = torch.empty(0, 128, 128, device="cuda")
    dash.gemm_batched(E, E.clone(), E.clone())
    dash.accumulate_factors(E, E.clone(), E.clone(), 0.9)
    dash.precondition(E, E.clone(), E.clone(), E.clone())
    assert dash.inverse_root(E).shape == (0, 128, 128)


@pytest.mark.parametrize("N,B", [(1, 64), (5, 128), (3, 512), (2, 1024)])
def test_accumulate_factors(dash, N, B):
    import torch
    print(f"accumulate N={N} B={B}", flush=True)
    L64 = np.zeros((N, B, B))
    R64 = np.zeros((N, B, B))
    S = torch.zeros(2 * N, B, B, device="cuda")
    L, R = S[:N], S[N:]
    for t in range(3):
        G = workloads.gradient_stack(N, B, 100 + t, std=1e-2)
        dash.accumulate_factors(torch.from_numpy(G).cuda(), L, R, beta=0.95)
        L64, R64 = oracle_shampoo.accumulate_factors(G, L64, R64, beta=0.95)
    Lh, Rh = L.cpu().numpy(), R.cpu().numpy()
    assert rel_frobenius_error(Lh, L64).max() < TOL_MM
    assert rel_frobenius_error(Rh, R64).max() < TOL_MM
    # G G^T computed with one summation order for (i,j) and (j,i): bit-symmetric factors
    assert np.array_equal(Lh, np.swapaxes(Lh, 1, 2)) and np.array_equal(Rh, np.swapaxes(Rh, 1, 2))
    # explicit alpha (the alpha = 1 reading of the EMA)
    L1 = torch.zeros(N, B, B, device="cuda")
    R1 = torch.zeros(N, B, B, device="cuda")
    dash.accumulate_factors(torch.from_numpy(G).cuda(), L1, R1, beta=0.5, alpha=1.0)
    Lr, Rr = oracle_shampoo.accumulate_factors(G, np.zeros((N, B, B)), np.zeros((N, B, B)), 0.5, 1.0)
    assert rel_frobenius_error(L1.cpu().numpy(), Lr).max() < TOL_MM
    assert rel_frobenius_error(R1.cpu().numpy(), Rr).max() < TOL_MM


@pytest.mark.parametrize("N,B", [(3, 128), (2, 512), (5, 256)])
def test_precondition(dash, N, B):
    import torch
    print(f"precondition N={N} B={B}", flush=True)
    Li, G, Ri = _rand(N, B, 11), workloads.gradient_stack(N, B, 12), _rand(N, B, 13)
    U = dash.precondition(torch.from_numpy(Li).cuda(), torch.from_numpy(G).cuda(), torch.from_numpy(Ri).cuda())
    ref = oracle_shampoo.precondition(Li, G, Ri)
    assert rel_frobenius_error(U.cpu().numpy(), ref).max() < 2 * TOL_MM
    # chunked through a workspace that holds only two blocks: same bits
    from paper_2602_02016_amd import Dash
    d2 = Dash(0)
    d2.set_workspace_bytes(2 * B * B * 4)
    U2 = torch.empty_like(U)
    tLi, tG, tRi = torch.from_numpy(Li).cuda(), torch.from_numpy(G).cuda(), torch.from_numpy(Ri).cuda()
    d2._check(d2.lib.dash_precondition(d2.h, d2._stack(tLi, "a"), d2._stack(tG, "b"), d2._stack(tRi, "c"),
                                       d2._stack(U2, "u"), N, B))
    torch.cuda.synchronize()
    assert torch.equal(U, U2)
    d2.close()


@pytest.mark.parametrize("N,B", [(1, 4096), (1, 8192)])
def test_gemm_large_block_edges_sampled(dash, N, B):
    """Block edges far above the benchmark's: the per-lane byte offsets of the direct loads are 32-bit and a
    block of 8192^2 fp32 is 256 MiB.  A float64 product of that size is out of reach for the oracle side, so
    sampled rows and columns are checked: C[r, :] = A[r, :] B and C[:, c] = A B[:, c], fp32 and bf16 operands,
    one transposed form."""
    import torch
    print(f"gemm large N={N} B={B}", flush=True)
    rng = np.random.default_rng(B)
    A = (rng.standard_normal((N, B, B)) / np.sqrt(B)).astype(np.float32)
    Bm = (rng.standard_normal((N, B, B)) / np.sqrt(B)).astype(np.float32)
    At, Bt = torch.from_numpy(A).cuda(), torch.from_numpy(Bm).cuda()
    C = torch.empty_like(At)
    rows = [0, 1, 127, 128, B // 2 + 5, B - 1]
    cols = [0, 63, 64, B // 3, B - 2, B - 1]
    A64, B64 = A[0].astype(np.float64), Bm[0].astype(np.float64)

    def check(Cn, opA, opB, tol):
        for r in rows:
            ref = opA[r, :] @ opB
            assert np.linalg.norm(Cn[r, :] - ref) <= tol * np.linalg.norm(ref), r
        for c in cols:
            ref = opA @ opB[:, c]
            assert np.linalg.norm(Cn[:, c] - ref) <= tol * np.linalg.norm(ref), c

    dash.gemm_batched(At, Bt, C)
    check(C[0].cpu().numpy().astype(np.float64), A64, B64, 2e-5)
    dash.gemm_batched(At, Bt, C, transA=True)
    check(C[0].cpu().numpy().astype(np.float64), A64.T, B64, 2e-5)
    dash.gemm_batched(At, Bt, C, precision="bf16")
    Ab = At[0].bfloat16().float().cpu().numpy().astype(np.float64)
    Bb = Bt[0].bfloat16().float().cpu().numpy().astype(np.float64)
    check(C[0].cpu().numpy().astype(np.float64), Ab, Bb, 2e-5)


@pytest.mark.parametrize("N,B", [(2048, 256), (130, 1024)])
def test_long_launches_match_short_ones_bit_for_bit(dash, N, B):
    """Launches of many rounds of workgroups (2048 blocks of 256, 130 of 1024): whatever tile edge and launch split the
    library picks for a launch size, every output element is accumulated over k in the same order, so a block must come
    out bit for bit as when it is computed alone; sampled blocks are also checked against the float64 product, and the
    mirrored accumulation for exact symmetry."""
    import torch
    gen = torch.Generator(device="cuda")
    gen.manual_seed(N + B)
    A = torch.randn(N, B, B, device="cuda", generator=gen)
    Bm = torch.randn(N, B, B, device="cuda", generator=gen)
    D = torch.randn(N, B, B, device="cuda", generator=gen)
    C = torch.empty_like(A)
    dash.gemm_batched(A, Bm, C, D=D, alpha=0.5, beta=-0.25, gamma=1.5)
    sample = [0, 1, N // 2, N - 1]
    for i in sample:
        Ci = torch.empty(1, B, B, device="cuda")
        dash.gemm_batched(A[i:i + 1].contiguous(), Bm[i:i + 1].contiguous(), Ci, D=D[i:i + 1].contiguous(), alpha=0.5, beta=-0.25,
                          gamma=1.5)
        torch.cuda.synchronize()
        assert torch.equal(Ci[0], C[i])
        ref = 0.5 * (A[i].double() @ Bm[i].double()) - 0.25 * D[i].double() + 1.5 * torch.eye(B, device="cuda", dtype=torch.float64)
        assert float((C[i].double() - ref).norm() / ref.norm()) < TOL_MM
    # the factor accumulation's products in a long symmetric launch: G G^T through the transposed instance
    L = torch.zeros(N, B, B, device="cuda")
    R = torch.zeros(N, B, B, device="cuda")
    dash.accumulate_factors(A, L, R, 0.0, alpha=1.0)
    for i in sample:
        ref = A[i].double() @ A[i].double().T
        assert float((L[i].double() - ref).norm() / ref.norm()) < TOL_MM
        assert torch.equal(L[i], L[i].T)
