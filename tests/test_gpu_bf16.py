"""bf16-operand path (matmul operands rounded to bf16, fp32 accumulation; paper Appendix A.3
recipe) through the C ABI, against the emulation in oracle/lowprec.py and the float64 roots.

The product itself is pinned tightly (same rounded operands, float64 sum).  For Newton-DB
the paper gives no reference numbers (it reports the low-precision iteration unstable), so
only few-iteration results are asserted against the emulation; longer runs are reported."""
import numpy as np
import pytest

import workloads
from oracle import chebyshev as ocheb
from oracle import lowprec
from oracle.evd import inverse_root_evd, rel_frobenius_error

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


@pytest.mark.parametrize("N,B", [(1, 64), (3, 128), (2, 256), (5, 512), (3, 1024)])
@pytest.mark.parametrize("ta,tb", [(0, 0), (0, 1), (1, 0), (1, 1)])
def test_gemm_bf16_operands(dash, N, B, ta, tb):
    import torch
    print(f"gemm bf16 N={N} B={B} ta={ta} tb={tb}", flush=True)
    rng = np.random.default_rng(B + 2 * ta + tb)
    A = rng.standard_normal((N, B, B)).astype(np.float32)
    Bm = rng.standard_normal((N, B, B)).astype(np.float32)
    D = rng.standard_normal((N, B, B)).astype(np.float32)
    alpha, beta, gamma = 0.5, -2.0, 3.0
    opA = np.swapaxes(A, 1, 2) if ta else A
    opB = np.swapaxes(Bm, 1, 2) if tb else Bm
    ref = alpha * (lowprec.round_bf16(opA).astype(np.float64) @ lowprec.round_bf16(opB).astype(np.float64)) \
        + beta * D.astype(np.float64) + gamma * np.eye(B)
    C = torch.empty(N, B, B, device="cuda")
    dash.gemm_batched(_to_gpu(A), _to_gpu(Bm), C, D=_to_gpu(D), transA=bool(ta), transB=bool(tb), alpha=alpha,
                      beta=beta, gamma=gamma, precision="bf16")
    torch.cuda.synchronize()
    # same rounded operands, fp32 accumulation against a float64 sum: fp32-level agreement
    assert rel_frobenius_error(C.cpu().numpy(), ref).max() < 1e-5
    # and it really used rounded operands: the unrounded product is ~1e-3 away
    full = alpha * (opA.astype(np.float64) @ opB.astype(np.float64)) + beta * D.astype(np.float64) + gamma * np.eye(B)
    assert rel_frobenius_error(C.cpu().numpy(), full).max() > 1e-4


@pytest.mark.parametrize("p", [2, 4])
@pytest.mark.parametrize("k", [1, 2, 3])
def test_ndb_bf16_few_iterations_match_emulation(dash, p, k):
    N, B = 3, 128
    A32, _, _ = workloads.spd_stack(N, B, -1.0, 0.0, seed=71)
    X_emu = lowprec.inverse_root_ndb_lowprec(A32, p, k, eps=1e-6)
    # the emulation computes every product in full, as the library does with symmetric mode off
    dash.set_symmetric(False)
    try:
        X = dash.inverse_root(_to_gpu(A32), p=p, iters=k, eps=1e-6, precision="bf16").cpu().numpy()
    finally:
        dash.set_symmetric(True)
    e = rel_frobenius_error(X, X_emu).max()
    # a bf16 rounding of an iterate can fall on the other side of a tie when the fp32 sum
    # differs in its last bit from the float64 sum: isolated 2^-8 relative flips, whose
    # Frobenius weight stays far below 2^-8
    assert e < 2e-4
    # symmetric mode mirrors tiles of products whose bf16-rounded operands no longer commute
    # exactly: same iteration, differences at the bf16 rounding level of single iterates
    Xs = dash.inverse_root(_to_gpu(A32), p=p, iters=k, eps=1e-6, precision="bf16").cpu().numpy()
    es = rel_frobenius_error(Xs, X_emu).max()
    print(f"ndb bf16 p={p} k={k}: vs emulation {e:.2e} (full products), {es:.2e} (symmetric mode)", flush=True)
    assert es < 4e-3


def test_ndb_bf16_error_table_well_conditioned(dash):
    """Spectrum in [0.1, 1]: bf16 operands plateau where the emulation says, fp32 converges."""
    N, B, p = 4, 256, 4
    A32, _, _ = workloads.spd_stack(N, B, -1.0, 0.0, seed=73, share_q=True)
    X_evd = inverse_root_evd(A32.astype(np.float64), p, eps=1e-6)
    rows = []
    for k in (5, 10, 15):
        nf = _to_gpu(np.zeros(N, dtype=np.int32))
        Xb = dash.inverse_root(_to_gpu(A32), p=p, iters=k, eps=1e-6, precision="bf16", nonfinite_out=nf).cpu().numpy()
        Xf = dash.inverse_root(_to_gpu(A32), p=p, iters=k, eps=1e-6).cpu().numpy()
        Xe = lowprec.inverse_root_ndb_lowprec(A32, p, k, eps=1e-6)
        rows.append((k, rel_frobenius_error(Xb, X_evd).max(), rel_frobenius_error(Xe, X_evd).max(),
                     rel_frobenius_error(Xf, X_evd).max(), int(nf.sum().item())))
    for r in rows:
        print("ndb bf16 table k=%d: bf16 %.2e (emulated %.2e) fp32 %.2e flagged %d" % r, flush=True)
    k, eb, ee, ef, flagged = rows[-1]
    assert ef < 1e-5 and flagged == 0
    assert 1e-4 < eb < 5e-2 and eb < 5 * ee + 1e-3 and ee < 5 * eb + 1e-3


def test_ndb_bf16_divergence_is_flagged(dash):
    """Ill-conditioned blocks: the bf16 iteration blows up (paper Section 5, Newton-DB in
    FP16/BF16 did not converge); every non-finite block must be flagged and every
    unflagged block finite."""
    N, B, p = 3, 128, 4
    A32, _, _ = workloads.spd_stack(N, B, -8.0, 0.0, seed=75)
    nf = _to_gpu(np.zeros(N, dtype=np.int32))
    X = dash.inverse_root(_to_gpu(A32), p=p, iters=40, eps=1e-6, precision="bf16", nonfinite_out=nf).cpu().numpy()
    flags = nf.cpu().numpy()
    for i in range(N):
        assert bool(flags[i]) == (not np.isfinite(X[i]).all())
    print("ndb bf16 kappa=1e8 k=40: flagged", flags.tolist(), flush=True)


@pytest.mark.parametrize("p", [2, 4])
def test_chebyshev_bf16(dash, p):
    """Clenshaw with bf16 operands, fp32 iterates (the paper's mixed-precision recipe)."""
    from paper_2602_02016_amd import chebyshev_fit
    N, B, d = 3, 128, 24
    A32, _, lam = workloads.spd_stack(N, B, -1.0, 0.0, seed=77)
    A = A32.astype(np.float64)
    s = np.sqrt((A ** 2).sum(axis=(1, 2)))
    a, b = float((lam.min(axis=1) / s).min()) * 0.99, 1.0
    coef = chebyshev_fit(p, d, a, b)
    Xb = dash.inverse_root(_to_gpu(A32), method="chebyshev", p=p, iters=d, cheb_coeffs=coef, cheb_a=a, cheb_b=b,
                           precision="bf16").cpu().numpy()
    X64 = ocheb.inverse_root_chebyshev(A, p, np.array(coef), a, b)
    e = rel_frobenius_error(Xb, X64).max()
    print(f"chebyshev bf16 p={p} d={d}: vs float64 Clenshaw {e:.2e}", flush=True)
    assert 1e-5 < e < 3e-2          # bf16 operand rounding (2^-8) accumulated over d-1 products
