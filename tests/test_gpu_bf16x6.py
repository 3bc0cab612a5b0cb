"""Three-plane split bf16 operands (DASH_BF16X6): x ~ hi + mid + lo represents a float exactly, the six plane
products of weight 2^-16 and above are summed in fp32 -- fp32 accuracy from bf16 MFMA products.  PARITY UNPINNED by
the paper (it leaves low-precision Newton-DB as future work): compared with the emulation in oracle/lowprec.py,
with the fp32 path and with the float64 roots."""
import numpy as np
import pytest

import workloads
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


@pytest.mark.parametrize("N,B", [(2, 64), (3, 128), (5, 512), (3, 1024)])
@pytest.mark.parametrize("ta,tb", [(0, 0), (0, 1), (1, 0), (1, 1)])
def test_gemm_three_planes(dash, N, B, ta, tb):
    import torch
    print(f"bf16x6 product N={N} B={B} ta={ta} tb={tb}", flush=True)
    rng = np.random.default_rng(7 * B + 2 * ta + tb)
    A = rng.standard_normal((N, B, B)).astype(np.float32)
    Bm = rng.standard_normal((N, B, B)).astype(np.float32)
    opA = np.swapaxes(A, 1, 2) if ta else A
    opB = np.swapaxes(Bm, 1, 2) if tb else Bm
    ref = np.stack([lowprec.matmul_lowprec(opA[i], opB[i], "bf16x6") for i in range(N)]).astype(np.float64)
    C = torch.empty(N, B, B, device="cuda")
    dash.gemm_batched(_to_gpu(A), _to_gpu(Bm), C, transA=bool(ta), transB=bool(tb), precision="bf16x6")
    Ch = C.cpu().numpy()
    assert rel_frobenius_error(Ch, ref).max() < 2e-6              # same planes, fp32 against float64 sums
    full = opA.astype(np.float64) @ opB.astype(np.float64)
    C32 = torch.empty(N, B, B, device="cuda")
    dash.gemm_batched(_to_gpu(A), _to_gpu(Bm), C32, transA=bool(ta), transB=bool(tb))
    e6, e32 = rel_frobenius_error(Ch, full).max(), rel_frobenius_error(C32.cpu().numpy(), full).max()
    print(f"   vs float64: bf16x6 {e6:.2e}  fp32 {e32:.2e}", flush=True)
    assert e6 < 3 * e32 + 1e-7                                    # the accuracy of the fp32 MFMA product


@pytest.mark.parametrize("p", [2, 4])
@pytest.mark.parametrize("k", [1, 2, 3])
def test_few_iterations_match_emulation(dash, p, k):
    N, B = 3, 128
    A32, _, _ = workloads.spd_stack(N, B, -1.0, 0.0, seed=141)
    dash.set_symmetric(False)
    try:
        X = dash.inverse_root(_to_gpu(A32), p=p, iters=k, eps=1e-6, precision="bf16x6").cpu().numpy()
    finally:
        dash.set_symmetric(True)
    X_emu = lowprec.inverse_root_ndb_lowprec(A32, p, k, eps=1e-6, rounding="bf16x6")
    e = rel_frobenius_error(X, X_emu).max()
    print(f"bf16x6 p={p} k={k}: vs emulation {e:.2e}", flush=True)
    assert e < 5e-6


@pytest.mark.parametrize("B,lo,k", [(256, -1.0, 12), (256, -3.0, 16), (512, -4.0, 22), (1024, -2.0, 14)])
def test_reaches_the_fp32_floor(dash, B, lo, k):
    """Error against the EVD root: the three-plane mode sits at the floor of the fp32 path, on spectra where two
    planes are one to two orders of magnitude above it."""
    N, p = 4, 4
    A32, _, _ = workloads.spd_stack(N, B, lo, 0.0, seed=143, share_q=True)
    X_evd = inverse_root_evd(A32.astype(np.float64), p, eps=1e-6)
    e = {}
    for prec in ("fp32", "bf16x6", "bf16x3"):
        nf = _to_gpu(np.zeros(N, dtype=np.int32))
        X = dash.inverse_root(_to_gpu(A32), p=p, iters=k, eps=1e-6, precision=prec, nonfinite_out=nf).cpu().numpy()
        assert int(nf.sum().item()) == 0 and np.isfinite(X).all()
        e[prec] = rel_frobenius_error(X, X_evd).max()
    print(f"B={B} kappa=1e{-lo:.0f} k={k}: vs EVD fp32 {e['fp32']:.2e}  bf16x6 {e['bf16x6']:.2e}  bf16x3 {e['bf16x3']:.2e}", flush=True)
    assert e["bf16x6"] < 3 * e["fp32"] + 1e-6
    assert e["bf16x6"] < e["bf16x3"] / 3


@pytest.mark.parametrize("p", [2, 4])
@pytest.mark.parametrize("B,d", [(128, 2), (128, 3), (128, 16), (256, 32), (1024, 24)])
def test_chebyshev_matches_float64_clenshaw(dash, p, B, d):
    """The Clenshaw recurrence with three-plane operands (B_k kept in fp32, as in Appendix A.3) against the float64
    recurrence with the same coefficients: the bar of the fp32 path."""
    from oracle import chebyshev as ocheb
    from paper_2602_02016_amd import chebyshev_fit
    N = 3
    A32, Q, lam = workloads.spd_stack(N, B, -1.0, 0.0, seed=147, share_q=B >= 512)
    A = A32.astype(np.float64)
    s = np.sqrt((A ** 2).sum(axis=(1, 2)))
    a, b = float((lam.min(axis=1) / s).min()) * 0.99, 1.0
    coef = chebyshev_fit(p, d, a, b)
    kw = dict(method="chebyshev", p=p, iters=d, cheb_coeffs=coef, cheb_a=a, cheb_b=b)
    X6 = dash.inverse_root(_to_gpu(A32), precision="bf16x6", **kw).cpu().numpy()
    X32 = dash.inverse_root(_to_gpu(A32), **kw).cpu().numpy()
    X_same = ocheb.inverse_root_chebyshev(A, p, np.array(coef), a, b)
    e6, e32 = rel_frobenius_error(X6, X_same).max(), rel_frobenius_error(X32, X_same).max()
    print(f"cheb bf16x6 p={p} B={B} d={d}: vs f64 Clenshaw {e6:.2e} (fp32 path {e32:.2e})", flush=True)
    assert e6 < 1e-5 and e6 < 3 * e32 + 1e-6


@pytest.mark.parametrize("p", [2, 4])
@pytest.mark.parametrize("k", [1, 2, 3])
def test_coupled_newton_few_iterations_match_emulation(dash, p, k):
    N, B = 3, 128
    A32, _, _ = workloads.spd_stack(N, B, -1.0, 0.0, seed=149)
    X = dash.inverse_root(_to_gpu(A32), method="coupled_newton", p=p, iters=k, eps=1e-6, precision="bf16x6").cpu().numpy()
    X_emu = lowprec.inverse_root_cn_lowprec(A32, p, k, eps=1e-6, fmt="bf16x6")
    e = rel_frobenius_error(X, X_emu).max()
    print(f"cn bf16x6 p={p} k={k}: vs emulation {e:.2e}", flush=True)
    assert e < 5e-6
    # and against Coupled-Newton in the printed order of Section 3.2 (no product or rounding saved)
    X_print = lowprec.inverse_root_cn_lowprec_as_printed(A32, p, k, eps=1e-6, fmt="bf16x6")
    assert rel_frobenius_error(X, X_print).max() < 1e-5


@pytest.mark.parametrize("p", [2, 4])
@pytest.mark.parametrize("B", [256, 1024])
def test_coupled_newton_reaches_the_fp32_floor(dash, p, B):
    N, k = 3, 25
    A32, _, _ = workloads.spd_stack(N, B, -1.0, 0.0, seed=151, share_q=B >= 512)
    X_evd = inverse_root_evd(A32.astype(np.float64), p, eps=1e-6)
    e = {}
    for prec in ("fp32", "bf16x6", "fp16"):
        nf = _to_gpu(np.zeros(N, dtype=np.int32))
        X = dash.inverse_root(_to_gpu(A32), method="coupled_newton", p=p, iters=k, eps=1e-6, precision=prec,
                              nonfinite_out=nf).cpu().numpy()
        assert int(nf.sum().item()) == 0
        e[prec] = rel_frobenius_error(X, X_evd).max()
    print(f"cn p={p} B={B} k={k}: vs EVD fp32 {e['fp32']:.2e}  bf16x6 {e['bf16x6']:.2e}  fp16 {e['fp16']:.2e}", flush=True)
    assert e["bf16x6"] < 3 * e["fp32"] + 1e-6 and e["bf16x6"] < e["fp16"] / 10
