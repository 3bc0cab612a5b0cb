"""fp16-operand paths (the paper's own low-precision format: Coupled-Newton and Clenshaw in fp16,
Sections 2.3, 5 and Appendix A.3) through the C ABI against the emulation and the float64 roots."""
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
    d.set_symmetric(False)      # the emulation computes every product in full
    yield d
    d.close()


def _to_gpu(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


@pytest.mark.parametrize("N,B", [(1, 64), (3, 128), (5, 512), (3, 1024)])
@pytest.mark.parametrize("ta,tb", [(0, 0), (1, 1)])
def test_gemm_fp16_operands(dash, N, B, ta, tb):
    import torch
    rng = np.random.default_rng(B + ta)
    A = rng.standard_normal((N, B, B)).astype(np.float32)
    Bm = rng.standard_normal((N, B, B)).astype(np.float32)
    opA = np.swapaxes(A, 1, 2) if ta else A
    opB = np.swapaxes(Bm, 1, 2) if tb else Bm
    ref = lowprec.round_fp16(opA).astype(np.float64) @ lowprec.round_fp16(opB).astype(np.float64)
    C = torch.empty(N, B, B, device="cuda")
    dash.gemm_batched(_to_gpu(A), _to_gpu(Bm), C, transA=bool(ta), transB=bool(tb), precision="fp16")
    assert rel_frobenius_error(C.cpu().numpy(), ref).max() < 1e-5
    ref_bf = lowprec.round_bf16(opA).astype(np.float64) @ lowprec.round_bf16(opB).astype(np.float64)
    assert rel_frobenius_error(C.cpu().numpy(), ref_bf).max() > 1e-4        # it is not the bf16 product


@pytest.mark.parametrize("method", ["ndb", "cn"])
@pytest.mark.parametrize("p", [2, 4])
@pytest.mark.parametrize("k", [1, 2, 3])
def test_few_iterations_match_emulation(dash, method, p, k):
    N, B = 3, 128
    A32, _, _ = workloads.spd_stack(N, B, -1.0, 0.0, seed=121)
    X = dash.inverse_root(_to_gpu(A32), method=method, p=p, iters=k, eps=1e-6, precision="fp16").cpu().numpy()
    if method == "ndb":
        X_emu = lowprec.inverse_root_ndb_lowprec(A32, p, k, eps=1e-6, rounding="fp16")
    else:
        X_emu = lowprec.inverse_root_cn_lowprec(A32, p, k, eps=1e-6, fmt="fp16")
    e = rel_frobenius_error(X, X_emu).max()
    print(f"fp16 {method} p={p} k={k}: vs emulation {e:.2e}", flush=True)
    assert e < 5e-5
    if method == "cn":
        # and against the iteration in the order Section 3.2 prints it (1/c as the rounded start matrix, every
        # product computed): the same root up to a few units of fp16 per iteration
        X_print = lowprec.inverse_root_cn_lowprec_as_printed(A32, p, k, eps=1e-6, fmt="fp16")
        assert rel_frobenius_error(X, X_print).max() < 6 * k * 2.0 ** -11 + 5e-5


@pytest.mark.parametrize("p", [2, 4])
def test_coupled_newton_fp16_converges_bf16_degrades(dash, p):
    """The paper's fastest configuration: Coupled-Newton with fp16 operands keeps working; with bf16 it
    loses accuracy (the paper reports divergence in training)."""
    N, B, k = 4, 512, 25
    A32, _, _ = workloads.spd_stack(N, B, -1.0, 0.0, seed=123, share_q=True)
    X_evd = inverse_root_evd(A32[:2].astype(np.float64), p, eps=1e-6)
    e = {}
    for prec in ("fp32", "fp16", "bf16"):
        nf = _to_gpu(np.zeros(N, dtype=np.int32))
        X = dash.inverse_root(_to_gpu(A32), method="cn", p=p, iters=k, eps=1e-6, precision=prec, nonfinite_out=nf)
        e[prec] = rel_frobenius_error(X[:2].cpu().numpy(), X_evd).max()
        assert int(nf.sum().item()) == 0
    emu = rel_frobenius_error(lowprec.inverse_root_cn_lowprec(A32[:2], p, k, eps=1e-6, fmt="fp16"), X_evd).max()
    print(f"cn p={p} B={B}: vs EVD fp32 {e['fp32']:.2e} fp16 {e['fp16']:.2e} (emulated {emu:.2e}) bf16 {e['bf16']:.2e}",
          flush=True)
    assert e["fp32"] < 1e-4
    assert e["fp16"] < 5e-3 and e["fp16"] < 3 * emu + 1e-4 and emu < 3 * e["fp16"] + 1e-4
    assert e["bf16"] > 2 * e["fp16"]


@pytest.mark.parametrize("p", [2, 4])
def test_chebyshev_fp16(dash, p):
    """Clenshaw as the paper runs it in mixed precision: B_k in fp32, S and the operand copy of B_{k+1} in fp16."""
    from paper_2602_02016_amd import chebyshev_fit
    N, B, d = 3, 256, 40
    A32, _, lam = workloads.spd_stack(N, B, -1.0, 0.0, seed=125)
    A = A32.astype(np.float64)
    s = np.sqrt((A ** 2).sum(axis=(1, 2)))
    a, b = float((lam.min(axis=1) / s).min()) * 0.99, 1.0
    coef = chebyshev_fit(p, d, a, b)
    X64 = ocheb.inverse_root_chebyshev(A, p, np.array(coef), a, b)
    e = {}
    for prec in ("fp16", "bf16"):
        X = dash.inverse_root(_to_gpu(A32), method="chebyshev", p=p, iters=d, cheb_coeffs=coef, cheb_a=a, cheb_b=b,
                              precision=prec).cpu().numpy()
        e[prec] = rel_frobenius_error(X, X64).max()
    print(f"chebyshev p={p} d={d}: vs float64 Clenshaw fp16 {e['fp16']:.2e} bf16 {e['bf16']:.2e}", flush=True)
    assert e["fp16"] < 5e-3 and e["fp16"] < e["bf16"] / 2
