"""Two-plane split fp16 operands (DASH_FP16X3): hi = fp16(x), lo = fp16((x - hi) 2^11) kept scaled, three fp16 MFMA
products per matmul with the low-plane terms scaled back in the accumulator -- 22 significand bits per operand.
PARITY UNPINNED by the paper (its half-precision runs use plain fp16 operands): compared with the emulation in
oracle/lowprec.py, with the fp32 path and with the float64 roots.  Also the two-plane modes on the methods other than
Newton-DB."""
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
def test_gemm_two_fp16_planes(dash, N, B, ta, tb):
    import torch
    print(f"fp16x3 product N={N} B={B} ta={ta} tb={tb}", flush=True)
    rng = np.random.default_rng(11 * B + 2 * ta + tb)
    # entries over five decades, as in the iterates: small ones are where an unscaled low plane would fail
    A = (rng.standard_normal((N, B, B)) * 10.0 ** rng.uniform(-4, 0, (N, B, B))).astype(np.float32)
    Bm = (rng.standard_normal((N, B, B)) * 10.0 ** rng.uniform(-4, 0, (N, B, B))).astype(np.float32)
    opA = np.swapaxes(A, 1, 2) if ta else A
    opB = np.swapaxes(Bm, 1, 2) if tb else Bm
    ref = np.stack([lowprec.matmul_lowprec(opA[i], opB[i], "fp16x3") for i in range(N)]).astype(np.float64)
    C = torch.empty(N, B, B, device="cuda")
    dash.gemm_batched(_to_gpu(A), _to_gpu(Bm), C, transA=bool(ta), transB=bool(tb), precision="fp16x3")
    Ch = C.cpu().numpy()
    assert rel_frobenius_error(Ch, ref).max() < 2e-6              # same planes, fp32 against float64 sums
    full = opA.astype(np.float64) @ opB.astype(np.float64)
    C32 = torch.empty(N, B, B, device="cuda")
    dash.gemm_batched(_to_gpu(A), _to_gpu(Bm), C32, transA=bool(ta), transB=bool(tb))
    e3, e32 = rel_frobenius_error(Ch, full).max(), rel_frobenius_error(C32.cpu().numpy(), full).max()
    print(f"   vs float64: fp16x3 {e3:.2e}  fp32 {e32:.2e}", flush=True)
    assert e3 < 3 * e32 + 3e-7


@pytest.mark.parametrize("method", ["newton_db", "coupled_newton"])
@pytest.mark.parametrize("p", [2, 4])
@pytest.mark.parametrize("k", [1, 2, 3])
def test_few_iterations_match_emulation(dash, method, p, k):
    N, B = 3, 128
    A32, _, _ = workloads.spd_stack(N, B, -1.0, 0.0, seed=161)
    dash.set_symmetric(False)
    try:
        X = dash.inverse_root(_to_gpu(A32), method=method, p=p, iters=k, eps=1e-6, precision="fp16x3").cpu().numpy()
    finally:
        dash.set_symmetric(True)
    if method == "newton_db":
        X_emu = lowprec.inverse_root_ndb_lowprec(A32, p, k, eps=1e-6, rounding="fp16x3")
    else:
        X_emu = lowprec.inverse_root_cn_lowprec(A32, p, k, eps=1e-6, fmt="fp16x3")
    e = rel_frobenius_error(X, X_emu).max()
    print(f"fp16x3 {method} p={p} k={k}: vs emulation {e:.2e}", flush=True)
    assert e < 5e-6
    if method != "newton_db":      # and against Coupled-Newton in the printed order of Section 3.2
        X_print = lowprec.inverse_root_cn_lowprec_as_printed(A32, p, k, eps=1e-6, fmt="fp16x3")
        assert rel_frobenius_error(X, X_print).max() < 1e-5


@pytest.mark.parametrize("method,k", [("newton_db", 16), ("coupled_newton", 25)])
@pytest.mark.parametrize("B,lo", [(256, -1.0), (256, -3.0), (1024, -2.0)])
def test_near_the_fp32_floor(dash, method, k, B, lo):
    """Error against the EVD root: within a small factor of the fp32 path, far below plain fp16 and two bf16 planes."""
    N, p = 3, 4
    A32, _, _ = workloads.spd_stack(N, B, lo, 0.0, seed=163, share_q=True)
    X_evd = inverse_root_evd(A32.astype(np.float64), p, eps=1e-6)
    e = {}
    for prec in ("fp32", "fp16x3", "bf16x3", "fp16"):
        nf = _to_gpu(np.zeros(N, dtype=np.int32))
        X = dash.inverse_root(_to_gpu(A32), method=method, p=p, iters=k, eps=1e-6, precision=prec, nonfinite_out=nf).cpu().numpy()
        e[prec] = rel_frobenius_error(X, X_evd).max() if np.isfinite(X).all() else float("inf")
        if prec in ("fp32", "fp16x3"):
            assert int(nf.sum().item()) == 0
    print(f"{method} B={B} kappa=1e{-lo:.0f} k={k}: vs EVD fp32 {e['fp32']:.2e}  fp16x3 {e['fp16x3']:.2e}  "
          f"bf16x3 {e['bf16x3']:.2e}  fp16 {e['fp16']:.2e}", flush=True)
    assert e["fp16x3"] < 10 * e["fp32"] + 2e-6
    assert e["fp16x3"] < e["bf16x3"] / 3 and e["fp16x3"] < e["fp16"] / 30


@pytest.mark.parametrize("prec", ["fp16x3", "bf16x3"])
@pytest.mark.parametrize("p", [2, 4])
def test_chebyshev_two_planes(dash, prec, p):
    from oracle import chebyshev as ocheb
    from paper_2602_02016_amd import chebyshev_fit
    N, B, d = 3, 256, 24
    A32, Q, lam = workloads.spd_stack(N, B, -1.0, 0.0, seed=165)
    A = A32.astype(np.float64)
    s = np.sqrt((A ** 2).sum(axis=(1, 2)))
    a, b = float((lam.min(axis=1) / s).min()) * 0.99, 1.0
    coef = chebyshev_fit(p, d, a, b)
    X = dash.inverse_root(_to_gpu(A32), method="chebyshev", p=p, iters=d, cheb_coeffs=coef, cheb_a=a, cheb_b=b,
                          precision=prec).cpu().numpy()
    e = rel_frobenius_error(X, ocheb.inverse_root_chebyshev(A, p, np.array(coef), a, b)).max()
    print(f"cheb {prec} p={p}: vs f64 Clenshaw {e:.2e}", flush=True)
    assert e < (1e-5 if prec == "fp16x3" else 3e-4)


def test_overflow_is_flagged_not_hidden(dash):
    """fp16's exponent range applies to the iterates: a block whose inverse square root has entries beyond 65504
    (kappa = 1e12, no damping) overflows; the per-block flag says so for exactly the blocks whose result is not
    finite, and a well-conditioned block in the same stack is untouched by its neighbour."""
    N, B, p = 3, 128, 4
    bad, _, _ = workloads.spd_stack(2, B, -12.0, 0.0, seed=167)
    good, _, _ = workloads.spd_stack(1, B, -1.0, 0.0, seed=168)
    A32 = np.concatenate([bad[:1], good, bad[1:]])
    nf = _to_gpu(np.zeros(N, dtype=np.int32))
    X = dash.inverse_root(_to_gpu(A32), p=p, iters=30, eps=0.0, precision="fp16x3", nonfinite_out=nf).cpu().numpy()
    flags = nf.cpu().numpy()
    for i in range(N):
        assert bool(flags[i]) == (not np.isfinite(X[i]).all()), (i, flags)
    assert flags[1] == 0
    e = rel_frobenius_error(X[1:2], inverse_root_evd(good.astype(np.float64), p))[0]
    print(f"fp16x3 overflow: flags {flags.tolist()}, good block vs EVD {e:.2e}", flush=True)
    assert e < 1e-5


@pytest.mark.parametrize("B", [64, 192, 320, 448, 768])
@pytest.mark.parametrize("N", [1, 5])
def test_split_modes_agree_with_fp32_on_odd_block_edges(dash, N, B):
    """Block edges that are multiples of 64 only (64-wide tiles, odd tile counts) and of 256 times an odd number:
    every split mode, every method, against the fp32 path on the same well-conditioned blocks."""
    from paper_2602_02016_amd import chebyshev_fit
    A32, _, lam = workloads.spd_stack(N, B, -1.0, 0.0, seed=170 + B)
    A = _to_gpu(A32)
    s = np.sqrt((A32.astype(np.float64) ** 2).sum(axis=(1, 2)))
    a = float((lam.min(axis=1) / s).min()) * 0.99
    cases = {"newton_db": dict(iters=14), "coupled_newton": dict(iters=20),
             "chebyshev": dict(iters=24, cheb_coeffs=chebyshev_fit(4, 24, a, 1.0), cheb_a=a, cheb_b=1.0)}
    for method, kw in cases.items():
        X32 = dash.inverse_root(A, method=method, p=4, eps=1e-6, **kw).cpu().numpy()
        for prec in ("fp16x3", "bf16x6", "bf16x3"):
            nf = _to_gpu(np.zeros(N, dtype=np.int32))
            X = dash.inverse_root(A, method=method, p=4, eps=1e-6, precision=prec, nonfinite_out=nf, **kw).cpu().numpy()
            e = rel_frobenius_error(X, X32.astype(np.float64)).max()
            assert int(nf.sum().item()) == 0
            assert e < (2e-4 if prec == "bf16x3" else 2e-5), (method, prec, B, N, e)
    print(f"split modes vs fp32 ok N={N} B={B}", flush=True)


@pytest.mark.parametrize("method,k", [("newton_db", 20), ("coupled_newton", 30)])
@pytest.mark.parametrize("B", [256, 512])
def test_illconditioned_blocks_kappa_1e4(dash, method, k, B):
    """Spectra log-uniform in [1e-4, 1], no damping (the shape of the block-size sweep): at the floor of the fp32
    path or below it."""
    N, p = 3, 4
    A32, _, _ = workloads.spd_stack(N, B, -4.0, 0.0, seed=500 + B, share_q=True)
    X_evd = inverse_root_evd(A32.astype(np.float64), p)
    e = {}
    for prec in ("fp32", "fp16x3", "bf16x6"):
        nf = _to_gpu(np.zeros(N, dtype=np.int32))
        X = dash.inverse_root(_to_gpu(A32), method=method, p=p, iters=k, precision=prec, nonfinite_out=nf).cpu().numpy()
        assert int(nf.sum().item()) == 0
        e[prec] = rel_frobenius_error(X, X_evd).max()
    print(f"{method} B={B} kappa=1e4 k={k}: vs EVD fp32 {e['fp32']:.2e}  fp16x3 {e['fp16x3']:.2e}  bf16x6 {e['bf16x6']:.2e}", flush=True)
    assert e["fp16x3"] < 2 * e["fp32"] + 1e-5 and e["bf16x6"] < 2 * e["fp32"] + 1e-5
