"""Split-operand bf16 (DASH_BF16X3): operands carried as two bf16 planes, three bf16 MFMA products per
matmul, fp32 accumulation -- about 16 significand bits per operand.  The paper leaves low-precision
Newton-DB as future work (Sections 2.3, 6); this is one way to make it stable.  PARITY UNPINNED by the
paper: compared with the emulation in oracle/lowprec.py and reported against the float64 roots."""
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
def test_gemm_split_operands(dash, N, B, ta, tb):
    import torch
    rng = np.random.default_rng(B + 2 * ta + tb)
    A = rng.standard_normal((N, B, B)).astype(np.float32)
    Bm = rng.standard_normal((N, B, B)).astype(np.float32)
    opA = np.swapaxes(A, 1, 2) if ta else A
    opB = np.swapaxes(Bm, 1, 2) if tb else Bm
    ref = np.stack([lowprec.matmul_lowprec(opA[i], opB[i], "bf16x3") for i in range(N)]).astype(np.float64)
    C = torch.empty(N, B, B, device="cuda")
    dash.gemm_batched(_to_gpu(A), _to_gpu(Bm), C, transA=bool(ta), transB=bool(tb), precision="bf16x3")
    Ch = C.cpu().numpy()
    assert rel_frobenius_error(Ch, ref).max() < 2e-6              # same planes, fp32 against float64 sums
    full = opA.astype(np.float64) @ opB.astype(np.float64)
    e_full = rel_frobenius_error(Ch, full).max()
    e_bf16 = rel_frobenius_error(np.stack([lowprec.matmul_lowprec(opA[i], opB[i], "bf16") for i in range(N)]), full).max()
    assert e_full < 2e-5 and e_full < e_bf16 / 50                 # ~2^-16 per operand against 2^-8


@pytest.mark.parametrize("p", [2, 4])
@pytest.mark.parametrize("k", [1, 2, 3])
def test_few_iterations_match_emulation(dash, p, k):
    N, B = 3, 128
    A32, _, _ = workloads.spd_stack(N, B, -1.0, 0.0, seed=131)
    dash.set_symmetric(False)
    try:
        X = dash.inverse_root(_to_gpu(A32), p=p, iters=k, eps=1e-6, precision="bf16x3").cpu().numpy()
    finally:
        dash.set_symmetric(True)
    X_emu = lowprec.inverse_root_ndb_lowprec(A32, p, k, eps=1e-6, rounding="bf16x3")
    e = rel_frobenius_error(X, X_emu).max()
    print(f"bf16x3 p={p} k={k}: vs emulation {e:.2e}", flush=True)
    assert e < 2e-5


@pytest.mark.parametrize("lo,k", [(-1.0, 12), (-3.0, 16), (-4.0, 22)])
def test_stable_where_plain_bf16_is_not(dash, lo, k):
    """Error against the EVD root: split operands stay close to fp32 on spectra where plain bf16 operands
    plateau at 1e-2 or diverge."""
    N, B, p = 4, 256, 4
    A32, _, _ = workloads.spd_stack(N, B, lo, 0.0, seed=133, share_q=True)
    X_evd = inverse_root_evd(A32.astype(np.float64), p, eps=1e-6)
    e = {}
    for prec in ("fp32", "bf16x3", "bf16"):
        nf = _to_gpu(np.zeros(N, dtype=np.int32))
        X = dash.inverse_root(_to_gpu(A32), p=p, iters=k, eps=1e-6, precision=prec, nonfinite_out=nf).cpu().numpy()
        e[prec] = rel_frobenius_error(X, X_evd).max() if np.isfinite(X).all() else float("inf")
        if prec != "bf16":
            assert int(nf.sum().item()) == 0
    print(f"kappa=1e{-lo:.0f} k={k}: vs EVD fp32 {e['fp32']:.2e}  bf16x3 {e['bf16x3']:.2e}  bf16 {e['bf16']:.2e}", flush=True)
    assert e["bf16x3"] < 200 * e["fp32"] + 1e-5
    assert e["bf16x3"] < e["bf16"] / 20
