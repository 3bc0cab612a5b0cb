"""Pins for the bf16-operand emulation (oracle/lowprec.py)."""
import numpy as np
import pytest
import torch

import workloads
from oracle import lowprec
from oracle import newton_db as ondb
from oracle.evd import inverse_root_evd, rel_frobenius_error


def test_round_bf16_exact_facts():
    # bf16 keeps 8 significand bits: spacing 2^-7 in [1, 2)
    f = np.float32
    assert lowprec.round_bf16(f(1.0)) == 1.0
    assert lowprec.round_bf16(f(1.0 + 2.0 ** -7)) == f(1.0 + 2.0 ** -7)          # representable
    assert lowprec.round_bf16(f(1.0 + 2.0 ** -8)) == 1.0                         # tie -> even (down)
    assert lowprec.round_bf16(f(1.0 + 3 * 2.0 ** -8)) == f(1.0 + 2.0 ** -6)      # tie -> even (up)
    assert lowprec.round_bf16(f(1.0 + 2.0 ** -8 + 2.0 ** -20)) == f(1.0 + 2.0 ** -7)   # above the tie
    assert lowprec.round_bf16(f(-0.3)) == -lowprec.round_bf16(f(0.3))
    assert np.isnan(lowprec.round_bf16(f(np.nan))) and np.isinf(lowprec.round_bf16(f(3.4e38)))
    assert lowprec.round_bf16(f(0.0)) == 0.0


def test_round_bf16_matches_torch_conversion():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(20000), rng.standard_normal(2000) * 1e-20,
                        rng.standard_normal(2000) * 1e20]).astype(np.float32)
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(lowprec.round_bf16(x), ref)


def test_matmul_bf16_on_representable_operands_is_exact():
    rng = np.random.default_rng(1)
    A = lowprec.round_bf16(rng.standard_normal((16, 16)).astype(np.float32))
    B = lowprec.round_bf16(rng.standard_normal((16, 16)).astype(np.float32))
    assert np.array_equal(lowprec.matmul_bf16(A, B), (A.astype(np.float64) @ B.astype(np.float64)).astype(np.float32))
    # and rounding really is applied to operands that are not representable
    C = rng.standard_normal((16, 16)).astype(np.float32)
    assert not np.array_equal(lowprec.matmul_bf16(C, B), (C.astype(np.float64) @ B).astype(np.float32))


@pytest.mark.parametrize("p", [2, 4])
def test_without_rounding_it_is_the_float64_iteration(p):
    A32, _, _ = workloads.spd_stack(2, 32, -1.0, 0.0, seed=3)
    X = lowprec.inverse_root_ndb_lowprec(A32, p, 8, eps=1e-6, rounding=False)
    X64 = ondb.inverse_root_ndb(A32.astype(np.float64), p, 8, eps=1e-6)
    assert rel_frobenius_error(X, X64).max() < 5e-6


def test_exactly_representable_iterates():
    # A = I/2 scaled by its Frobenius norm: every iterate is a multiple of I; with B = 4 the scale
    # is exactly 1 (||I/2||_F = 1) and the first iterates 1.25, 0.625*... are short binary fractions
    A = 0.5 * np.eye(4, dtype=np.float32)
    X1 = lowprec.inverse_root_ndb_lowprec(A, 2, 1)
    assert np.array_equal(X1, np.float32(1.25) * np.eye(4, dtype=np.float32))   # Z_1 = 1.5 - 0.25
    X2 = lowprec.inverse_root_ndb_lowprec(A, 2, 2)
    y1, z1 = 0.5 * 1.25, 1.25
    e2 = 1.5 - 0.5 * z1 * y1
    assert np.allclose(np.diag(X2), e2 * z1, rtol=2e-3)       # operands 1.25, 0.625 exact; E_2 rounds to bf16


def test_bf16_plateau_is_where_expected():
    # well-conditioned block: bf16 operands stall around 1e-3..1e-2 while fp32/float64 converge
    A32, Q, lam = workloads.spd_stack(1, 64, -1.0, 0.0, seed=5)
    X_true = (Q[0] * lam[0] ** -0.25) @ Q[0].T
    e_lo = rel_frobenius_error(lowprec.inverse_root_ndb_lowprec(A32[0], 4, 12), X_true)[0]
    e_hi = rel_frobenius_error(lowprec.inverse_root_ndb_lowprec(A32[0], 4, 12, rounding=False), X_true)[0]
    assert e_hi < 1e-5 and 1e-4 < e_lo < 5e-2


def test_round_fp16_exact_facts_and_library():
    f = np.float32
    assert lowprec.round_fp16(f(1.0 + 2.0 ** -10)) == f(1.0 + 2.0 ** -10)        # 11 significand bits
    assert lowprec.round_fp16(f(1.0 + 2.0 ** -11)) == 1.0                        # tie -> even
    assert lowprec.round_fp16(f(1.0 + 3 * 2.0 ** -11)) == f(1.0 + 2.0 ** -9)
    assert lowprec.round_fp16(f(65504.0)) == 65504.0 and np.isinf(lowprec.round_fp16(f(70000.0)))
    assert lowprec.round_fp16(f(2.0 ** -24)) == f(2.0 ** -24)                    # smallest subnormal
    assert lowprec.round_fp16(f(2.0 ** -26)) == 0.0                              # underflows to zero
    rng = np.random.default_rng(1)
    x = np.concatenate([rng.standard_normal(20000), rng.standard_normal(2000) * 1e-6]).astype(np.float32)
    ref = torch.from_numpy(x).to(torch.float16).to(torch.float32).numpy()
    assert np.array_equal(lowprec.round_fp16(x), ref)


@pytest.mark.parametrize("p", [2, 4])
def test_cn_emulation_without_rounding_is_the_paper_iteration(p):
    from oracle import coupled_newton as ocn
    A32, _, _ = workloads.spd_stack(2, 32, -1.0, 0.0, seed=7)
    for k in (1, 2, 3, 9):
        X = lowprec.inverse_root_cn_lowprec(A32, p, k, eps=1e-6, fmt="none")
        X64 = ocn.inverse_root_cn(A32.astype(np.float64), p, k, eps=1e-6)
        assert rel_frobenius_error(X, X64).max() < 2e-6


@pytest.mark.parametrize("p", [2, 4])
@pytest.mark.parametrize("fmt,unit", [("fp16", 2.0 ** -11), ("bf16", 2.0 ** -8), ("bf16x3", 2.0 ** -16),
                                      ("fp16x3", 2.0 ** -22), ("bf16x6", 2.0 ** -24)])
def test_cn_emulation_agrees_with_the_printed_order(p, fmt, unit):
    """The emulation the GPU path is compared with carries 1/c to the end (no product for X_1, no last M); the
    iteration in the order Section 3.2 prints it, with the same operand rounding, must give the same root up to a
    few units of the operand format -- so the reading changes rounding, not the method.  Without rounding both are
    the float64 iteration of the oracle."""
    from oracle import coupled_newton as ocn
    A32, _, _ = workloads.spd_stack(2, 48, -1.0, 0.0, seed=21)
    for k in (1, 2, 4, 8):
        X_read = lowprec.inverse_root_cn_lowprec(A32, p, k, eps=1e-6, fmt=fmt)
        X_print = lowprec.inverse_root_cn_lowprec_as_printed(A32, p, k, eps=1e-6, fmt=fmt)
        e = rel_frobenius_error(X_read, X_print).max()
        assert e < 6 * k * unit + 4e-7, (fmt, p, k, e)
    X_print = lowprec.inverse_root_cn_lowprec_as_printed(A32, p, 6, eps=1e-6, fmt="none")
    assert rel_frobenius_error(X_print, ocn.inverse_root_cn(A32.astype(np.float64), p, 6, eps=1e-6)).max() < 2e-6


def test_fp16_beats_bf16_on_a_well_conditioned_block():
    # Sections 2.3 / 5: Coupled-Newton works in fp16 and diverges or degrades in bf16; Newton-DB
    # plateaus higher with bf16's 8 significand bits than with fp16's 11
    A32, Q, lam = workloads.spd_stack(1, 64, -1.0, 0.0, seed=9)
    X_true = (Q[0] * lam[0] ** -0.25) @ Q[0].T
    e = {}
    for fmt in ("fp16", "bf16"):
        e["cn", fmt] = rel_frobenius_error(lowprec.inverse_root_cn_lowprec(A32[0], 4, 25, fmt=fmt), X_true)[0]
        e["ndb", fmt] = rel_frobenius_error(lowprec.inverse_root_ndb_lowprec(A32[0], 4, 12, rounding=fmt), X_true)[0]
    assert e["cn", "fp16"] < 3e-3 and e["cn", "fp16"] < e["cn", "bf16"] / 3
    assert e["ndb", "fp16"] < e["ndb", "bf16"] / 3


def test_split_bf16_planes():
    # hi + lo reproduces x to ~2^-16 relative (two 8-bit significands), hi is the plain bf16 rounding
    rng = np.random.default_rng(3)
    x = rng.standard_normal(20000).astype(np.float32)
    hi, lo = lowprec.split_bf16(x)
    assert np.array_equal(hi, lowprec.round_bf16(x))
    assert np.all(np.abs(lo) <= np.abs(x) * 2.0 ** -8)
    rel = np.abs((hi.astype(np.float64) + lo) - x) / np.abs(x)
    assert rel.max() <= 2.0 ** -16 and rel.max() > 2.0 ** -20
    # values with at most 16 significant bits split exactly
    y = (np.arange(1, 4097, dtype=np.float32) * np.float32(2.0 ** -12))
    hi, lo = lowprec.split_bf16(y)
    assert np.array_equal(hi + lo, y)


def test_split_product_is_far_closer_than_plain_bf16():
    rng = np.random.default_rng(4)
    A = rng.standard_normal((64, 64)).astype(np.float32)
    B = rng.standard_normal((64, 64)).astype(np.float32)
    exact = A.astype(np.float64) @ B.astype(np.float64)
    e3 = rel_frobenius_error(lowprec.matmul_lowprec(A, B, "bf16x3"), exact)[0]
    e1 = rel_frobenius_error(lowprec.matmul_lowprec(A, B, "bf16"), exact)[0]
    assert e3 < 2e-5 and e1 > 1e-3
    # the three-term form is exactly hi*hi + hi*lo + lo*hi: adding lo*lo gives the product of the sums
    ah, al = lowprec.split_bf16(A); bh, bl = lowprec.split_bf16(B)
    full = (ah.astype(np.float64) + al) @ (bh.astype(np.float64) + bl)
    three = lowprec.matmul_lowprec(A, B, "bf16x3").astype(np.float64)
    assert np.allclose(three + al.astype(np.float64) @ bl, full, rtol=0, atol=1e-5)


def test_split3_bf16_planes():
    # three planes carry 24 significand bits: a float32 splits exactly (away from the subnormal range)
    rng = np.random.default_rng(5)
    x = (rng.standard_normal(20000) * 10.0 ** rng.uniform(-6, 6, 20000)).astype(np.float32)
    hi, mid, lo = lowprec.split3_bf16(x)
    assert np.array_equal(hi, lowprec.round_bf16(x))
    assert np.array_equal((hi.astype(np.float64) + mid) + lo, x.astype(np.float64))
    assert np.all(np.abs(mid) <= np.abs(x) * 2.0 ** -8) and np.all(np.abs(lo) <= np.abs(x) * 2.0 ** -16)


def test_six_term_product_reaches_float32_accuracy():
    rng = np.random.default_rng(6)
    A = rng.standard_normal((96, 96)).astype(np.float32)
    B = rng.standard_normal((96, 96)).astype(np.float32)
    exact = A.astype(np.float64) @ B.astype(np.float64)
    e6 = rel_frobenius_error(lowprec.matmul_lowprec(A, B, "bf16x6"), exact)[0]
    e3 = rel_frobenius_error(lowprec.matmul_lowprec(A, B, "bf16x3"), exact)[0]
    e32 = rel_frobenius_error((A @ B).astype(np.float32), exact)[0]
    assert e6 < 1.5e-7 and e6 < e3 / 30 and e6 < 4 * max(e32, 3e-8)
    # the six terms are the product of the plane sums minus the three dropped ones (mid*lo, lo*mid, lo*lo)
    ah, am, al = (t.astype(np.float64) for t in lowprec.split3_bf16(A))
    bh, bm, bl = (t.astype(np.float64) for t in lowprec.split3_bf16(B))
    six = al @ bh + ah @ bl + am @ bm + am @ bh + ah @ bm + ah @ bh
    assert np.allclose(six + am @ bl + al @ bm + al @ bl, exact, rtol=0, atol=1e-12)
    assert np.abs(six - exact).max() < 96 * 3 * 2.0 ** -24 * 16      # dropped terms: 2^-24 relative each


def test_ndb_with_six_term_products_matches_the_float32_floor():
    A32, _, _ = workloads.spd_stack(2, 64, -3.0, 0.0, seed=17)
    X = inverse_root_evd(A32.astype(np.float64), 4)
    e6 = rel_frobenius_error(lowprec.inverse_root_ndb_lowprec(A32, 4, 14, rounding="bf16x6"), X).max()
    e32 = rel_frobenius_error(lowprec.inverse_root_ndb_lowprec(A32, 4, 14, rounding="none"), X).max()
    e3 = rel_frobenius_error(lowprec.inverse_root_ndb_lowprec(A32, 4, 14, rounding="bf16x3"), X).max()
    print(f"NDB p=4 k=14 kappa=1e3: no rounding {e32:.2e}, bf16x6 {e6:.2e}, bf16x3 {e3:.2e}")
    assert e6 < 3 * e32 + 1e-6 and e3 > 3 * e6


def test_split_fp16_planes():
    # two fp16 planes carry 22 significand bits down to where the high plane goes subnormal (6e-5); below that the
    # error is absolute: half a subnormal step of the high plane's format at most
    rng = np.random.default_rng(7)
    x = (rng.standard_normal(40000) * 10.0 ** rng.uniform(-4, 0.5, 40000)).astype(np.float32)
    hi, lo = lowprec.split_fp16(x)
    assert np.array_equal(hi, lowprec.round_fp16(x))
    err = np.abs((hi.astype(np.float64) + lo) - x)
    assert np.all(err <= np.maximum(np.abs(x) * 2.0 ** -22, 2.0 ** -36))
    big = np.abs(x) > 1e-3
    assert (err[big] / np.abs(x[big])).max() > 2.0 ** -26          # and it is not better than that: a real bound
    # unscaled, the low plane is subnormal for values well inside the range of the iterates and loses its bits
    small = (np.abs(x) > 1e-3) & (np.abs(x) < 1e-2)
    naive = lowprec.round_fp16(x - hi)
    assert np.abs((hi.astype(np.float64) + naive) - x)[small].max() > 5 * err[small].max()


def test_fp16x3_product_is_close_to_the_float32_product():
    rng = np.random.default_rng(8)
    A = rng.standard_normal((96, 96)).astype(np.float32)
    B = rng.standard_normal((96, 96)).astype(np.float32)
    exact = A.astype(np.float64) @ B.astype(np.float64)
    e = {f: rel_frobenius_error(lowprec.matmul_lowprec(A, B, f), exact)[0] for f in ("fp16x3", "bf16x3", "bf16x6", "fp16")}
    e32 = rel_frobenius_error((A @ B).astype(np.float32), exact)[0]
    print(e, e32)
    assert e["fp16x3"] < 6e-7 and e["fp16x3"] < e["bf16x3"] / 20 and e["fp16x3"] < e["fp16"] / 500


def test_ndb_with_fp16x3_products_is_near_the_float32_floor():
    A32, _, _ = workloads.spd_stack(2, 64, -3.0, 0.0, seed=17)
    X = inverse_root_evd(A32.astype(np.float64), 4)
    e = {f: rel_frobenius_error(lowprec.inverse_root_ndb_lowprec(A32, 4, 14, rounding=f), X).max()
         for f in ("none", "fp16x3", "bf16x3", "fp16")}
    print("NDB p=4 k=14 kappa=1e3:", e)
    assert e["fp16x3"] < 10 * e["none"] and e["fp16x3"] < e["bf16x3"] / 5
