#!/usr/bin/env python3
"""Benchmark of the block-diagonal Shampoo hot path on one MI355X.

A step = one pass of the whole hot path over one synthetic gradient of the workload:
  accumulate (Algorithm 1 EMA lines) -> inverse 4th roots of all damped factor blocks by
  Newton-DB after Frobenius scaling (Sections 3.3, 3.4) -> preconditioned update.
Workload = one 4096 x 4096 linear layer with B = 1024: 16 gradient blocks, 32 stacked
1024 x 1024 factor blocks, gradient N(0, 1e-2^2), beta = 0.95, eps = 1e-6, p = 4, 10
Newton-DB updates per call, factors warmed with 20 seeded gradients.

Prints ONE JSON line.  `value` is factor blocks brought through the whole step per second
(inputs resident in HBM; nothing but the step's launches inside the timed region).  `roofline`
is for the batched matmul kernel, from HIP events recorded around each of its launches on the
library's stream in a separate instrumented pass after the timed steps.  `other_product_mode`
is the same workload with symmetric mode switched the other way, `configs` carries the other
four workload configurations (cfg1, cfg3, cfg4, cfg5), each with its own sampled float64-oracle
baseline, and `cpu_baseline` times the oracle step of the headline workload on the host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP32_MFMA_TFLOPS = 157.3      # MI355X dense fp32 matrix peak
PEAK_16BIT_MFMA_TFLOPS = 2500.0    # dense bf16 / fp16 matrix peak
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "gemm_f32_cfg2_hbm_traffic.txt")


def measured_traffic_per_block_product():
    """HBM bytes the fp32 matmul kernel moves per block product on the headline stack, as the committed rocprofv3
    summary states it (two --pmc runs, FETCH_SIZE and WRITE_SIZE, scaled by a copy kernel of known size; the
    algorithmic figure is 12 B^2 = 12.58e6).  Read from the summary, not typed here; None when it is missing."""
    import re
    try:
        m = re.search(r"=\s*([0-9.]+)e6 bytes per block product", open(TRAFFIC_PROFILE).read())
        return float(m.group(1)) * 1e6 if m else None
    except OSError:
        return None


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def blas_threads() -> int:
    import numpy  # noqa: F401  (loads the BLAS whose pool is counted)
    try:
        from threadpoolctl import threadpool_info
        return int(max([i.get("num_threads", 1) for i in threadpool_info()] or [1]))
    except Exception:
        return os.cpu_count() or 1


def cpu_root_baseline(N: int, B: int, p: int, seconds: float, what: str, of_total: int):
    """The float64 oracle root (eigendecomposition, oracle/evd.py) on well-conditioned seeded SPD blocks of edge B,
    repeated over `N` blocks until about `seconds` have passed (at least one pass).  Timing does not depend on the
    spectrum.  Returns blocks/s on the host threads the BLAS uses."""
    import numpy as np
    from oracle.evd import inverse_root_evd
    rng = np.random.default_rng(B + N)
    G = rng.standard_normal((N, B, B))
    A = np.matmul(G, np.swapaxes(G, 1, 2)) / B + 0.1 * np.eye(B)
    done, t0 = 0, time.perf_counter()
    while True:
        inverse_root_evd(A, p, eps=1e-6)
        done += N
        if time.perf_counter() - t0 >= seconds:
            break
    dt = time.perf_counter() - t0
    return dict(value=done / dt, unit="blocks/s", cores=blas_threads(), kind="oracle",
                sample=f"float64 eigendecomposition roots (p={p}) of {N} of the {of_total} {B}x{B} blocks of {what}, "
                       f"{done // N} pass(es), {dt:.1f} s")


def cpu_baseline(sample_blocks: int, B: int, beta: float, eps: float, p: int, repeats: int = 3):
    """Float64 oracle step (eigendecomposition roots) on `sample_blocks` gradient blocks."""
    import numpy as np
    import workloads
    from oracle import shampoo as oshampoo
    threads = blas_threads()
    L = np.zeros((sample_blocks, B, B))
    R = np.zeros((sample_blocks, B, B))
    for t in range(2):
        L, R = oshampoo.accumulate_factors(workloads.gradient_stack(sample_blocks, B, 9000 + t), L, R, beta)
    G = workloads.gradient_stack(sample_blocks, B, 9002)
    t0 = time.perf_counter()
    for _ in range(repeats):
        oshampoo.step(G, L, R, beta=beta, eps=eps, p=p)
    dt = (time.perf_counter() - t0) / repeats
    return dict(value=2 * sample_blocks / dt, unit="blocks/s", cores=int(threads), kind="oracle",
                seconds_per_step=dt,
                sample=f"{repeats} float64 oracle steps (accumulate, eigh roots of {2 * sample_blocks} factor "
                       f"blocks, precondition) on {sample_blocks} of the 16 gradient blocks, B={B}")


def sweep(dash, only_16bit=False):
    """Throughput of the inverse root alone on the shapes of the other workload configurations
    (cfg1: 16 x 128; cfg4: 256 x 256, 64 x 512, 4 x 2048; cfg5: 1024 x 1024), every method and
    precision.  Timing does not depend on the values, so the stacks are well-conditioned random SPD
    blocks; accuracy on the configurations' own spectra is the business of tests/test_gpu_configs.py.
    Returns a list of records; `mfma_frac` prices the executed flops against the peak of the operand type.
    `only_16bit` keeps the 16-bit cases on the cfg5 shape (short enough to run under a kernel trace)."""
    import torch
    from paper_2602_02016_amd import chebyshev_fit
    rows = []
    shapes = [("cfg1", 16, 128), ("cfg4", 256, 256), ("cfg4", 64, 512), ("cfg4", 4, 2048), ("cfg5", 1024, 1024)]
    if only_16bit:
        shapes = shapes[-1:]
    for cfg, N, B in shapes:
        gen = torch.Generator(device="cuda")
        gen.manual_seed(N + B)
        A = torch.empty(N, B, B, device="cuda")
        chunk = max(1, min(N, (1 << 28) // (B * B)))
        for i in range(0, N, chunk):                       # A = G G^T / B + 0.1 I, built in chunks
            Gm = torch.randn(min(chunk, N - i), B, B, device="cuda", generator=gen)
            A[i:i + chunk] = Gm @ Gm.transpose(1, 2) / B
        A += 0.1 * torch.eye(B, device="cuda")
        X = torch.empty_like(A)
        cases = []
        for pp in (2, 4):
            for k in (5, 10, 20):
                cases.append(("newton_db", pp, k, "fp32"))
            for d in (8, 16, 32):
                cases.append(("chebyshev", pp, d, "fp32"))
            cases.append(("coupled_newton", pp, 10, "fp32"))
        if cfg != "cfg5":          # the fastest fp32-accurate mode on the smaller shapes as well
            cases += [("newton_db", 4, 10, "fp16x3"), ("coupled_newton", 4, 10, "fp16x3"), ("chebyshev", 4, 16, "fp16x3")]
        if cfg == "cfg5":
            cases += [("newton_db", 4, 10, "bf16"), ("newton_db", 4, 10, "fp16"), ("newton_db", 4, 10, "bf16x3"),
                      ("newton_db", 4, 10, "bf16x6"), ("chebyshev", 4, 16, "bf16x6"),
                      ("coupled_newton", 4, 10, "bf16x6"),
                      ("newton_db", 4, 10, "fp16x3"), ("coupled_newton", 4, 10, "fp16x3"), ("chebyshev", 4, 16, "fp16x3"),
                      ("coupled_newton", 4, 10, "fp16"), ("chebyshev", 4, 16, "fp16")]
        if only_16bit:
            cases = [c for c in cases if c[3] != "fp32"]
        for method, pp, it, prec in cases:
            kw = dict(method=method, p=pp, iters=it, eps=1e-6, precision=prec)
            if method == "chebyshev":
                kw.update(cheb_coeffs=chebyshev_fit(pp, it, 0.05, 1.0), cheb_a=0.05, cheb_b=1.0)
            dash.inverse_root(A, X, **kw)                  # warm-up (also sizes the workspace)
            torch.cuda.synchronize()
            reps = 3 if N * B * B >= (1 << 28) else 10
            dash.reset_stats()
            t0 = time.perf_counter()
            for _ in range(reps):
                dash.inverse_root(A, X, **kw)
            torch.cuda.synchronize()
            ms = (time.perf_counter() - t0) * 1e3 / reps
            fl = dash.get_stats()["matmul_flops"] / reps
            peak = PEAK_FP32_MFMA_TFLOPS if prec == "fp32" else 2500.0
            rows.append(dict(cfg=cfg, N=N, B=B, method=method, p=pp, iters=it, precision=prec, ms=ms,
                             blocks_per_s=N / (ms * 1e-3), executed_tflops=fl / (ms * 1e-3) / 1e12,
                             mfma_frac=fl / (ms * 1e-3) / 1e12 / peak))
            log(f"{cfg} N={N:5d} B={B:5d} {method:14s} p={pp} it={it:2d} {prec:6s}: {ms:9.3f} ms "
                f"{rows[-1]['blocks_per_s']:10.0f} blocks/s {rows[-1]['executed_tflops']:7.1f} TFLOP/s "
                f"({100 * rows[-1]['mfma_frac']:.1f}%)")
        del A, X
    return rows


def hbm_kernels(dash):
    """Achieved HBM bandwidth of the memory-bound kernels of the path on a long stack (256 blocks of
    1024 x 1024 fp32 = 1 GiB, plus a ragged 4096 x 4000 layer for block()).  bytes = algorithmic bytes of
    the call (every operand read once, every result written once); peak 8 TB/s."""
    import torch
    N, B = 256, 1024
    gen = torch.Generator(device="cuda")
    gen.manual_seed(5)
    A = torch.randn(N, B, B, device="cuda", generator=gen)
    A = (A + A.transpose(1, 2)) * 0.01 + torch.eye(B, device="cuda")
    G = torch.randn(N, B, B, device="cuda", generator=gen) * 0.01
    U = torch.randn(N, B, B, device="cuda", generator=gen)
    Acc = torch.zeros(N, B, B, device="cuda")
    X = torch.empty_like(A)
    g = torch.randn(N, B, device="cuda", generator=gen)
    u = torch.empty_like(g)
    Wl = torch.randn(4096, 4000, device="cuda", generator=gen)
    V0 = torch.randn(B, 16, device="cuda", generator=gen)
    dash.set_power_iteration(V0, 4)
    blk = B * B * 4
    groups = {}

    def block():
        groups.update(dash.block_layer(Wl, 1024))

    cases = [
        ("block_norms frobenius (norm_partials + finalize)", lambda: dash.block_norms(A, scaling="frobenius"), N * blk),
        ("block_norms power iteration, 4 sweeps of pool 16", lambda: dash.block_norms(A, scaling="pi"), 4 * N * blk),
        ("graft_update (read G, U, Acc; write Acc)", lambda: dash.graft_update(G, U, Acc), 4 * N * blk),
        ("graft_scale in place (read G, U, Acc; then U again; write Acc, U)", lambda: dash.graft_scale(G, U, Acc), 6 * N * blk),
        ("accumulate_vector (read + write L)", lambda: dash.accumulate_vector(g, A, 0.95), 2 * N * blk),
        ("precondition_vector (read L)", lambda: dash.precondition_vector(A, g, u), N * blk),
        ("block_layer 4096 x 4000, B = 1024 (read + write)", block, 2 * Wl.numel() * 4),
        ("apply_update (read theta, update; write theta)", lambda: dash.apply_update(U, G, 0.1), 3 * N * blk),
    ]
    rows = []
    for name, fn, nbytes in cases:
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        reps = 10
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        us = (time.perf_counter() - t0) * 1e6 / reps
        rows.append(dict(kernel=name, us=us, algorithmic_bytes=nbytes, tb_per_s=nbytes / us / 1e6, frac_of_hbm_peak=nbytes / us / 1e6 / 8.0))
        log(f"{name:75s} {us:9.1f} us  {rows[-1]['tb_per_s']:5.2f} TB/s ({100 * rows[-1]['frac_of_hbm_peak']:.0f}% of 8 TB/s)")
    return rows



def _timed(fn, reps):
    """Mean wall time of fn() in ms over `reps` back-to-back calls, device idle before and after."""
    import torch
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / reps


def _root_record(dash, A, X, reps, peak, **kw):
    """One inverse-root configuration on the resident stack A: ms per call, blocks/s, and the flops of the tiles the
    launches computed (library statistics) against `peak`."""
    dash.inverse_root(A, X, **kw)                      # warm-up, sizes the workspace
    dash.reset_stats()
    ms = _timed(lambda: dash.inverse_root(A, X, **kw), reps)
    fl = dash.get_stats()["matmul_flops"] / reps
    tf = fl / (ms * 1e-3) / 1e12
    return dict(ms=ms, blocks_per_s=A.shape[0] / (ms * 1e-3), executed_tflops=tf, mfma_frac=tf / peak)


def _spd_stack_on_device(N, B, seed):
    """Well-conditioned random SPD blocks built on the device (timing does not depend on the values; accuracy on the
    configurations' own spectra is what tests/test_gpu_configs.py checks)."""
    import torch
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed)
    A = torch.empty(N, B, B, device="cuda")
    chunk = max(1, min(N, (1 << 28) // (B * B)))
    for i in range(0, N, chunk):
        Gm = torch.randn(min(chunk, N - i), B, B, device="cuda", generator=gen)
        A[i:i + chunk] = Gm @ Gm.transpose(1, 2) / B
    A += 0.1 * torch.eye(B, device="cuda")
    return A


def other_configs(dash, cpu: bool):
    """Driver-visible numbers of the workload configurations other than the headline one.  Inputs are resident in HBM
    before any timed call; each record carries its own sampled float64-oracle baseline (host threads stated)."""
    import torch
    import workloads
    from paper_2602_02016_amd import chebyshev_fit
    out = {}
    coef16 = chebyshev_fit(4, 16, 0.05, 1.0)
    cheb = dict(method="chebyshev", p=4, iters=16, eps=1e-6, cheb_coeffs=coef16, cheb_a=0.05, cheb_b=1.0)
    ndb = dict(method="newton_db", p=4, iters=10, eps=1e-6)

    # cfg1: 16 blocks of 128 -- bound by launch latency, reported as time per stack
    c1 = workloads.CFG1
    A = _spd_stack_on_device(c1["N"], c1["B"], 11)
    X = torch.empty_like(A)
    r_ndb = _root_record(dash, A, X, 50, PEAK_FP32_MFMA_TFLOPS, **ndb)
    r_ch = _root_record(dash, A, X, 50, PEAK_FP32_MFMA_TFLOPS, **cheb)
    out["cfg1"] = {"workload": "cfg1: inverse 4th root of 16 fp32 SPD blocks, B=128",
                   "newton_db_k10": dict(us_per_stack=r_ndb["ms"] * 1e3, **r_ndb),
                   "chebyshev_d16": dict(us_per_stack=r_ch["ms"] * 1e3, **r_ch),
                   "note": "latency-bound: dependent launches of a few microseconds each; not a roofline point"}
    if cpu:
        out["cfg1"]["cpu_baseline"] = cpu_root_baseline(c1["N"], c1["B"], 4, 1.0, "cfg1", c1["N"])
    del A, X

    # cfg4: 64 MiB stacks of three block sizes
    out["cfg4"] = {"workload": "cfg4: N*B^2 = 2^24 stacks, Newton-DB k=10 and Chebyshev d=16, p=4", "shapes": []}
    for B, N in workloads.CFG4["shapes"]:
        A = _spd_stack_on_device(N, B, 40 + B)
        X = torch.empty_like(A)
        rec = {"B": B, "N": N, "newton_db_k10": _root_record(dash, A, X, 10, PEAK_FP32_MFMA_TFLOPS, **ndb),
               "chebyshev_d16": _root_record(dash, A, X, 10, PEAK_FP32_MFMA_TFLOPS, **cheb)}
        if cpu:
            n_cpu = max(1, min(N, (1 << 22) // (B * B) * 4))          # 64 / 16 / 4 blocks
            rec["cpu_baseline"] = cpu_root_baseline(n_cpu, B, 4, 2.0, "cfg4", N)
        out["cfg4"]["shapes"].append(rec)
        del A, X

    # cfg5: 1024 blocks of 1024, fp32 and bf16 operands (the latter priced against the 16-bit peak)
    c5 = workloads.CFG5
    A = _spd_stack_on_device(c5["N"], c5["B"], 55)
    X = torch.empty_like(A)
    out["cfg5"] = {"workload": "cfg5 shape: 1024 blocks of 1024x1024, Newton-DB p=4 k=10 (timing; the ill-conditioned "
                               "spectra and the error-vs-k table are in tests/test_gpu_configs.py)",
                   "fp32": _root_record(dash, A, X, 3, PEAK_FP32_MFMA_TFLOPS, **ndb),
                   "bf16_operands": _root_record(dash, A, X, 5, PEAK_16BIT_MFMA_TFLOPS, precision="bf16", **ndb),
                   "fp16x3_operands": _root_record(dash, A, X, 3, PEAK_16BIT_MFMA_TFLOPS, precision="fp16x3", **ndb)}
    out["cfg5"]["fp16x3_operands"]["note"] = ("two fp16 planes, three plane products per product: executed_tflops counts "
                                              "one product per multi-segment product; MFMA work is three times that")
    if cpu:
        out["cfg5"]["cpu_baseline"] = cpu_root_baseline(8, c5["B"], 4, 3.0, "cfg5", c5["N"])
    del A, X

    # cfg3: the whole 24-layer stack, one step (accumulate, 3072 roots in chunks of 512, 1536 updates)
    c3 = workloads.CFG3
    N, B = workloads.cfg3_num_gradient_blocks(), c3["B"]
    S = torch.zeros(2 * N, B, B, device="cuda")
    X = torch.empty_like(S)
    G = torch.empty(N, B, B, device="cuda")
    U = torch.empty_like(G)
    nf = torch.zeros(2 * N, dtype=torch.int32, device="cuda")
    gen = torch.Generator(device="cuda")
    gen.manual_seed(c3["seed_base"])
    ws = dash.workspace_bytes(512, B)
    for t in range(3):                                   # two warm-up gradients, then the gradient of the timed step
        torch.randn(G.shape, device="cuda", generator=gen, out=G)
        G.mul_(c3["grad_std"])
        if t < 2:
            dash.accumulate_factors(G, S[:N], S[N:], c3["beta"])
    step = lambda: dash.step(G, S, X, U, beta=c3["beta"], eps=c3["eps"], p=c3["p"], iters=c3["ndb_iters"],
                             nonfinite_out=nf, workspace_max_bytes=ws)
    step()                                               # warm-up step
    dash.reset_stats()
    ms = _timed(step, 2)
    fl = dash.get_stats()["matmul_flops"] / 2
    assert int(nf.sum().item()) == 0, "non-finite root in cfg3"
    out["cfg3"] = {"workload": "cfg3: 24-layer decoder (d=2048, FFN 8192), B=1024: 1536 gradient blocks, 3072 factor blocks "
                               "(12 GiB), one step = accumulate + 3072 inverse 4th roots (chunks of 512) + 1536 updates",
                   "step_s": ms * 1e-3, "blocks_per_s": 2 * N / (ms * 1e-3),
                   "executed_tflops": fl / (ms * 1e-3) / 1e12,
                   "mfma_frac_executed": fl / (ms * 1e-3) / 1e12 / PEAK_FP32_MFMA_TFLOPS}
    del S, X, G, U
    if cpu:
        b = cpu_baseline(8, B, c3["beta"], c3["eps"], c3["p"], repeats=1)
        b["sample"] = b["sample"].replace("of the 16 gradient blocks", f"of the {N} gradient blocks")
        out["cfg3"]["cpu_baseline"] = b
    torch.cuda.empty_cache()
    return out


def vendor_context(dash):
    """Context only: the vendor's batched matmul (torch.bmm, i.e. the library the paper's own implementation calls) on
    the same shapes as the library's plain product, and Newton-DB (Section 3.3, p=4, k=10) written with torch ops -- bmm
    plus separate elementwise passes, every product in full, nothing skipped -- beside dash_inverse_root on the same
    stack.  None of this is part of the product or of any reported roofline figure."""
    import torch
    torch.backends.cuda.matmul.allow_tf32 = False
    rows = []
    for N, B in ((32, 1024), (256, 1024), (256, 256), (64, 512)):
        gen = torch.Generator(device="cuda")
        gen.manual_seed(N + B)
        A = torch.randn(N, B, B, device="cuda", generator=gen) * 0.1
        Bm = torch.randn(N, B, B, device="cuda", generator=gen) * 0.1
        Cm = torch.empty_like(A)
        fl = N * 2.0 * B ** 3
        rec = {"N": N, "B": B}
        for name, fn in (("vendor_fp32_tflops", lambda: torch.bmm(A, Bm, out=Cm)),
                         ("dash_fp32_tflops", lambda: dash.gemm_batched(A, Bm, Cm))):
            fn()
            rec[name] = fl / (_timed(fn, 10) * 1e-3) / 1e12
        Ah, Bh = A.bfloat16(), Bm.bfloat16()
        Ch = torch.empty_like(Ah)
        torch.bmm(Ah, Bh, out=Ch)
        rec["vendor_bf16_in_bf16_out_tflops"] = fl / (_timed(lambda: torch.bmm(Ah, Bh, out=Ch), 10) * 1e-3) / 1e12
        dash.gemm_batched(A, Bm, Cm, precision="bf16")
        rec["dash_bf16_incl_operand_cast_fp32_out_tflops"] = fl / (_timed(lambda: dash.gemm_batched(A, Bm, Cm, precision="bf16"), 10) * 1e-3) / 1e12
        rows.append(rec)
        log("  ".join(f"{k}={v:.1f}" if isinstance(v, float) else f"{k}={v}" for k, v in rec.items()))
        del A, Bm, Cm, Ah, Bh, Ch
    N, B, k = 32, 1024, 10
    A = _spd_stack_on_device(N, B, 5)
    I = torch.eye(B, device="cuda")

    def call(M):
        E = 1.5 * I - 0.5 * M
        Y, Z = torch.bmm(M, E), E
        for _ in range(k - 1):
            E = 1.5 * I - 0.5 * torch.bmm(Z, Y)
            Y, Z = torch.bmm(Y, E), torch.bmm(E, Z)
        return Y, Z

    def root4():
        s = torch.linalg.matrix_norm(A + 1e-6 * I).view(-1, 1, 1)
        Y, _ = call((A + 1e-6 * I) / s)
        _, Z = call(Y)
        return Z * s ** -0.25

    Xt = root4()
    ms_t = _timed(root4, 5)
    X = torch.empty_like(A)
    dash.inverse_root(A, X, p=4, iters=k, eps=1e-6)
    ms_d = _timed(lambda: dash.inverse_root(A, X, p=4, iters=k, eps=1e-6), 5)
    diff = float(((Xt - X).flatten(1).norm(dim=1) / X.flatten(1).norm(dim=1)).max())
    ndb = {"workload": "Newton-DB p=4 k=10 on 32 blocks of 1024, fp32", "torch_ops_ms": ms_t, "dash_inverse_root_ms": ms_d,
           "max_rel_diff": diff}
    log(f"Newton-DB p=4 k=10, 32 x 1024: torch ops {ms_t:.2f} ms, dash_inverse_root {ms_d:.2f} ms, results differ by {diff:.1e}")
    return {"matmul": rows, "newton_db": ndb}


def design_choices(dash):
    """Before/after rows of the design choices that can be switched from outside (all through the C ABI): symmetric
    mode, lanes, chunk size.  Wall time per inverse-root call on resident stacks, each pair measured back to back on
    the same box.  Returns a list of records (and prints a table on stderr)."""
    import torch
    from paper_2602_02016_amd import chebyshev_fit
    coef = chebyshev_fit(4, 16, 0.05, 1.0)
    cheb = dict(method="chebyshev", p=4, iters=16, eps=1e-6, cheb_coeffs=coef, cheb_a=0.05, cheb_b=1.0)
    ndb = dict(method="newton_db", p=4, iters=10, eps=1e-6)
    cn = dict(method="coupled_newton", p=4, iters=10, eps=1e-6)
    rows = []

    def pair(choice, what, setter, A, X, reps, kw, cap_off=None, cap_on=None):
        res = {}
        for state in ("off", "on", "off", "on"):             # two alternating repetitions: the mean of each
            setter(state == "on")
            cap = cap_on if state == "on" else cap_off
            call = lambda: dash.inverse_root(A, X, **kw)
            call()                                            # (sizes the binding's workspace tensor for the whole stack)
            if cap is not None:                               # hand the library only `cap` bytes of it: it walks the stack in chunks
                import ctypes
                dash._check(dash.lib.dash_set_workspace(dash.h, ctypes.c_void_p(dash._ws.data_ptr()), int(cap)))
                call()
            res.setdefault(state, []).append(_timed(call, reps))
        setter(True)
        if cap_on is not None:
            dash.set_workspace_bytes(0)                       # the whole tensor again
        off, on = sum(res["off"]) / 2, sum(res["on"]) / 2
        rows.append(dict(choice=choice, workload=what, off_ms=off, on_ms=on, gain=off / on - 1.0))
        log(f"{choice:34s} {what:58s} off {off:9.3f} ms   on {on:9.3f} ms   {100 * (off / on - 1):+6.1f} %")

    for N, B, reps in ((32, 1024, 5), (256, 1024, 3), (256, 256, 10)):
        A = _spd_stack_on_device(N, B, 90 + B)
        X = torch.empty_like(A)
        for name, kw in (("Newton-DB p=4 k=10", ndb), ("Chebyshev d=16", cheb)):
            pair("symmetric mode (mirrored products)", f"{N} x {B}, {name}, fp32", dash.set_symmetric, A, X, reps, kw)
        del A, X
    for N, B in ((256, 256), (1024, 256), (64, 512), (128, 384)):
        A = _spd_stack_on_device(N, B, 91 + B)
        X = torch.empty_like(A)
        for name, kw in (("Newton-DB p=4 k=10", ndb), ("Chebyshev d=16", cheb), ("Coupled-Newton p=4 k=10", cn),
                         ("Newton-DB, two fp16 planes", dict(ndb, precision="fp16x3")), ("Newton-DB, bf16 operands", dict(ndb, precision="bf16"))):
            pair("lanes (two streams, B <= 512)", f"{N} x {B}, {name}", dash.set_lanes, A, X, 10, kw)
        del A, X
    A = _spd_stack_on_device(1024, 1024, 92)
    X = torch.empty_like(A)
    for chunk in (32, 128, 256):
        pair(f"chunks of 1024 (off) vs {chunk} blocks (on)", "1024 x 1024, Newton-DB p=4 k=10, fp32", lambda on: None, A, X, 2, ndb,
             cap_off=dash.workspace_bytes(1024, 1024), cap_on=dash.workspace_bytes(chunk, 1024))
    del A, X
    return rows


def headline(dash, args, symmetric: bool, grads, S, X, U, nf, c):
    """W untimed warm-up steps, then exactly K timed steps of the cfg2 workload with the library's event timing OFF
    (nothing but the step's own launches inside the timed region); after that a second, instrumented pass of a few
    steps with HIP events around every matmul launch for the roofline figure.  Returns (ms_per_step, stats of the
    instrumented pass, its number of steps)."""
    import torch
    B, beta, eps, p, k = c["B"], c["beta"], c["eps"], c["p"], c["ndb_iters"]
    dash.set_symmetric(symmetric)

    def one_step(i):
        dash.step(grads[i % len(grads)], S, X, U, beta=beta, eps=eps, p=p, iters=k, nonfinite_out=nf)

    for i in range(args.warmup):
        one_step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        one_step(args.warmup + i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    assert int(nf.sum().item()) == 0, "non-finite root in the benchmark workload"
    # instrumented pass: per-launch HIP events on the library's stream (not part of ms_per_step)
    n_inst = max(2, min(args.steps, 5))
    dash.set_timing(True)
    one_step(0)                      # creates the library's event pool (host work that would starve the stream)
    torch.cuda.synchronize()
    dash.reset_stats()
    for i in range(n_inst):
        one_step(i)
    st = dash.get_stats()
    dash.set_timing(False)
    return dt * 1e3 / args.steps, st, n_inst


def roofline_of(st, n_inst, B, ms_per_step):
    """Roofline object of the dominant kernel (the non-transposed fp32 matmul instance: every Newton-DB and
    precondition product) from the instrumented pass."""
    flop_per_product = 2.0 * B ** 3
    mm_ms = st["variant_ms"][0]
    launches = st["variant_launches"][0]
    # flops of the output tiles the launches really computed (symmetric products compute the tiles on and above the
    # diagonal only), never the full-product count
    achieved = st["variant_flops"][0] / (mm_ms * 1e-3) / 1e12 if mm_ms > 0 else 0.0
    tile_fraction = st["variant_flops"][0] / (flop_per_product * st["variant_block_products"][0])
    per_product = measured_traffic_per_block_product()
    return dict(bound="mfma", kernel="dash::gemm_f32_kernel<128, false, false, false>",
                achieved=achieved, peak=PEAK_FP32_MFMA_TFLOPS, unit="TFLOP/s", frac=achieved / PEAK_FP32_MFMA_TFLOPS,
                computed_tile_fraction=tile_fraction,
                full_product_equivalent_tflops=achieved / tile_fraction,
                traffic=None if per_product is None else per_product * st["variant_block_products"][0] / max(launches, 1),
                traffic_note="HBM bytes per mean launch = bytes per block product stated in "
                             "profiles/gemm_f32_cfg2_hbm_traffic.txt (rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE runs, "
                             "scaled by a copy kernel of known size; collected offline on full-product launches) x "
                             "block products per launch of this run",
                algorithmic_bytes=12.0 * B * B * st["variant_block_products"][0] / max(launches, 1),
                launches_per_step=launches / n_inst,
                mean_launch_ms=mm_ms / max(launches, 1),
                timing_note="HIP events around each launch on the library's stream, in a separate instrumented pass of "
                            f"{n_inst} steps after the timed steps (the timed steps run with event timing off)",
                instrumented_matmul_ms_per_step=mm_ms / n_inst)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-blocks", type=int, default=16)
    ap.add_argument("--cpu-repeats", type=int, default=4)
    ap.add_argument("--root-only-reps", type=int, default=-1,
                    help="extra timed calls of the inverse root alone (default steps/2; 0 = none)")
    ap.add_argument("--full-products", action="store_true",
                    help="headline with the library's symmetric mode off (every product computed in full); the default "
                         "run reports that variant beside the headline anyway")
    ap.add_argument("--headline-only", action="store_true",
                    help="skip the records of the other configurations and of the variants (short run, e.g. under a profiler)")
    ap.add_argument("--pmc-probe", action="store_true",
                    help="for rocprofv3 --pmc: one device copy of known size, then three launches of the "
                         "matmul kernel on the workload's 32-block stack; prints nothing else")
    ap.add_argument("--pmc-probe-16bit", action="store_true",
                    help="as --pmc-probe with the 16-bit kernel: a device copy of known size, then three launches "
                         "of the bf16-operand matmul on 256 blocks (fp32 result)")
    ap.add_argument("--pmc-probe-step", action="store_true",
                    help="for rocprofv3 --pmc: the headline workload's factors, then two whole steps (every launch of "
                         "the step under the counters); prints the host-side flop count of those two steps")
    ap.add_argument("--pmc-probe-ndb16", action="store_true",
                    help="for rocprofv3 --pmc: one bf16-operand Newton-DB call (p=4, k=10) on 256 blocks of 1024; "
                         "prints the host-side flop count")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the headline step: inverse-root throughput on the shapes of the other "
                         "configurations, all methods and precisions (table on stderr, one JSON line)")
    ap.add_argument("--sweep-16bit", action="store_true",
                    help="as --sweep, but only the 16-bit cases on 1024 blocks of 1024 (bf16, fp16, split bf16)")
    ap.add_argument("--vendor-context", action="store_true",
                    help="context only: the vendor's batched matmul (torch.bmm) and a torch-ops Newton-DB beside the library "
                         "on the same shapes (table on stderr, one JSON line)")
    ap.add_argument("--design-choices", action="store_true",
                    help="instead of the headline step: before/after rows of the switchable design choices (symmetric "
                         "mode, lanes, chunk size) on resident stacks (table on stderr, one JSON line)")
    ap.add_argument("--hbm-kernels", action="store_true",
                    help="instead of the headline step: achieved bandwidth of the memory-bound kernels on a "
                         "1 GiB stack (table on stderr, one JSON line)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (blocks are independent, so the path would shard over "
              "them, but no multi-GPU code is built); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import workloads
    from paper_2602_02016_amd import Dash

    c = workloads.CFG2
    B, beta, eps, p, k = c["B"], c["beta"], c["eps"], c["p"], c["ndb_iters"]
    N = workloads.cfg2_num_blocks()            # 16 gradient blocks -> 32 factor blocks
    dev = torch.device("cuda", 0)
    dash = Dash(0)
    dash.set_symmetric(not args.full_products)

    if args.vendor_context:
        print(json.dumps({"vendor_context": vendor_context(dash), "n_gpus": 1, "data": "synthetic"}))
        return

    if args.design_choices:
        print(json.dumps({"design_choices": design_choices(dash), "unit": "ms per inverse-root call", "n_gpus": 1, "data": "synthetic"}))
        return

    if args.hbm_kernels:
        print(json.dumps({"hbm_kernels": hbm_kernels(dash), "peak_tb_per_s": 8.0, "n_gpus": 1, "data": "synthetic"}))
        return

    if args.sweep or args.sweep_16bit:
        print(json.dumps({"sweep": sweep(dash, only_16bit=args.sweep_16bit), "unit": "blocks/s", "n_gpus": 1, "data": "synthetic",
                          "symmetric_products": not args.full_products}))
        return

    if args.pmc_probe_16bit:
        gen = torch.Generator(device=dev)
        gen.manual_seed(1)
        nb = 256
        A = torch.randn(nb, B, B, device=dev, generator=gen)
        Bm = torch.randn(nb, B, B, device=dev, generator=gen)
        Cm = torch.empty_like(A)
        dash.gemm_batched(A[:8], Bm[:8], Cm[:8], precision="bf16")      # sizes the workspace
        torch.cuda.synchronize()
        Cm[:32].copy_(A[:32])                   # reference: reads 128 MiB, writes 128 MiB
        torch.cuda.synchronize()
        for _ in range(3):
            # casts the operands to bf16 (elementwise kernel), then the 16-bit matmul kernel:
            # algorithmic reads 2 x 512 MiB of bf16, writes 1 GiB of fp32
            dash.gemm_batched(A, Bm, Cm, precision="bf16")
        torch.cuda.synchronize()
        print(json.dumps({"pmc_probe_16bit": "copy of %d bytes then 3 bf16 matmul launches on %d blocks" % (32 * B * B * 4, nb)}))
        return

    if args.pmc_probe_ndb16:
        A = _spd_stack_on_device(256, B, 55)
        Xo = torch.empty_like(A)
        kw = dict(p=4, iters=10, eps=1e-6, precision="bf16")
        dash.inverse_root(A[:8], Xo[:8], **kw)
        dash.ensure_workspace(256, B, "newton_db", 4, "bf16")
        torch.cuda.synchronize()
        dash.reset_stats()
        dash.inverse_root(A, Xo, **kw)
        torch.cuda.synchronize()
        st = dash.get_stats()
        print(json.dumps({"pmc_probe_ndb16": "one bf16-operand Newton-DB call, p=4 k=10, 256 blocks of 1024",
                          "host_side_matmul_flops": st["matmul_flops"], "matmul_launches": st["matmul_launches"]}))
        return

    if args.pmc_probe:
        gen = torch.Generator(device=dev)
        gen.manual_seed(1)
        A = torch.randn(2 * N, B, B, device=dev, generator=gen)
        Bm = torch.randn(2 * N, B, B, device=dev, generator=gen)
        Cm = torch.empty_like(A)
        torch.cuda.synchronize()
        Cm.copy_(A)                             # reference: reads 128 MiB, writes 128 MiB
        torch.cuda.synchronize()
        for _ in range(3):
            dash.gemm_batched(A, Bm, Cm)        # algorithmic: reads 256 MiB, writes 128 MiB
        torch.cuda.synchronize()
        print(json.dumps({"pmc_probe": "copy of %d bytes then 3 matmul launches" % (A.numel() * 4)}))
        return

    S = torch.zeros(2 * N, B, B, device=dev)
    X = torch.empty_like(S)
    U = torch.empty(N, B, B, device=dev)
    nf = torch.zeros(2 * N, dtype=torch.int32, device=dev)

    # warm the factors with the seeded gradients of the workload recipe
    for t in range(c["warm_steps"]):
        G = torch.from_numpy(workloads.gradient_stack(N, B, c["seed_base"] + t, c["grad_std"])).to(dev)
        dash.accumulate_factors(G, S[:N], S[N:], beta)
    torch.cuda.synchronize()

    # gradients of the warm-up and timed steps, resident in HBM before timing starts
    gen = torch.Generator(device=dev)
    gen.manual_seed(c["seed_base"] + 1000)
    total = args.warmup + args.steps
    grads = [torch.randn(N, B, B, device=dev, generator=gen) * c["grad_std"] for _ in range(min(total, 8))]

    if args.pmc_probe_step:
        dash.step(grads[0], S, X, U, beta=beta, eps=eps, p=p, iters=k, nonfinite_out=nf)     # sizes the workspace
        torch.cuda.synchronize()
        dash.reset_stats()
        for i in range(2):
            dash.step(grads[i + 1], S, X, U, beta=beta, eps=eps, p=p, iters=k, nonfinite_out=nf)
        torch.cuda.synchronize()
        st = dash.get_stats()
        print(json.dumps({"pmc_probe_step": "20 accumulations, one untimed step, then two whole cfg2 steps",
                          "host_side_matmul_flops_of_the_two_steps": st["matmul_flops"],
                          "matmul_launches_of_the_two_steps": st["matmul_launches"],
                          "symmetric_products": not args.full_products}))
        return

    S_warm = S.clone()
    symmetric = not args.full_products
    ms_per_step, st, n_inst = headline(dash, args, symmetric, grads, S, X, U, nf, c)
    blocks_per_s = 2 * N / (ms_per_step * 1e-3)
    roofline = roofline_of(st, n_inst, B, ms_per_step)
    flop_per_product = 2.0 * B ** 3
    achieved_tflops = roofline["achieved"]

    # the inverse roots alone (same stack, same call the step makes), timed the same way
    reps = args.root_only_reps if args.root_only_reps >= 0 else max(1, args.steps // 2)
    if args.headline_only:
        reps = 0
    root_ms = _timed(lambda: dash.inverse_root(S, X, p=p, iters=k, eps=eps, nonfinite_out=nf), reps) if reps > 0 else 0.0

    # the same workload with the other setting of symmetric mode (a reading of the paper, not its product set: with it
    # on, the residual Z Y of Section 3.3 is computed on its upper triangle of tiles and mirrored)
    other_mode = None
    if not args.headline_only:
        S_now = S.clone()
        S.copy_(S_warm)
        ms2, st2, n2 = headline(dash, args, not symmetric, grads, S, X, U, nf, c)
        r2 = roofline_of(st2, n2, B, ms2)
        other_mode = {"symmetric_products": not symmetric, "ms_per_step": ms2, "value": 2 * N / (ms2 * 1e-3),
                      "unit": "blocks/s", "steps": args.steps, "warmup": args.warmup,
                      "roofline": {kk: r2[kk] for kk in ("achieved", "peak", "unit", "frac", "computed_tile_fraction",
                                                         "launches_per_step", "mean_launch_ms")},
                      "step_mfma_frac_executed": st2["matmul_flops"] / n2 / (ms2 * 1e-3) / 1e12 / PEAK_FP32_MFMA_TFLOPS}
        dash.set_symmetric(symmetric)
        S.copy_(S_now)
        dash.inverse_root(S, X, p=p, iters=k, eps=eps, nonfinite_out=nf)      # X of the headline mode again
        del S_now
    del S_warm

    # the same stack with the paper's multi-Power-Iteration scaling (Sections 3.4, 3.5), which converges in
    # half the updates on these factors: 5 per call against the headline's 10 (context, not the headline)
    pi_variant = None
    if reps > 0:
        import numpy as np
        X10 = X[:2].cpu().numpy().astype(np.float64)
        V0 = torch.from_numpy(workloads.start_vectors(B, 16, 77)).to(dev)
        dash.set_power_iteration(V0, 4)
        Xp = torch.empty_like(S)
        dash.inverse_root(S, Xp, p=p, iters=5, eps=eps, scaling="pi", nonfinite_out=nf)
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        for _ in range(reps):
            dash.inverse_root(S, Xp, p=p, iters=5, eps=eps, scaling="pi", nonfinite_out=nf)
        torch.cuda.synchronize()
        pi_ms = (time.perf_counter() - t2) * 1e3 / reps
        X5 = Xp[:2].cpu().numpy().astype(np.float64)
        diff = float(max(np.linalg.norm(X5[i] - X10[i]) / np.linalg.norm(X10[i]) for i in range(2)))
        pi_variant = {"scaling": "2*lambda_PI, 4 sweeps, pool 16", "ndb_iters": 5, "ms": pi_ms,
                      "blocks_per_s": 2 * N / (pi_ms * 1e-3),
                      "rel_diff_to_headline_roots": diff}
        # and both together: that scaling with two-plane split fp16 operands (DASH_FP16X3)
        dash.inverse_root(S, Xp, p=p, iters=5, eps=eps, scaling="pi", precision="fp16x3", nonfinite_out=nf)
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        for _ in range(reps):
            dash.inverse_root(S, Xp, p=p, iters=5, eps=eps, scaling="pi", precision="fp16x3", nonfinite_out=nf)
        torch.cuda.synchronize()
        pi3_ms = (time.perf_counter() - t2) * 1e3 / reps
        X5 = Xp[:2].cpu().numpy().astype(np.float64)
        diff3 = float(max(np.linalg.norm(X5[i] - X10[i]) / np.linalg.norm(X10[i]) for i in range(2)))
        pi_variant["with_fp16x3_operands"] = {"ms": pi3_ms, "blocks_per_s": 2 * N / (pi3_ms * 1e-3),
                                              "rel_diff_to_headline_roots": diff3}
        del Xp

    # the same roots with split 16-bit operands (context, not the headline): three bf16 planes and six plane
    # products (DASH_BF16X6), two fp16 planes with a scaled low plane and three products (DASH_FP16X3); fp32
    # accumulation in both.  Time, difference to the fp32 roots, the residual ||X^4 (A + eps I) - I||_F / sqrt(B)
    # formed in float64 on one block, and the whole step with these roots (accumulation and update stay on the
    # fp32 MFMA path).
    split_variants = {}
    if reps > 0:
        def residual(Xb, Ab):
            X64 = Xb.double()
            X2 = X64 @ X64
            R = X2 @ X2 @ (Ab.double() + eps * torch.eye(B, device=dev, dtype=torch.float64)) - torch.eye(B, device=dev, dtype=torch.float64)
            return float(R.norm() / B ** 0.5)
        S_keep = S.clone()                  # the steps below move the factors on: every variant starts from the same
        res32 = residual(X[0], S[0])
        notes = {"bf16x6": "operands as three bf16 planes, six plane products, fp32 accumulation",
                 "fp16x3": "operands as two fp16 planes (low plane scaled by 2^11), three plane products, fp32 accumulation"}
        for prec in ("bf16x6", "fp16x3"):
            S.copy_(S_keep)
            Xs = torch.empty_like(S)
            dash.inverse_root(S, Xs, p=p, iters=k, eps=eps, precision=prec, nonfinite_out=nf)
            torch.cuda.synchronize()
            t3 = time.perf_counter()
            for _ in range(reps):
                dash.inverse_root(S, Xs, p=p, iters=k, eps=eps, precision=prec, nonfinite_out=nf)
            torch.cuda.synchronize()
            v_ms = (time.perf_counter() - t3) * 1e3 / reps
            # the 16-bit kernel's own roofline on these calls: HIP events around each of its launches (a second,
            # instrumented pass; the library counts one product per multi-segment product, hence the factor)
            segs = 6 if prec == "bf16x6" else 3
            dash.reset_stats(); dash.set_timing(True)
            for _ in range(max(1, reps // 2)):
                dash.inverse_root(S, Xs, p=p, iters=k, eps=eps, precision=prec, nonfinite_out=nf)
            torch.cuda.synchronize()
            sv = dash.get_stats(); dash.set_timing(False)
            half_tflops = segs * sv["variant_flops"][0] / (sv["variant_ms"][0] * 1e-3) / 1e12
            dv = float(((Xs[:2] - X[:2]).double().flatten(1).norm(dim=1) / X[:2].double().flatten(1).norm(dim=1)).max())
            rec = {"precision": prec + " (" + notes[prec] + ")", "ndb_iters": k, "ms": v_ms,
                   "blocks_per_s": 2 * N / (v_ms * 1e-3), "speedup_over_fp32_roots": root_ms / v_ms,
                   "rel_diff_to_headline_roots": dv, "residual_fp32": res32, "residual": residual(Xs[0], S[0]),
                   "roofline": {"bound": "mfma", "kernel": "dash::gemm_half_kernel<dash::%s, 256, false, false>"
                                                            % ("Bf16" if prec == "bf16x6" else "Fp16"),
                                "achieved": half_tflops, "peak": 2500.0, "unit": "TFLOP/s", "frac": half_tflops / 2500.0,
                                "launches_per_call": sv["variant_launches"][0] / max(1, reps // 2),
                                "mean_launch_ms": sv["variant_ms"][0] / max(sv["variant_launches"][0], 1),
                                "note": "MFMA work of the K segments executed (symmetric launches: computed tiles only)"}}
            Us = torch.empty_like(U)
            dash.step(grads[0], S, Xs, Us, beta=beta, eps=eps, p=p, iters=k, nonfinite_out=nf, precision=prec)
            torch.cuda.synchronize()
            t4 = time.perf_counter()
            for i in range(reps):
                dash.step(grads[(i + 1) % len(grads)], S, Xs, Us, beta=beta, eps=eps, p=p, iters=k, nonfinite_out=nf,
                          precision=prec)
            torch.cuda.synchronize()
            rec["step_ms"] = (time.perf_counter() - t4) * 1e3 / reps
            rec["step_blocks_per_s"] = 2 * N / (rec["step_ms"] * 1e-3)
            assert int(nf.sum().item()) == 0, "non-finite root with " + prec + " operands"
            split_variants[prec] = rec
            del Xs, Us
        S.copy_(S_keep)
        del S_keep

    # the paper's own matmul count for the root (3k-2 per call, two calls) prices the
    # inverse root alone: what the headline "blocks/s at B=1024" would be without the
    # accumulate and precondition products of the step
    paper_products_root = 2 * (3 * k - 2)
    exec_products_root = 2 * (3 * k - 3)
    out = {
        "metric": "inverse-4th-root blocks/sec at B=1024 (Newton-DB), whole optimizer step",
        "value": blocks_per_s,
        "unit": "blocks/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "cfg2: one Shampoo step of a 4096x4096 layer, B=1024, 16 gradient blocks / 32 factor "
                               "blocks, Newton-DB p=4 with 10 updates per call, Frobenius scaling, beta=0.95, "
                               "eps=1e-6, factors warmed with 20 seeded gradients; symmetric mode "
                               + ("on: the residual product Z Y of Newton-DB and G G^T, G^T G compute their upper "
                                  "triangle of tiles and mirror it -- a reading of the paper, whose Section 3.3 computes "
                                  "Z Y in full (the full-products twin of this number is in other_product_mode)"
                                  if symmetric else "off: every product computed in full, the paper's product set"),
                   "N_gradient_blocks": N, "N_factor_blocks": 2 * N, "B": B, "p": p, "ndb_iters": k,
                   "symmetric_products": symmetric},
        "roofline": roofline,
        "step_mfma_frac_paper_count": (2 * N * paper_products_root + 4 * N) * flop_per_product
                                      / (ms_per_step * 1e-3) / 1e12 / PEAK_FP32_MFMA_TFLOPS,
        "step_mfma_frac_executed": st["matmul_flops"] / n_inst / (ms_per_step * 1e-3) / 1e12 / PEAK_FP32_MFMA_TFLOPS,
        "inverse_root_only": None if reps == 0 else {"blocks_per_s": 2 * N / (root_ms * 1e-3), "ms": root_ms,
                              "mfma_frac_paper_count": 2 * N * paper_products_root * flop_per_product
                              / (root_ms * 1e-3) / 1e12 / PEAK_FP32_MFMA_TFLOPS,
                              "note": "mfma_frac_paper_count prices every product of the paper's count in full; "
                                      "it is a throughput figure, not a utilisation"},
    }
    out["other_product_mode"] = other_mode
    out["inverse_root_power_iteration_scaling"] = pi_variant
    out["inverse_root_bf16x6"] = split_variants.get("bf16x6")
    out["inverse_root_fp16x3"] = split_variants.get("fp16x3")
    if not args.headline_only:
        del X, U
        torch.cuda.empty_cache()
        out["configs"] = other_configs(dash, cpu=not args.no_cpu_baseline)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(min(args.cpu_sample_blocks, N), B, beta, eps, p, args.cpu_repeats)
    log(f"step {ms_per_step:.2f} ms, {blocks_per_s:.0f} factor blocks/s, matmul kernel {achieved_tflops:.1f} TFLOP/s "
        f"({100 * roofline['frac']:.1f}% of fp32 MFMA peak)")
    print(json.dumps(out))


if __name__ == "__main__":
    main()
