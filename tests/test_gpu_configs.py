"""The five benchmark configurations at their full sizes, in the launch configuration the
benchmark uses, checked on sampled blocks the float64 oracle computes one by one (blocks
are independent through the whole path, so a block's oracle needs only that block's inputs)."""
import time

import numpy as np
import pytest

import workloads
from oracle import chebyshev as ocheb
from oracle import newton_db as ondb
from oracle import shampoo as oshampoo
from oracle.evd import inverse_root_evd, rel_frobenius_error
from tolerances import SYMMETRIC_OVER_FULL_ILLCONDITIONED, clenshaw_fp32_floor, fp32_floor, fp32_floor_typical, max_abs_bar, rel_max_abs_error

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


# ---- config 2: one Shampoo step of a 4096 x 4096 layer, B = 1024 -----------------------------

def test_config2_full_step(dash):
    import torch
    c = workloads.CFG2
    N, B = workloads.cfg2_num_blocks(), c["B"]
    sample = list(range(N))             # all 16 gradient blocks: 32 factors, 32 roots, 16 updates
    S = torch.zeros(2 * N, B, B, device="cuda")
    L64 = np.zeros((len(sample), B, B))
    R64 = np.zeros((len(sample), B, B))
    t0 = time.time()
    for t in range(c["warm_steps"]):
        G = workloads.gradient_stack(N, B, c["seed_base"] + t, c["grad_std"])
        dash.accumulate_factors(_to_gpu(G), S[:N], S[N:], c["beta"])
        L64, R64 = oshampoo.accumulate_factors(G[sample], L64, R64, c["beta"])
    print(f"cfg2: factors warmed with {c['warm_steps']} gradients ({time.time() - t0:.1f} s)", flush=True)
    G = workloads.gradient_stack(N, B, c["seed_base"] + c["warm_steps"], c["grad_std"])
    X = torch.empty_like(S)
    U = torch.empty(N, B, B, device="cuda")
    nf = torch.ones(2 * N, dtype=torch.int32, device="cuda")
    dash.step(_to_gpu(G), S, X, U, beta=c["beta"], eps=c["eps"], p=c["p"], iters=c["ndb_iters"], nonfinite_out=nf)
    torch.cuda.synchronize()
    ref = oshampoo.step(G[sample], L64, R64, beta=c["beta"], eps=c["eps"], p=c["p"])
    print(f"cfg2: oracle step on all {len(sample)} gradient blocks done ({time.time() - t0:.1f} s)", flush=True)
    idx = torch.tensor(sample, device="cuda")
    eL = rel_frobenius_error(S[:N][idx].cpu().numpy(), ref["L"]).max()
    eR = rel_frobenius_error(S[N:][idx].cpu().numpy(), ref["R"]).max()
    eXL = rel_frobenius_error(X[:N][idx].cpu().numpy(), ref["X_L"]).max()
    eXR = rel_frobenius_error(X[N:][idx].cpu().numpy(), ref["X_R"]).max()
    eU = rel_frobenius_error(U[idx].cpu().numpy(), ref["U"]).max()
    lam = np.linalg.eigvalsh(ref["L"][0])
    print(f"cfg2: factors {max(eL, eR):.2e} roots {max(eXL, eXR):.2e} update {eU:.2e}; kappa(L_0) = "
          f"{lam.max() / lam.min():.2f}, lambda/||L||_F in [{lam.min() / np.linalg.norm(ref['L'][0]):.3f}, "
          f"{lam.max() / np.linalg.norm(ref['L'][0]):.3f}]", flush=True)
    assert max(eL, eR) < 1e-5
    assert max(eXL, eXR) < 1e-4
    assert eU < 1e-4
    assert int(nf.sum().item()) == 0
    # element by element, scaled by the largest entry of the reference block
    mS = max(rel_max_abs_error(S[:N][idx].cpu().numpy(), ref["L"]).max(), rel_max_abs_error(S[N:][idx].cpu().numpy(), ref["R"]).max())
    mX = max(rel_max_abs_error(X[:N][idx].cpu().numpy(), ref["X_L"]).max(), rel_max_abs_error(X[N:][idx].cpu().numpy(), ref["X_R"]).max())
    mU = rel_max_abs_error(U[idx].cpu().numpy(), ref["U"]).max()
    print(f"cfg2: largest element-wise deviation / max|ref|: factors {mS:.2e} roots {mX:.2e} update {mU:.2e}", flush=True)
    assert mS < max_abs_bar(1e-5) and mX < max_abs_bar(1e-4) and mU < max_abs_bar(1e-4)
    # the same roots with split 16-bit operands, to the same bar
    for prec in ("fp16x3", "bf16x6"):
        X2 = torch.empty_like(S)
        dash.inverse_root(S, X2, p=c["p"], iters=c["ndb_iters"], eps=c["eps"], precision=prec, nonfinite_out=nf)
        U2 = torch.empty_like(U)
        dash.precondition(X2[:N], _to_gpu(G), X2[N:], U2)
        torch.cuda.synchronize()
        eX = max(rel_frobenius_error(X2[:N][idx].cpu().numpy(), ref["X_L"]).max(),
                 rel_frobenius_error(X2[N:][idx].cpu().numpy(), ref["X_R"]).max())
        eU2 = rel_frobenius_error(U2[idx].cpu().numpy(), ref["U"]).max()
        mX2 = max(rel_max_abs_error(X2[:N][idx].cpu().numpy(), ref["X_L"]).max(),
                  rel_max_abs_error(X2[N:][idx].cpu().numpy(), ref["X_R"]).max())
        print(f"cfg2 with {prec} operands: roots {eX:.2e} (element-wise {mX2:.2e}) update {eU2:.2e}", flush=True)
        assert eX < 1e-4 and eU2 < 1e-4 and mX2 < max_abs_bar(1e-4) and int(nf.sum().item()) == 0
        del X2, U2
    # properties that hold for every block, sampled or not: symmetric roots, finite update
    Xs = X.cpu().numpy()
    asym = np.sqrt(((Xs - np.swapaxes(Xs, 1, 2)) ** 2).sum(axis=(1, 2))) / np.sqrt((Xs ** 2).sum(axis=(1, 2)))
    assert asym.max() < 1e-5 and np.isfinite(U.cpu().numpy()).all()


# ---- config 3: 24-layer decoder stack, 3072 factor blocks -------------------------------------

CFG3_SAMPLE_SIZE = 256        # gradient blocks compared with the float64 oracle (512 of the 3072 factor blocks)
CFG3_SAMPLE_SEED = 20260203


def cfg3_sample(N):
    """First and last gradient block of each third of the stack -- they own the first and last factor block of all
    six 512-block chunks the library walks ([L; R] with L = factors 0..1535, R = 1536..3071) -- plus seeded random
    others, CFG3_SAMPLE_SIZE in all."""
    must = [0, 511, 512, 1023, 1024, N - 1]
    rng = np.random.default_rng(CFG3_SAMPLE_SEED)
    rest = [int(i) for i in rng.permutation(N) if int(i) not in must][:CFG3_SAMPLE_SIZE - len(must)]
    return sorted(must + rest)


def test_config3_full_stack(dash, tmp_path):
    """All 1536 gradient blocks / 3072 factor blocks (12 GiB of factors) in one step call, walked by the library
    in chunks of 512 blocks.  Four warm-up gradients instead of 20 bound the set-up time.  Gradients are drawn on
    the device (seeded); 256 seeded gradient blocks -- their 512 factors, 512 roots and 256 updates -- are compared
    with the float64 oracle, which runs in worker processes on exactly the fp32 gradients the GPU received."""
    import multiprocessing as mp
    import os
    from concurrent.futures import ProcessPoolExecutor, as_completed
    import torch
    import block_oracle_worker
    c = workloads.CFG3
    N, B = workloads.cfg3_num_gradient_blocks(), c["B"]
    assert N == 1536
    sample = cfg3_sample(N)
    assert len(sample) == CFG3_SAMPLE_SIZE and len(set(sample)) == CFG3_SAMPLE_SIZE
    idx = torch.tensor(sample, device="cuda")
    warm = 4
    t0 = time.time()
    S = torch.zeros(2 * N, B, B, device="cuda")
    G = torch.empty(N, B, B, device="cuda")
    gen = torch.Generator(device="cuda")

    def save(name, t):
        np.save(os.path.join(tmp_path, name + ".npy"), t.cpu().numpy())

    def make_gradient(t):
        gen.manual_seed(c["seed_base"] + 77 * t)
        torch.randn(G.shape, device="cuda", generator=gen, out=G)
        G.mul_(c["grad_std"])
        save(f"G_{t}", G[idx])

    for t in range(warm):
        make_gradient(t)
        dash.accumulate_factors(G, S[:N], S[N:], c["beta"])
    torch.cuda.synchronize()
    print(f"cfg3: 3072 factor blocks warmed with {warm} gradients ({time.time() - t0:.1f} s)", flush=True)
    make_gradient(warm)
    X = torch.empty_like(S)
    U = torch.empty_like(G)
    nf = torch.ones(2 * N, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    t1 = time.time()
    dash.step(G, S, X, U, beta=c["beta"], eps=c["eps"], p=c["p"], iters=c["ndb_iters"], nonfinite_out=nf,
              workspace_max_bytes=dash.workspace_bytes(512, B))
    torch.cuda.synchronize()
    dt = time.time() - t1
    flop = (2 * N * 2 * (3 * c["ndb_iters"] - 3) + 4 * N) * 2.0 * B ** 3
    print(f"cfg3: step over 3072 factor blocks {dt * 1e3:.0f} ms = {2 * N / dt:.0f} blocks/s, "
          f"{flop / dt / 1e12:.1f} TFLOP/s full-product equivalent (symmetric mode computes fewer tiles)", flush=True)
    for name, t in (("gpu_L", S[:N][idx]), ("gpu_R", S[N:][idx]), ("gpu_XL", X[:N][idx]), ("gpu_XR", X[N:][idx]),
                    ("gpu_U", U[idx])):
        save(name, t)
    print(f"cfg3: inputs and results of the {len(sample)} sampled gradient blocks written for the oracle "
          f"({time.time() - t0:.1f} s)", flush=True)
    workers = max(1, min(16, os.cpu_count() or 1))
    jobs = [(str(tmp_path), j, warm + 1, c["beta"], c["eps"], c["p"]) for j in range(len(sample))]
    worst = {k: [0.0, 0.0] for k in ("L", "R", "XL", "XR", "U")}
    done = 0
    # a worker that dies breaks the pool with an exception here (it is never silently restarted)
    with ProcessPoolExecutor(max_workers=workers, mp_context=mp.get_context("spawn")) as pool:
        for fut in as_completed([pool.submit(block_oracle_worker.check_block, job) for job in jobs]):
            j, errs = fut.result()
            for k, (ef, em) in errs.items():
                worst[k][0] = max(worst[k][0], ef)
                worst[k][1] = max(worst[k][1], em)
            done += 1
            if done % 32 == 0:
                print(f"cfg3: oracle step of {done}/{len(sample)} sampled blocks done ({time.time() - t0:.1f} s)", flush=True)
    eS, mS = max(worst["L"][0], worst["R"][0]), max(worst["L"][1], worst["R"][1])
    eX, mX = max(worst["XL"][0], worst["XR"][0]), max(worst["XL"][1], worst["XR"][1])
    eU, mU = worst["U"]
    print(f"cfg3: {len(sample)} gradient blocks (sample seed {CFG3_SAMPLE_SEED}) on {workers} oracle workers: factors {eS:.2e} "
          f"roots {eX:.2e} update {eU:.2e}; element-wise {mS:.2e} {mX:.2e} {mU:.2e}", flush=True)
    assert eS < 1e-5 and eX < 1e-4 and eU < 1e-4
    assert mS < max_abs_bar(1e-5) and mX < max_abs_bar(1e-4) and mU < max_abs_bar(1e-4)
    assert int(nf.sum().item()) == 0
    assert bool(torch.isfinite(U).all())
    # every block, sampled or not: the root commutes with its factor up to rounding (X S = S X), on the device
    for lo in range(0, 2 * N, 768):
        Sc, Xc = S[lo:lo + 768], X[lo:lo + 768]
        comm = torch.linalg.matrix_norm(Xc @ Sc - Sc @ Xc) / (torch.linalg.matrix_norm(Xc) * torch.linalg.matrix_norm(Sc))
        assert float(comm.max()) < 1e-5


# ---- config 4: block-size and method sweep ----------------------------------------------------

@pytest.mark.parametrize("B,N,nsample", [(256, 256, 6), (512, 64, 3), (2048, 4, 1)])
def test_config4_sweep(dash, B, N, nsample):
    """N * B^2 = 2^24.  Newton-DB k in {5,10,20}, Chebyshev d in {8,16,32}, p in {2,4}, spectra
    log-uniform in [1e-4, 1].  For each run the distance of the GPU result to the EVD root must
    equal the method's own truncation error (from the float64 spectral model) up to the fp32 floor."""
    from paper_2602_02016_amd import chebyshev_fit
    c = workloads.CFG4
    t0 = time.time()
    A32, _, lam_true = workloads.spd_stack(N, B, c["lo_exp"], c["hi_exp"], c["seed"] + B, share_q=True)
    print(f"cfg4 B={B} N={N}: inputs built ({time.time() - t0:.1f} s)", flush=True)
    A = _to_gpu(A32)
    sample = list(range(0, N, max(1, N // nsample)))[:nsample]
    eig = []
    for i in sample:
        Ai = A32[i].astype(np.float64)
        lam, Q = np.linalg.eigh(0.5 * (Ai + Ai.T))
        eig.append((lam, Q, float(np.sqrt((Ai ** 2).sum()))))
    print(f"cfg4 B={B}: eigendecomposition of blocks {sample} done ({time.time() - t0:.1f} s)", flush=True)
    s_all = np.sqrt((A32.astype(np.float64) ** 2).sum(axis=(1, 2)))
    a_lo = float((lam_true.min(axis=1) / s_all).min()) * 0.99

    def check(X, p, model_scalar, label, floor):
        Xh = np.stack([X[i].cpu().numpy() for i in sample])
        worst, worst_gpu, worst_mod, worst_abs = 0.0, 0.0, 0.0, 0.0
        for j, (lam, Q, s) in enumerate(eig):
            X_evd = (Q * lam ** (-1.0 / p)) @ Q.T
            X_mod = (Q * model_scalar(lam, s)) @ Q.T
            e_gpu = rel_frobenius_error(Xh[j], X_evd)[0]
            e_mod = rel_frobenius_error(X_mod, X_evd)[0]
            e_same = rel_frobenius_error(Xh[j], X_mod)[0]
            m_same = rel_max_abs_error(Xh[j], X_mod)[0]
            worst, worst_gpu, worst_mod = max(worst, e_same), max(worst_gpu, e_gpu), max(worst_mod, e_mod)
            worst_abs = max(worst_abs, m_same)
            assert abs(e_gpu - e_mod) <= 0.1 * e_mod + floor, (label, e_gpu, e_mod)
            # against the float64 model of the same iteration count (same truncation, so only rounding differs),
            # in norm and element by element: the rounding floor
            assert e_same <= floor and m_same <= max_abs_bar(floor), (label, e_same, m_same, floor)
        print(f"cfg4 B={B} {label}: err vs EVD {worst_gpu:.2e} (model {worst_mod:.2e}), vs model {worst:.2e}, "
              f"element-wise vs model {worst_abs:.2e} (bars {floor:.2e}, {max_abs_bar(floor):.2e})", flush=True)

    for p in c["ps"]:
        for k in c["ndb_iters"]:
            X = dash.inverse_root(A, p=p, iters=k)

            def model(lam, s, p=p, k=k):
                y, z = ondb.ndb_scalar(lam / s, k)
                if p == 4:
                    _, z = ondb.ndb_scalar(y, k)
                return z * s ** (-1.0 / p)
            check(X, p, model, f"ndb p={p} k={k}", fp32_floor(1e4, p, B))
        for d in c["cheb_degrees"]:
            coef = chebyshev_fit(p, d, a_lo, 1.0)
            X = dash.inverse_root(A, method="chebyshev", p=p, iters=d, cheb_coeffs=coef, cheb_a=a_lo, cheb_b=1.0)

            def model(lam, s, p=p, coef=coef):
                return ocheb.clenshaw_scalar(ocheb.to_unit_interval(lam / s, a_lo, 1.0), np.array(coef)) * s ** (-1.0 / p)
            check(X, p, model, f"cheb p={p} d={d}", clenshaw_fp32_floor(d, p, B))


# ---- config 5: ill-conditioned stack, fp32 against bf16 operands -------------------------------

def test_config5_illconditioned_table(dash):
    """1024 blocks of 1024 x 1024, spectra log-uniform in [1e-8, 1], eps = 1e-6.  Error against
    the EVD root versus iteration count for fp32 and for bf16 operands; fp32 must follow the
    float64 model of the method, bf16 is reported (non-finite blocks must be flagged)."""
    import torch
    c = workloads.CFG5
    N, B, p, eps = c["N"], c["B"], c["p"], c["eps"]
    t0 = time.time()
    A32, _, _ = workloads.spd_stack(N, B, c["lo_exp"], c["hi_exp"], c["seed"], share_q=True)
    print(f"cfg5: {N} blocks built ({time.time() - t0:.1f} s)", flush=True)
    A = _to_gpu(A32)
    sample = [0, 341, 1023]
    eig = []
    for i in sample:
        Ad = A32[i].astype(np.float64) + eps * np.eye(B)
        lam, Q = np.linalg.eigh(0.5 * (Ad + Ad.T))
        eig.append((lam, Q, float(np.sqrt((Ad ** 2).sum()))))
    kappa = max(l.max() / l.min() for l, _, _ in eig)
    print(f"cfg5: eigendecomposition of blocks {sample} done, kappa = {kappa:.2e} ({time.time() - t0:.1f} s)", flush=True)
    X = torch.empty_like(A)
    nf = torch.zeros(N, dtype=torch.int32, device="cuda")
    ws_cap = dash.workspace_bytes(256, B)
    # the bar of fp32 with every product computed in full, and the typical floor behind it, both derived on the
    # CPU (tests/test_fp32_floor.py).  Symmetric mode (the library's default, mirrored residual product) about
    # doubles the floor on these spectra: it is held to a stated multiple of what full products reach.
    floor = fp32_floor(kappa, p, B, symmetric=False)
    typ = fp32_floor_typical(kappa, p, B)
    print(f"cfg5: fp32 floor law {typ:.2e}, full-products bar {floor:.2e}, symmetric mode within "
          f"{SYMMETRIC_OVER_FULL_ILLCONDITIONED} x the full-products excess over the model", flush=True)
    print("cfg5:  k | fp32 vs EVD (symmetric mode) | fp32 vs EVD (full products) | float64 model | bf16 vs EVD | "
          "bf16 blocks flagged non-finite | fp32 ms | bf16 ms")
    for k in c["iters"]:
        dash.set_symmetric(False)
        try:
            dash.inverse_root(A, X, p=p, iters=k, eps=eps, nonfinite_out=nf, workspace_max_bytes=ws_cap)
        finally:
            dash.set_symmetric(True)
        assert int(nf.sum().item()) == 0
        e32_full = [rel_frobenius_error(X[sample[j]].cpu().numpy(), (Q * lam ** (-1.0 / p)) @ Q.T)[0]
                    for j, (lam, Q, s) in enumerate(eig)]
        torch.cuda.synchronize(); t1 = time.time()
        dash.inverse_root(A, X, p=p, iters=k, eps=eps, nonfinite_out=nf, workspace_max_bytes=ws_cap)
        torch.cuda.synchronize(); ms32 = (time.time() - t1) * 1e3
        assert int(nf.sum().item()) == 0
        e32, emod = [], []
        for j, (lam, Q, s) in enumerate(eig):
            X_evd = (Q * lam ** (-1.0 / p)) @ Q.T
            y, z = ondb.ndb_scalar(lam / s, k)
            _, z = ondb.ndb_scalar(y, k)
            X_mod = (Q * (z * s ** (-1.0 / p))) @ Q.T
            e32.append(rel_frobenius_error(X[sample[j]].cpu().numpy(), X_evd)[0])
            emod.append(rel_frobenius_error(X_mod, X_evd)[0])
        torch.cuda.synchronize(); t1 = time.time()
        dash.inverse_root(A, X, p=p, iters=k, eps=eps, precision="bf16", nonfinite_out=nf, workspace_max_bytes=ws_cap)
        torch.cuda.synchronize(); ms16 = (time.time() - t1) * 1e3
        flagged = int(nf.sum().item())
        e16 = []
        for j, (lam, Q, s) in enumerate(eig):
            Xj = X[sample[j]].cpu().numpy()
            assert bool(nf[sample[j]].item()) == (not np.isfinite(Xj).all())
            e16.append(rel_frobenius_error(Xj, (Q * lam ** (-1.0 / p)) @ Q.T)[0] if np.isfinite(Xj).all() else float("nan"))
        # three-plane split bf16 operands: the same bar as fp32
        torch.cuda.synchronize(); t1 = time.time()
        dash.inverse_root(A, X, p=p, iters=k, eps=eps, precision="bf16x6", nonfinite_out=nf, workspace_max_bytes=ws_cap)
        torch.cuda.synchronize(); ms6 = (time.time() - t1) * 1e3
        assert int(nf.sum().item()) == 0
        e6 = [rel_frobenius_error(X[sample[j]].cpu().numpy(), (Q * lam ** (-1.0 / p)) @ Q.T)[0]
              for j, (lam, Q, s) in enumerate(eig)]
        # two fp16 planes with a scaled low plane: reported, and held to three times the fp32 path's error
        torch.cuda.synchronize(); t1 = time.time()
        dash.inverse_root(A, X, p=p, iters=k, eps=eps, precision="fp16x3", nonfinite_out=nf, workspace_max_bytes=ws_cap)
        torch.cuda.synchronize(); ms3 = (time.time() - t1) * 1e3
        assert int(nf.sum().item()) == 0
        e3 = [rel_frobenius_error(X[sample[j]].cpu().numpy(), (Q * lam ** (-1.0 / p)) @ Q.T)[0]
              for j, (lam, Q, s) in enumerate(eig)]
        assert max(e3) <= 3 * max(e32) + floor, ("fp16x3", k, e3, e32)
        print(f"cfg5: {k:2d} | {max(e32):.3e} | {max(e32_full):.3e} | {max(emod):.3e} | {np.nanmax(e16) if not np.all(np.isnan(e16)) else float('nan'):.3e} "
              f"| {flagged:4d} | {ms32:7.0f} | {ms16:7.0f} | bf16x6 vs EVD {max(e6):.3e} in {ms6:7.0f} ms "
              f"| fp16x3 vs EVD {max(e3):.3e} in {ms3:7.0f} ms", flush=True)
        for a_, f_, m_ in zip(e32, e32_full, emod):
            assert abs(f_ - m_) <= 0.1 * m_ + floor, ("full products", k, f_, m_, floor)
            assert abs(a_ - m_) <= 0.1 * m_ + SYMMETRIC_OVER_FULL_ILLCONDITIONED * max(abs(f_ - m_), typ), \
                ("symmetric mode", k, a_, f_, m_, typ)
        for a_, m_ in zip(e6, emod):
            assert abs(a_ - m_) <= 0.1 * m_ + floor, ("bf16x6", k, a_, m_, floor)
