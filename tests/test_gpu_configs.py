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


def fp32_floor(kappa: float, p: int, B: int = 256) -> float:
    """Rounding floor of fp32 Newton-DB (see tests/test_gpu_inverse_root.py): ~0.1 kappa 2^-24 at
    B = 256, growing like sqrt(B) with the length of the fp32 dot products, x2.5 for p = 2, x4 margin."""
    return 4.0 * max(1e-6, 0.1 * kappa * 2.0 ** -24) * max(1.0, (B / 256.0) ** 0.5) * (2.5 if p == 2 else 1.0)


# ---- config 2: one Shampoo step of a 4096 x 4096 layer, B = 1024 -----------------------------

def test_config2_full_step(dash):
    import torch
    c = workloads.CFG2
    N, B = workloads.cfg2_num_blocks(), c["B"]
    sample = [0, 5, 10, 15]
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
    print(f"cfg2: oracle step on blocks {sample} done ({time.time() - t0:.1f} s)", flush=True)
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
        print(f"cfg2 with {prec} operands: roots {eX:.2e} update {eU2:.2e}", flush=True)
        assert eX < 1e-4 and eU2 < 1e-4 and int(nf.sum().item()) == 0
        del X2, U2
    # properties that hold for every block, sampled or not: symmetric roots, finite update
    Xs = X.cpu().numpy()
    asym = np.sqrt(((Xs - np.swapaxes(Xs, 1, 2)) ** 2).sum(axis=(1, 2))) / np.sqrt((Xs ** 2).sum(axis=(1, 2)))
    assert asym.max() < 1e-5 and np.isfinite(U.cpu().numpy()).all()


# ---- config 3: 24-layer decoder stack, 3072 factor blocks -------------------------------------

def test_config3_full_stack(dash):
    """All 1536 gradient blocks / 3072 factor blocks (12 GiB of factors) in one step call,
    walked by the library in chunks of 512 blocks.  Four warm-up gradients instead of 20 bound
    the set-up time.  Sampled blocks get numpy-seeded gradients (shared generator) and are
    checked against the oracle; the others are filled on the device."""
    import torch
    c = workloads.CFG3
    N, B = workloads.cfg3_num_gradient_blocks(), c["B"]
    assert N == 1536
    sample = [0, 511, 512, 1000, 1535]
    warm = 4
    t0 = time.time()
    S = torch.zeros(2 * N, B, B, device="cuda")
    G = torch.empty(N, B, B, device="cuda")
    gen = torch.Generator(device="cuda")
    L64 = np.zeros((len(sample), B, B))
    R64 = np.zeros((len(sample), B, B))

    def make_gradient(t):
        gen.manual_seed(c["seed_base"] + 77 * t)
        torch.randn(G.shape, device="cuda", generator=gen, out=G)
        G.mul_(c["grad_std"])
        Gs = np.stack([workloads.gradient_stack(1, B, c["seed_base"] + 1000 * t + i, c["grad_std"])[0] for i in sample])
        G[torch.tensor(sample, device="cuda")] = _to_gpu(Gs)
        return Gs

    for t in range(warm):
        Gs = make_gradient(t)
        dash.accumulate_factors(G, S[:N], S[N:], c["beta"])
        L64, R64 = oshampoo.accumulate_factors(Gs, L64, R64, c["beta"])
    torch.cuda.synchronize()
    print(f"cfg3: 3072 factor blocks warmed with {warm} gradients ({time.time() - t0:.1f} s)", flush=True)
    Gs = make_gradient(warm)
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
    ref = oshampoo.step(Gs, L64, R64, beta=c["beta"], eps=c["eps"], p=c["p"])
    print(f"cfg3: oracle step on blocks {sample} done ({time.time() - t0:.1f} s)", flush=True)
    idx = torch.tensor(sample, device="cuda")
    eS = max(rel_frobenius_error(S[:N][idx].cpu().numpy(), ref["L"]).max(),
             rel_frobenius_error(S[N:][idx].cpu().numpy(), ref["R"]).max())
    eX = max(rel_frobenius_error(X[:N][idx].cpu().numpy(), ref["X_L"]).max(),
             rel_frobenius_error(X[N:][idx].cpu().numpy(), ref["X_R"]).max())
    eU = rel_frobenius_error(U[idx].cpu().numpy(), ref["U"]).max()
    print(f"cfg3: factors {eS:.2e} roots {eX:.2e} update {eU:.2e}", flush=True)
    assert eS < 1e-5 and eX < 1e-4 and eU < 1e-4
    assert int(nf.sum().item()) == 0
    assert bool(torch.isfinite(U).all())
    # every block: the root commutes with its factor up to rounding (X S = S X), checked on the device
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
        worst, worst_gpu, worst_mod = 0.0, 0.0, 0.0
        for j, (lam, Q, s) in enumerate(eig):
            X_evd = (Q * lam ** (-1.0 / p)) @ Q.T
            X_mod = (Q * model_scalar(lam, s)) @ Q.T
            e_gpu = rel_frobenius_error(Xh[j], X_evd)[0]
            e_mod = rel_frobenius_error(X_mod, X_evd)[0]
            e_same = rel_frobenius_error(Xh[j], X_mod)[0]
            worst, worst_gpu, worst_mod = max(worst, e_same), max(worst_gpu, e_gpu), max(worst_mod, e_mod)
            assert abs(e_gpu - e_mod) <= 0.1 * e_mod + floor, (label, e_gpu, e_mod)
        print(f"cfg4 B={B} {label}: err vs EVD {worst_gpu:.2e} (model {worst_mod:.2e}), vs model {worst:.2e}", flush=True)

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
            check(X, p, model, f"cheb p={p} d={d}", 2e-5)


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
    floor = fp32_floor(kappa, p, B)
    print("cfg5:  k | fp32 vs EVD | float64 model | bf16 vs EVD | bf16 blocks flagged non-finite | fp32 ms | bf16 ms")
    for k in c["iters"]:
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
        print(f"cfg5: {k:2d} | {max(e32):.3e} | {max(emod):.3e} | {np.nanmax(e16) if not np.all(np.isnan(e16)) else float('nan'):.3e} "
              f"| {flagged:4d} | {ms32:7.0f} | {ms16:7.0f} | bf16x6 vs EVD {max(e6):.3e} in {ms6:7.0f} ms "
              f"| fp16x3 vs EVD {max(e3):.3e} in {ms3:7.0f} ms", flush=True)
        for a_, m_ in zip(e32, emod):
            assert abs(a_ - m_) <= 0.1 * m_ + floor, (k, a_, m_, floor)
        for a_, m_ in zip(e6, emod):
            assert abs(a_ - m_) <= 0.1 * m_ + floor, ("bf16x6", k, a_, m_, floor)
