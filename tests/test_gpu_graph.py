"""HIP graph capture of the library's call sequences: every entry point only launches kernels on the
context's stream, so a captured inverse root / step must replay to the bit-identical eager result, on
every replay, with eager work and synchronisations in between."""
import time

import numpy as np
import pytest

import workloads

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("precision", ["fp32", "fp16x3"])
def test_captured_inverse_root_and_step_replay_bit_identical(precision):
    import torch
    from paper_2602_02016_amd import Dash
    d = Dash(0)
    s = torch.cuda.Stream()
    N, B = workloads.CFG1["N"], workloads.CFG1["B"]
    A32, _, _ = workloads.spd_stack(N, B, -3.0, 0.0, seed=1000)
    A = torch.from_numpy(A32).cuda()
    X = torch.empty_like(A)
    G = torch.zeros(N, B, B, device="cuda")
    S = torch.zeros(2 * N, B, B, device="cuda"); XS = torch.zeros_like(S); U = torch.zeros_like(G)
    d.ensure_workspace(2 * N, B, "newton_db", 4, precision)          # sized before capture: nothing allocates inside
    torch.cuda.synchronize()
    d.set_stream(s)
    g_root, g_step = torch.cuda.CUDAGraph(), torch.cuda.CUDAGraph()
    with torch.cuda.graph(g_root, stream=s):
        d.inverse_root(A, X, method="newton_db", p=4, iters=10, eps=1e-6, precision=precision)
    with torch.cuda.graph(g_step, stream=s):
        d.step(G, S, XS, U, beta=0.95, eps=1e-6, method="newton_db", p=4, iters=10, precision=precision)
    torch.cuda.synchronize()
    d.set_stream(torch.cuda.current_stream())
    S_eager = torch.zeros_like(S); XS_eager = torch.zeros_like(S); U_eager = torch.zeros_like(G)
    for rep in range(4):
        # new inputs written in place by eager work, then replay, then the same call eagerly
        A_new, _, _ = workloads.spd_stack(N, B, -3.0, 0.0, seed=1100 + rep)
        A.copy_(torch.from_numpy(A_new).cuda())
        G.copy_(torch.from_numpy(workloads.gradient_stack(N, B, 1200 + rep)).cuda())
        torch.cuda.synchronize()
        g_root.replay()
        g_step.replay()
        torch.cuda.synchronize()
        X_replay, U_replay, S_replay = X.clone(), U.clone(), S.clone()
        X_e = d.inverse_root(A, method="newton_db", p=4, iters=10, eps=1e-6, precision=precision)
        d.step(G, S_eager, XS_eager, U_eager, beta=0.95, eps=1e-6, method="newton_db", p=4, iters=10, precision=precision)
        torch.cuda.synchronize()
        assert torch.equal(X_replay, X_e), rep
        assert torch.equal(S_replay, S_eager) and torch.equal(U_replay, U_eager), rep
        assert torch.isfinite(X_replay).all()
    # launch-bound small case: time per stack, eager against replay
    def timed(fn, n=20):
        fn(); torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / n * 1e6
    t_eager = timed(lambda: d.inverse_root(A, X, method="newton_db", p=4, iters=10, eps=1e-6, precision=precision))
    t_graph = timed(g_root.replay)
    print(f"cfg1 inverse root (N={N}, B={B}, p=4, k=10, {precision}): eager {t_eager:.0f} us, graph replay {t_graph:.0f} us", flush=True)
    d.close()
