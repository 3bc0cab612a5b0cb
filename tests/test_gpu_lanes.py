"""Lanes: on stacks of small blocks dash_inverse_root sends the two halves of a chunk through the same launch
sequence on two streams (the context's and one of its own, forked and joined with events).  Blocks are independent,
so with every product computed in full the result must not change by a bit, whatever the method, precision, block
count (odd counts split unevenly) and chunking.  In symmetric mode the tile edge decides which entries of a mirrored
product are computed and which are copies, and the tile edge follows the launch size -- there (as with any change of
the stack length) the two agree to rounding.  The statistics count every launch once; the second stream is joined
when the call returns."""
import numpy as np
import pytest

import workloads

pytestmark = pytest.mark.gpu


@pytest.fixture()
def pair():
    from paper_2602_02016_amd import Dash
    on, off = Dash(0), Dash(0)
    off.set_lanes(False)
    on.set_symmetric(False); off.set_symmetric(False)          # every product in full: bit-exact comparisons
    yield on, off
    on.close(); off.close()


def _to_gpu(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


@pytest.mark.parametrize("method,iters", [("newton_db", 6), ("coupled_newton", 6), ("chebyshev", 12)])
@pytest.mark.parametrize("precision", ["fp32", "fp16x3", "bf16"])
@pytest.mark.parametrize("N,B", [(1037, 128), (257, 256), (65, 512)])
def test_lanes_do_not_change_a_bit(pair, method, iters, precision, N, B):
    import torch
    from paper_2602_02016_amd import chebyshev_fit
    on, off = pair
    A32, _, _ = workloads.spd_stack(N, B, -1.0, 0.0, seed=300 + B, share_q=True)
    A = _to_gpu(A32)
    kw = dict(method=method, p=4, iters=iters, eps=1e-6, precision=precision)
    if method == "chebyshev":
        kw.update(cheb_coeffs=chebyshev_fit(4, iters, 0.02, 1.0), cheb_a=0.02, cheb_b=1.0)
    nf_on = torch.ones(N, dtype=torch.int32, device="cuda")
    nf_off = torch.ones(N, dtype=torch.int32, device="cuda")
    on.reset_stats(); off.reset_stats()
    X_on = on.inverse_root(A, nonfinite_out=nf_on, **kw)
    X_off = off.inverse_root(A, nonfinite_out=nf_off, **kw)
    torch.cuda.synchronize()
    assert torch.equal(X_on, X_off)
    assert torch.equal(nf_on, nf_off) and int(nf_on.sum().item()) == 0
    s_on, s_off = on.get_stats(), off.get_stats()
    assert s_on["matmul_products"] == s_off["matmul_products"] and s_on["matmul_launches"] == s_off["matmul_launches"]
    assert s_on["matmul_block_products"] == s_off["matmul_block_products"]
    if precision != "bf16":         # symmetric mode: the same roots to rounding (plain bf16 amplifies any difference)
        on.set_symmetric(True); off.set_symmetric(True)
        try:
            Xs_on, Xs_off = on.inverse_root(A, **kw), off.inverse_root(A, **kw)
            torch.cuda.synchronize()
        finally:
            on.set_symmetric(False); off.set_symmetric(False)
        rel = (Xs_on - Xs_off).double().flatten(1).norm(dim=1) / Xs_off.double().flatten(1).norm(dim=1)
        assert float(rel.max()) < 1e-5


def test_lanes_with_chunks_and_following_work(pair):
    """A workspace that holds 1100 of 2500 blocks of 128: chunks of 1100, 1100 and 300 (the last one below the lane
    threshold), each forked and joined on its own; work enqueued on the context's stream right after the call must
    see the finished roots of every lane."""
    import torch
    on, off = pair
    N, B = 2500, 128
    A = _to_gpu(workloads.spd_stack(4, B, -1.0, 0.0, seed=311, share_q=True)[0]).repeat(N // 4, 1, 1).contiguous()
    A += 0.01 * torch.rand(N, 1, 1, device="cuda") * torch.eye(B, device="cuda")
    cap = on.workspace_bytes(1100, B)
    X_on = on.inverse_root(A, p=4, iters=8, eps=1e-6, workspace_max_bytes=cap)
    total_on = X_on.sum(dim=(1, 2))                       # torch work on the same (current) stream, no synchronisation
    X_off = off.inverse_root(A, p=4, iters=8, eps=1e-6, workspace_max_bytes=cap)
    total_off = X_off.sum(dim=(1, 2))
    torch.cuda.synchronize()
    assert torch.equal(X_on, X_off) and torch.equal(total_on, total_off)


def test_lanes_inside_a_captured_graph():
    """The second stream joins a stream capture at the fork and leaves it at the join: a captured inverse root on 256
    blocks of 256 replays to the eager result, several times, with eager work in between."""
    import torch
    from paper_2602_02016_amd import Dash
    d = Dash(0)
    s = torch.cuda.Stream()
    N, B = 256, 256
    A32, _, _ = workloads.spd_stack(N, B, -2.0, 0.0, seed=321, share_q=True)
    A = _to_gpu(A32)
    X = torch.empty_like(A)
    d.ensure_workspace(N, B, "newton_db", 4, "fp32")
    torch.cuda.synchronize()
    d.set_stream(s)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=s):
        d.inverse_root(A, X, p=4, iters=10, eps=1e-6)
    torch.cuda.synchronize()
    d.set_stream(torch.cuda.current_stream())
    for rep in range(3):
        A_new, _, _ = workloads.spd_stack(N, B, -2.0, 0.0, seed=330 + rep, share_q=True)
        A.copy_(_to_gpu(A_new))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        X_replay = X.clone()
        X_eager = d.inverse_root(A, p=4, iters=10, eps=1e-6)
        torch.cuda.synchronize()
        assert torch.equal(X_replay, X_eager), rep
    d.close()
