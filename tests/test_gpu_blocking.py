"""block()/unblock, ragged (rectangular) gradient blocks and 1-D parameters (paper Section 4.1)
through the C ABI against the float64 oracle."""
import numpy as np
import pytest

from oracle import blocking as oblocking
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


def _layer(m, n, seed, std=1e-2):
    return (np.random.default_rng(seed).standard_normal((m, n)) * std).astype(np.float32)


@pytest.mark.parametrize("m,n,B", [(500, 32, 16), (320, 256, 128), (256, 320, 128), (333, 205, 64), (7, 5, 2),
                                   (40, 300, 64), (300, 40, 64), (128, 128, 128), (1000, 2048, 256)])
def test_block_unblock_bit_exact(dash, m, n, B):
    import torch
    print(f"block m={m} n={n} B={B}", flush=True)
    W = np.arange(m * n, dtype=np.float32).reshape(m, n) * 0.5 + 1.0
    ref = oblocking.block_layer(W, B)
    got = dash.block_layer(_to_gpu(W), B)
    for k, v in ref.items():
        if v.size == 0:
            assert got[k] is None
        else:
            assert got[k].shape == v.shape and np.array_equal(got[k].cpu().numpy(), v), k
    W2 = torch.full((m, n), -1.0, device="cuda")
    dash.unblock_layer(W2, B, got)
    assert np.array_equal(W2.cpu().numpy(), W)


@pytest.mark.parametrize("m,n,B,pm,pn", [(300, 250, 128, 64, 64), (333, 205, 64, 16, 32), (131, 257, 128, 64, 64),
                                         (1, 190, 128, 1, 64), (1000, 2048, 256, 64, 64), (77, 61, 64, 64, 64)])
def test_block_unblock_padded(dash, m, n, B, pm, pn):
    """Padded blocking: the rest extents are rounded up inside the stacks, the real entries are where the
    unpadded blocking puts them, the padding is zero, and unblocking ignores it."""
    import torch
    print(f"padded block m={m} n={n} B={B} pad=({pm},{pn})", flush=True)
    W = np.arange(m * n, dtype=np.float32).reshape(m, n) * 0.5 + 1.0
    ref = oblocking.block_layer(W, B)
    got = dash.block_layer(_to_gpu(W), B, pm, pn)
    for k, v in ref.items():
        if v.size == 0:
            assert got[k] is None
            continue
        g = got[k].cpu().numpy()
        assert g.shape[0] == v.shape[0] and g.shape[1] % (pm if k != "col_rest" else 1) == 0 and g.shape[1] >= v.shape[1]
        assert g.shape[2] >= v.shape[2] and g.shape[2] - v.shape[2] < pn
        assert np.array_equal(g[:, :v.shape[1], :v.shape[2]], v), k
        pad = g.copy(); pad[:, :v.shape[1], :v.shape[2]] = 0.0
        assert not pad.any(), k
        got[k][:, v.shape[1]:, :] = 3.0                 # poison the padding: unblocking must not look at it
        got[k][:, :, v.shape[2]:] = 3.0
    W2 = torch.full((m, n), -1.0, device="cuda")
    dash.unblock_layer(W2, B, got, pm, pn)
    assert np.array_equal(W2.cpu().numpy(), W)


def test_apply_update_any_length(dash):
    import torch
    for n in (1, 3, 4, 5, 1023, 4099, 77 * 61):
        rng = np.random.default_rng(n)
        t, u = rng.standard_normal(n).astype(np.float32), rng.standard_normal(n).astype(np.float32)
        tg = torch.from_numpy(t).cuda()
        dash.apply_update(tg, torch.from_numpy(u).cuda(), 0.25)
        assert np.array_equal(tg.cpu().numpy(), t - np.float32(0.25) * u), n


def test_block_empty_layer(dash):
    import torch
    got = dash.block_layer(torch.zeros(0, 64, device="cuda"), 64)
    assert all(v is None for v in got.values())


@pytest.mark.parametrize("sym", [True, False])
@pytest.mark.parametrize("N,Bm,Bn", [(2, 256, 1024), (3, 64, 192), (5, 128, 64), (1, 1024, 256), (40, 128, 256)])
def test_rect_accumulate_and_precondition(dash, N, Bm, Bn, sym):
    import torch
    print(f"rect N={N} Bm={Bm} Bn={Bn} sym={sym}", flush=True)
    dash.set_symmetric(sym)
    try:
        rng = np.random.default_rng(1000 + Bm + Bn)
        L = torch.zeros(N, Bm, Bm, device="cuda"); R = torch.zeros(N, Bn, Bn, device="cuda")
        L64, R64 = np.zeros((N, Bm, Bm)), np.zeros((N, Bn, Bn))
        for t in range(3):
            G = (rng.standard_normal((N, Bm, Bn)) * 1e-2).astype(np.float32)
            dash.accumulate_factors_rect(_to_gpu(G), L, R, 0.9)
            L64, R64 = oshampoo.accumulate_factors(G, L64, R64, float(np.float32(0.9)), float(np.float32(1.0) - np.float32(0.9)))
        assert rel_frobenius_error(L.cpu().numpy(), L64).max() < 2e-6
        assert rel_frobenius_error(R.cpu().numpy(), R64).max() < 2e-6
        Lg, Rg = L.cpu().numpy(), R.cpu().numpy()
        assert np.array_equal(Lg, np.swapaxes(Lg, 1, 2)) or not sym     # mirrored: exactly symmetric
        # precondition with arbitrary (non-symmetric) left and right matrices
        Xl = rng.standard_normal((N, Bm, Bm)).astype(np.float32); Xr = rng.standard_normal((N, Bn, Bn)).astype(np.float32)
        U = dash.precondition_rect(_to_gpu(Xl), _to_gpu(G), _to_gpu(Xr)).cpu().numpy()
        assert rel_frobenius_error(U, oshampoo.precondition(Xl, G, Xr)).max() < 2e-6
    finally:
        dash.set_symmetric(True)


def test_rect_chunked_workspace_and_errors(dash):
    import torch
    from paper_2602_02016_amd import DashError
    N, Bm, Bn = 6, 64, 128
    rng = np.random.default_rng(77)
    G = rng.standard_normal((N, Bm, Bn)).astype(np.float32)
    Xl = rng.standard_normal((N, Bm, Bm)).astype(np.float32); Xr = rng.standard_normal((N, Bn, Bn)).astype(np.float32)
    ref = oshampoo.precondition(Xl, G, Xr)
    U = torch.zeros(N, Bm, Bn, device="cuda")
    dash.set_workspace_bytes(2 * Bm * Bn * 4)        # room for two blocks: three chunks
    import ctypes as C
    dXl, dG, dXr = _to_gpu(Xl), _to_gpu(G), _to_gpu(Xr)
    st = dash.lib.dash_precondition_rect(dash.h, C.c_void_p(dXl.data_ptr()), C.c_void_p(dG.data_ptr()),
                                         C.c_void_p(dXr.data_ptr()), C.c_void_p(U.data_ptr()), N, Bm, Bn)
    assert st == 0
    dash.reset_stats()
    assert rel_frobenius_error(U.cpu().numpy(), ref).max() < 2e-6
    with pytest.raises(DashError):
        dash.accumulate_factors_rect(torch.zeros(1, 100, 64, device="cuda"), torch.zeros(1, 100, 100, device="cuda"),
                                     torch.zeros(1, 64, 64, device="cuda"), 0.9)
    z = torch.zeros(0, 64, 128, device="cuda")
    dash.accumulate_factors_rect(z, torch.zeros(0, 64, 64, device="cuda"), torch.zeros(0, 128, 128, device="cuda"), 0.9)


@pytest.mark.parametrize("N,B", [(1, 64), (6, 256), (8, 1024), (3, 192)])
def test_vector_accumulate_and_precondition(dash, N, B):
    import torch
    print(f"vector N={N} B={B}", flush=True)
    rng = np.random.default_rng(B + N)
    L = torch.zeros(N, B, B, device="cuda")
    L64 = np.zeros((N, B, B))
    b32 = float(np.float32(0.95)); a32 = float(np.float32(1.0) - np.float32(0.95))
    for t in range(3):
        g = rng.standard_normal((N, B)).astype(np.float32)
        dash.accumulate_vector(_to_gpu(g), L, 0.95)
        L64 = oblocking.accumulate_vector(g, L64, b32, a32)
    assert rel_frobenius_error(L.cpu().numpy(), L64).max() < 1e-6
    X = rng.standard_normal((N, B, B)).astype(np.float32)
    u = dash.precondition_vector(_to_gpu(X), _to_gpu(g)).cpu().numpy()
    ref = oblocking.precondition_vector(X, g)
    assert np.abs(u - ref).max() <= 2e-6 * np.sqrt((X.astype(np.float64) ** 2).sum(-1)).max() * np.sqrt((g.astype(np.float64) ** 2).sum(-1)).max()


def test_norm_layers_step(dash):
    """N normalisation layers of size E: accumulate, inverse square root (Newton-DB, p = 2), u = L^(-1/2) g."""
    import torch
    N, E, B = 5, 512, 256
    rng = np.random.default_rng(31)
    nb = N * E // B
    L = torch.zeros(nb, B, B, device="cuda")
    L64 = np.zeros((nb, B, B))
    b32 = float(np.float32(0.9)); a32 = float(np.float32(1.0) - np.float32(0.9))
    eps = 1e-3
    for t in range(4):
        grads = rng.standard_normal((N, E)).astype(np.float32)
        g = _to_gpu(grads).view(nb, B)
        dash.accumulate_vector(g, L, 0.9)
        if t < 3:
            _, L64 = oblocking.norm_layers_step(grads, L64, B, b32, eps, a32)
    U_ref, L64 = oblocking.norm_layers_step(grads, L64, B, b32, eps, a32)
    X = dash.inverse_root(L, method="newton_db", p=2, iters=25, eps=eps)
    u = dash.precondition_vector(X, g).view(N, E).cpu().numpy()
    # L has rank 4 plus damping: kappa ~ |g|^2 / eps ~ 1e5..1e6, so the fp32 root carries ~kappa 2^-24
    assert rel_frobenius_error(u[None], U_ref[None]).max() < 2e-3


def test_ragged_layer_step_end_to_end(dash):
    """A (320, 256) layer with B = 128: four full blocks and two 64 x 128 rest blocks.  The B x B factors
    L_full, R_full and R_rest go through ONE inverse-root call as S_full = stack(L_full, R_full, R_rest);
    S_rest = L_rest (64 x 64) through another (Section 4.1)."""
    import torch
    m, n, B = 320, 256, 128
    beta, eps, p, k = 0.9, 1e-5, 4, 30
    b32 = float(np.float32(beta)); a32 = float(np.float32(1.0) - np.float32(beta))
    plan = oblocking.stack_shapes(m, n, B)
    nf, nr = plan["G_full"][0], plan["G_row_rest"][0]
    assert (nf, nr) == (4, 2) and plan["S_full"] == (10, B, B) and plan["S_rest"] == [(2, 64, 64)]
    S_full = torch.zeros(2 * nf + nr, B, B, device="cuda")
    S_rest = torch.zeros(nr, 64, 64, device="cuda")
    factors = None
    for t in range(4):
        Wg = _layer(m, n, 500 + t)
        gr = dash.block_layer(_to_gpu(Wg), B)
        assert gr["col_rest"] is None and gr["corner"] is None
        dash.accumulate_factors(gr["full"], S_full[:nf], S_full[nf:2 * nf], beta)
        dash.accumulate_factors_rect(gr["row_rest"], S_rest, S_full[2 * nf:], beta)
        U_ref, factors = oblocking.layer_step(Wg, factors, B, b32, eps, p, a32)
    X_full = dash.inverse_root(S_full, method="newton_db", p=p, iters=k, eps=eps)
    X_rest = dash.inverse_root(S_rest, method="newton_db", p=p, iters=k, eps=eps)
    out = dict(full=dash.precondition(X_full[:nf], gr["full"], X_full[nf:2 * nf]),
               row_rest=dash.precondition_rect(X_rest, gr["row_rest"], X_full[2 * nf:]))
    U = torch.zeros(m, n, device="cuda")
    dash.unblock_layer(U, B, out)
    e = rel_frobenius_error(U.cpu().numpy()[None], U_ref[None]).max()
    print(f"ragged layer step: U vs per-slice EVD step {e:.2e}", flush=True)
    assert e < 1e-4


def test_invalid_arguments_of_the_new_entry_points(dash):
    import ctypes as C
    import torch
    from paper_2602_02016_amd import DashError
    z = lambda *sh: torch.zeros(*sh, device="cuda")
    with pytest.raises(DashError):
        dash.accumulate_vector(z(2, 100), z(2, 100, 100), 0.9)                  # B not a multiple of 64
    with pytest.raises(DashError):
        dash.precondition_vector(z(2, 64, 64), z(2, 128))                       # shapes do not match
    with pytest.raises(DashError):
        dash.graft_scale(z(2, 3, 2), z(2, 3, 2), z(2, 3, 2))                    # 6 elements per block: not a multiple of 4
    with pytest.raises(DashError):
        dash.apply_update(z(8)[1:], z(8)[1:], 0.1)                              # pointers not 16-byte aligned
    with pytest.raises(DashError):
        dash.block_layer(z(100, 100), 64, 48, 1)                                # the padding unit must divide B
    with pytest.raises(DashError):
        dash.precondition_rect(z(1, 64, 64), z(1, 64, 128), z(1, 64, 64))       # Rinv must be 128 x 128
    # null pointers reach the library and come back as status 1, not as a fault
    vp = C.c_void_p
    assert dash.lib.dash_accumulate_factors_rect(dash.h, vp(None), vp(None), vp(None), 1, 64, 128, 0.9, 0.1) == 1
    assert dash.lib.dash_block_layer(dash.h, vp(None), 64, 64, 64, vp(None), vp(None), vp(None), vp(None)) == 1
    assert dash.lib.dash_apply_update(dash.h, vp(None), vp(None), 64, 0.1) == 1
    assert dash.lib.dash_graft_scale(dash.h, vp(None), vp(None), vp(None), 1, 64, 0.9, 1e-8, vp(None), vp(None)) == 1
    # and an un-aligned parameter pointer is refused
    t = z(65)
    assert dash.lib.dash_apply_update(dash.h, vp(t.data_ptr() + 4), vp(t.data_ptr() + 4), 64, 0.1) == 1
