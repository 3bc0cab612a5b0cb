"""All layers of a small model in shared stacks (paper Section 4.1, stacking at the GPU level) through
dash_model_step, against the float64 oracle that steps every layer block by block on slices."""
import numpy as np
import pytest

from oracle import blocking as oblocking
from oracle.evd import rel_frobenius_error

pytestmark = pytest.mark.gpu

LAYERS = [(320, 256), (256, 320), (192, 192), (256,), (256,), (320,)]
B = 128


@pytest.fixture(scope="module")
def dash():
    from paper_2602_02016_amd import Dash
    d = Dash(0)
    yield d
    d.close()


def _grads(step):
    rng = np.random.default_rng(7000 + step)
    return [(rng.standard_normal(s) * (1e-2 if len(s) == 2 else 3e-3)).astype(np.float32) for s in LAYERS]


def _oracle_step(grads, state, beta, eps, refresh):
    b32 = float(np.float32(beta)); a32 = float(np.float32(1.0) - np.float32(beta))
    out, new = [], []
    for g, st in zip(grads, state):
        f, r = st if st is not None else (None, None)
        if g.ndim == 2:
            U, f, r = oblocking.layer_step_cached(g, f, r, B, b32, eps, 4, a32, refresh)
        else:
            U, f, r = oblocking.vector_param_step_cached(g, f, r, B, b32, eps, 2, a32, refresh)
        out.append(U); new.append((f, r))
    return out, new


@pytest.mark.parametrize("precision", ["fp32", "bf16x6", "fp16x3"])
@pytest.mark.parametrize("ws_cap", [None, 3 << 20])
def test_model_step_matches_per_layer_oracle(dash, ws_cap, precision):
    import torch
    from paper_2602_02016_amd import DashModel
    model = DashModel(dash, LAYERS, B, p=4, p_vec=2)
    plan = model.plan
    print("plan", plan["buckets"], plan["stacks"], flush=True)
    assert plan["buckets"] == [(128, 128, 9), (64, 128, 3), (128, 64, 3), (64, 64, 1), (128, 0, 6), (64, 0, 1)]
    assert plan["stacks"] == [(128, 4, 24), (64, 4, 8), (128, 2, 6), (64, 2, 1)]
    beta, eps, k = 0.9, 1e-5, 30
    state = [None] * len(LAYERS)
    nf = torch.ones(plan["info"]["n_factor_blocks"], dtype=torch.int32, device="cuda")
    if ws_cap is not None:
        dash.set_workspace_bytes(ws_cap)
    for step, refresh in enumerate([True, True, True, False, True]):
        g_np = _grads(step)
        grads = [torch.from_numpy(g).cuda() for g in g_np]
        ups = [torch.full_like(g, 7.0) for g in grads]
        dash.reset_stats()
        model.step(grads, ups, beta=beta, eps=eps, method="newton_db", iters=k, refresh=refresh, nonfinite_out=nf,
                   workspace_max_bytes=ws_cap, precision=precision)
        st = dash.get_stats()
        ref, state = _oracle_step(g_np, state, beta, eps, refresh)
        errs = [rel_frobenius_error(u.cpu().numpy().reshape(1, -1, 1) if u.dim() == 1 else u.cpu().numpy()[None],
                                    r.reshape(1, -1, 1) if r.ndim == 1 else r[None]).max() for u, r in zip(ups, ref)]
        print(f"step {step} refresh={refresh}: max err {max(errs):.2e}, matmul launches {st['matmul_launches']}", flush=True)
        assert max(errs) < 2e-4, errs
        assert int(nf.sum().item()) == 0
        if not refresh:
            # no inverse-root product ran: 2 per square bucket (accumulate, one launch for both factors ...)
            assert st["matmul_launches"] <= 4 * 4
    # the factor stacks hold what the oracle holds: stack 0 = all 128 x 128 factors, left factors first
    S0, _ = model.stack(0)
    f_first = state[0][0][(0, 0)][0]                      # L of block (0, 0) of layer 0 = first block of the stack
    assert rel_frobenius_error(S0[0].cpu().numpy()[None], f_first[None]).max() < 1e-5
    model.close()


def test_model_step_with_grafting_and_parameter_update(dash):
    """Grafted updates s_b U_b per block of every bucket shape and theta <- theta - lr * update (Section 2.3,
    Algorithm 1) against the oracle working on slices of each layer."""
    import torch
    from paper_2602_02016_amd import DashModel
    model = DashModel(dash, LAYERS, B, p=4, p_vec=2)
    beta, eps, k, beta_g, eps_g, lr = 0.9, 1e-5, 30, float(np.float32(0.999)), 1e-8, 0.01
    state = [None] * len(LAYERS)
    accs = [np.zeros(s) for s in LAYERS]
    rng = np.random.default_rng(99)
    theta_np = [rng.standard_normal(s).astype(np.float32) for s in LAYERS]
    thetas = [torch.from_numpy(t).cuda() for t in theta_np]
    theta_ref = [t.astype(np.float64) for t in theta_np]
    for step in range(3):
        g_np = _grads(step)
        grads = [torch.from_numpy(g).cuda() for g in g_np]
        ups = [torch.zeros_like(g) for g in grads]
        model.step(grads, ups, beta=beta, eps=eps, method="newton_db", iters=k, graft=True, beta_g=beta_g, eps_g=eps_g,
                   thetas=thetas, lr=lr)
        ref, state = _oracle_step(g_np, state, beta, eps, True)
        for i, (g, u) in enumerate(zip(g_np, ref)):
            ug, accs[i] = oblocking.graft_layer(g, u, accs[i], B, beta_g, eps_g)
            theta_ref[i] = theta_ref[i] - float(np.float32(lr)) * ug
            got = ups[i].cpu().numpy()
            e = np.linalg.norm(got - ug) / np.linalg.norm(ug)
            assert e < 2e-4, (step, i, e)
            et = np.abs(thetas[i].cpu().numpy() - theta_ref[i]).max()
            assert et < 1e-5, (step, i, et)
    print("grafted model step ok", flush=True)
    model.close()


ODD_LAYERS = [(300, 250), (131, 257), (64, 100), (190,), (77,)]


def test_model_step_any_layer_shape(dash):
    """Layers whose rest extents are not multiples of 64: the model pads them with zeros inside its stacks
    (rest blocks of 44 x 122 become 64 x 128, ...), which leaves the real part of factors, roots and updates
    what it is.  Against the oracle, which works on the exact shapes; with grafting and the parameter update."""
    import torch
    from paper_2602_02016_amd import DashModel
    model = DashModel(dash, ODD_LAYERS, B, p=4, p_vec=2)
    print("plan", model.plan["buckets"], model.plan["stacks"], flush=True)
    assert all(bm % 64 == 0 and bn % 64 == 0 for bm, bn, _ in model.plan["buckets"])
    beta, eps, k, beta_g, eps_g, lr = 0.9, 1e-5, 30, float(np.float32(0.999)), 1e-8, 0.01
    b32 = float(np.float32(beta)); a32 = float(np.float32(1.0) - np.float32(beta))
    state = [None] * len(ODD_LAYERS)
    accs = [np.zeros(s) for s in ODD_LAYERS]
    rng = np.random.default_rng(123)
    theta_np = [rng.standard_normal(s).astype(np.float32) for s in ODD_LAYERS]
    thetas = [torch.from_numpy(t).cuda() for t in theta_np]
    theta_ref = [t.astype(np.float64) for t in theta_np]
    nf = torch.ones(model.plan["info"]["n_factor_blocks"], dtype=torch.int32, device="cuda")
    for step in range(3):
        g_np = [(rng.standard_normal(s) * (1e-2 if len(s) == 2 else 3e-3)).astype(np.float32) for s in ODD_LAYERS]
        grads = [torch.from_numpy(g).cuda() for g in g_np]
        ups = [torch.full_like(g, 7.0) for g in grads]
        model.step(grads, ups, beta=beta, eps=eps, method="newton_db", iters=k, graft=True, beta_g=beta_g, eps_g=eps_g,
                   thetas=thetas, lr=lr, nonfinite_out=nf)
        assert int(nf.sum().item()) == 0
        for i, g in enumerate(g_np):
            f, r = state[i] if state[i] is not None else (None, None)
            if g.ndim == 2:
                u, f, r = oblocking.layer_step_cached(g, f, r, B, b32, eps, 4, a32, True)
            else:
                u, f, r = oblocking.vector_param_step_cached(g, f, r, B, b32, eps, 2, a32, True)
            state[i] = (f, r)
            ug, accs[i] = oblocking.graft_layer(g, u, accs[i], B, beta_g, eps_g)
            theta_ref[i] = theta_ref[i] - float(np.float32(lr)) * ug
            got = ups[i].cpu().numpy()
            e = np.linalg.norm(got - ug) / np.linalg.norm(ug)
            assert e < 2e-4, (step, i, ODD_LAYERS[i], e)
            assert np.abs(thetas[i].cpu().numpy() - theta_ref[i]).max() < 1e-5, (step, i)
    print("odd-shaped model step ok", flush=True)
    model.close()


def test_model_errors(dash):
    import torch
    from paper_2602_02016_amd import DashModel, DashError
    padded = DashModel(dash, [(100, 128)], 128)            # 100 rows: one rest block, padded to 128 x 128
    assert padded.plan["buckets"] == [(128, 128, 1)]
    padded.close()
    model = DashModel(dash, [(128, 128)], 128)
    g = torch.zeros(128, 128, device="cuda")
    with pytest.raises(DashError):
        model.step([g], [g, g], beta=0.9, eps=1e-6)
    with pytest.raises(DashError):
        model.step([torch.zeros(64, 128, device="cuda")], [g], beta=0.9, eps=1e-6)
    empty = DashModel(dash, [], 128)
    empty.step([], [], beta=0.9, eps=1e-6)
    assert empty.plan["info"]["n_factor_blocks"] == 0
