"""Pins of oracle/blocking.py: the worked example of paper Section 4.1 (shapes and counts), round
trips, the blocked step against the un-blocked definition, and the 1-D case against closed forms."""
import os

import numpy as np
import pytest

from oracle import blocking, shampoo
from oracle.evd import inverse_root_evd

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_blocking_example.txt")


def _golden():
    out = {}
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        k, v = [t.strip() for t in line.split("=")]
        out[k] = tuple(int(t) for t in v.split(",")) if "," in v else int(v)
    return out


def test_paper_worked_example_shapes():
    g = _golden()
    sh = blocking.stack_shapes(g["V"], g["E"], g["B"])
    assert sh["G_full"] == g["G_full"] and sh["G_row_rest"] == g["G_rest"]
    assert sh["L_row_rest"] == g["L_rest"] and sh["R_row_rest"] == g["R_rest"]
    assert sh["S_full"] == g["S_full"] and sh["S_rest"] == [g["S_rest"]]
    assert "G_col_rest" not in sh and "G_corner" not in sh
    # the classification head is the transposed layer: L_rest and R_rest swap roles
    sh_t = blocking.stack_shapes(g["E"], g["V"], g["B"])
    assert sh_t["R_col_rest"] == g["L_rest"] and sh_t["L_col_rest"] == g["R_rest"] and sh_t["S_full"] == g["S_full"]
    # the library's host-side plan gives the same group shapes
    from paper_2602_02016_amd.binding import layer_plan
    plan = layer_plan(g["V"], g["E"], g["B"])
    assert plan["full"] == g["G_full"] and plan["row_rest"] == g["G_rest"] and plan["col_rest"][0] == 0 and plan["corner"][0] == 0


def test_small_scale_example_array_shapes():
    # the same layer scaled down 64x: (500, 32), B = 16 -> 31 x 2 full blocks and 2 rest blocks of 4 rows
    W = np.arange(500 * 32, dtype=np.float64).reshape(500, 32)
    gr = blocking.block_layer(W, 16)
    assert gr["full"].shape == (62, 16, 16) and gr["row_rest"].shape == (2, 4, 16)
    assert gr["col_rest"].shape[0] == 0 and gr["corner"].shape[0] == 0
    # block (i, j) sits at index i*Nn + j: element (0,0) of block (3,1) is W[48, 16]
    assert gr["full"][3 * 2 + 1][0, 0] == W[48, 16] and gr["row_rest"][1][3, 15] == W[499, 31]


@pytest.mark.parametrize("m,n,B", [(7, 5, 2), (8, 8, 4), (3, 9, 4), (10, 3, 4), (5, 5, 8)])
def test_round_trip_and_every_element_once(m, n, B):
    W = np.arange(m * n, dtype=np.float64).reshape(m, n) + 1
    gr = blocking.block_layer(W, B)
    assert sum(v.size for v in gr.values()) == m * n
    allv = np.sort(np.concatenate([v.ravel() for v in gr.values()]))
    assert np.array_equal(allv, np.sort(W.ravel()))
    assert np.array_equal(blocking.unblock_layer(gr, m, n, B), W)


def test_blocked_step_equals_per_group_stack_step():
    """layer_step (slices of the layer) against the stacked route: block -> accumulate/precondition per
    group with oracle.shampoo -> unblock."""
    rng = np.random.default_rng(5)
    m, n, B = 11, 10, 4
    Wg = rng.standard_normal((m, n))
    U_ref, fac = blocking.layer_step(Wg, None, B, beta=0.9, eps=1e-3, p=4)
    gr = blocking.block_layer(Wg, B)
    out = {}
    for k, G in gr.items():
        if G.shape[0] == 0:
            out[k] = G
            continue
        L0 = np.zeros((G.shape[0], G.shape[1], G.shape[1])); R0 = np.zeros((G.shape[0], G.shape[2], G.shape[2]))
        L, R = shampoo.accumulate_factors(G, L0, R0, 0.9)
        out[k] = shampoo.precondition(inverse_root_evd(L, 4, 1e-3), G, inverse_root_evd(R, 4, 1e-3))
    U = blocking.unblock_layer(out, m, n, B)
    assert np.allclose(U, U_ref, rtol=1e-10, atol=1e-12)
    # one block covering the whole layer (B >= m, n) is full-matrix Shampoo
    U_one, _ = blocking.layer_step(Wg, None, 16, beta=0.9, eps=1e-3, p=4)
    L = 0.1 * Wg @ Wg.T; R = 0.1 * Wg.T @ Wg
    assert np.allclose(U_one, inverse_root_evd(L, 4, 1e-3) @ Wg @ inverse_root_evd(R, 4, 1e-3), rtol=1e-10, atol=1e-12)


def test_vector_step_closed_form():
    """From L = 0, one accumulation gives the rank-one L = alpha g g^T, whose damped inverse square
    root acts on g as (alpha |g|^2 + eps)^(-1/2): u = g / sqrt(alpha |g|^2 + eps)."""
    rng = np.random.default_rng(9)
    N, E, B = 3, 8, 4
    grads = rng.standard_normal((N, E))
    L0 = np.zeros((N * E // B, B, B))
    U, L1 = blocking.norm_layers_step(grads, L0, B, beta=0.75, eps=1e-2)
    g = grads.reshape(-1, B)
    expect = g / np.sqrt(0.25 * (g * g).sum(axis=1, keepdims=True) + 1e-2)
    assert np.allclose(U, expect.reshape(N, E), rtol=1e-10)
    assert np.allclose(L1, 0.25 * g[:, :, None] * g[:, None, :])
    # a vector is a B x 1 matrix: the matrix functions give the same L and the same u
    Lm, Rm = shampoo.accumulate_factors(g[:, :, None], L0, np.zeros((g.shape[0], 1, 1)), 0.75)
    assert np.allclose(Lm, L1) and np.allclose(Rm[:, 0, 0], 0.25 * (g * g).sum(axis=1))
    assert np.allclose(blocking.precondition_vector(L1, g)[:, :, None], np.matmul(L1, g[:, :, None]))


def test_cached_roots_schedule():
    """refresh = True reproduces layer_step; refresh = False keeps the old roots but still moves the factors."""
    rng = np.random.default_rng(21)
    m, n, B = 6, 7, 4
    G1, G2 = rng.standard_normal((m, n)), rng.standard_normal((m, n))
    U1, f1 = blocking.layer_step(G1, None, B, 0.9, 1e-3)
    U1c, f1c, r1c = blocking.layer_step_cached(G1, None, None, B, 0.9, 1e-3)
    assert np.array_equal(U1, U1c) and all(np.array_equal(f1[k][0], f1c[k][0]) for k in f1)
    U2s, f2s, r2s = blocking.layer_step_cached(G2, f1c, r1c, B, 0.9, 1e-3, refresh=False)
    _, f2 = blocking.layer_step(G2, f1, B, 0.9, 1e-3)
    assert all(np.array_equal(f2[k][1], f2s[k][1]) for k in f2)            # factors moved
    assert all(r2s[k][0] is r1c[k][0] for k in r1c)                        # roots did not
    XL, XR = r1c[(4, 4)]
    assert np.allclose(U2s[4:, 4:], XL @ G2[4:, 4:] @ XR)
    # a 1-D parameter is the E x 1 layer with the right factor (a positive scalar) dropped
    g = rng.standard_normal(10)
    u, fv, rv = blocking.vector_param_step_cached(g, None, None, 4, 0.9, 1e-3, p=2)
    un, Ln = blocking.norm_layers_step(g[None, :8], np.zeros((2, 4, 4)), 4, 0.9, 1e-3)
    assert np.allclose(u[:8], un[0]) and np.allclose(fv[1], Ln[1]) and fv[2].shape == (2, 2)


def test_model_plan_matches_paper_example_and_counts():
    """The library's host-side plan (no GPU needed): the paper's embedding example gives S_full of 126
    blocks of 1024 and S_rest of 2 blocks of 256; sharing stacks across layers only adds counts."""
    from paper_2602_02016_amd import model_plan
    g = _golden()
    plan = model_plan([(g["V"], g["E"])], g["B"])
    assert plan["buckets"] == [(1024, 1024, 62), (256, 1024, 2)]
    assert plan["stacks"] == [(g["S_full"][1], 4, g["S_full"][0]), (g["S_rest"][1], 4, g["S_rest"][0])]
    # embedding + classification head (transposed) + two square layers + two normalisation layers
    plan = model_plan([(32000, 2048), (2048, 32000), (2048, 2048), (2048, 8192), (2048,), (2048,)], 1024)
    sh = [blocking.stack_shapes(m, n, 1024) for m, n in [(32000, 2048), (2048, 32000), (2048, 2048), (2048, 8192)]]
    assert dict((s, c) for s, p, c in plan["stacks"] if p == 4) == {1024: sum(x["S_full"][0] for x in sh), 256: 4}
    assert [(s, p, c) for s, p, c in plan["stacks"] if p == 2] == [(1024, 2, 4)]
    assert plan["info"]["n_gradient_blocks"] == sum(x["G_full"][0] for x in sh) + 2 + 2 + 4
    # a rest extent that is not a multiple of 64 is rounded up inside the model's stacks (zero padding):
    # 1000 rows -> one row of rest blocks padded to 1024 x 1024; 100 rows, 130 columns -> 128 x 1024, 1024 x 64, 128 x 64
    assert model_plan([(1000, 2048)], 1024)["buckets"] == [(1024, 1024, 2)]
    assert model_plan([(1124, 1154)], 1024)["buckets"] == [(1024, 1024, 1), (128, 1024, 1), (1024, 192, 1), (128, 192, 1)]
    assert model_plan([(1100,)], 1024)["buckets"] == [(1024, 0, 1), (128, 0, 1)]


def test_graft_layer_against_stack_grafting_and_norm_property():
    """graft_layer (slices of the layer) equals oracle.shampoo.adam_graft on the blocked stacks, and the
    grafted block has exactly the Frobenius norm of the Adam direction of that block."""
    rng = np.random.default_rng(33)
    m, n, B = 8, 12, 4
    G, U, Acc = rng.standard_normal((m, n)), rng.standard_normal((m, n)), rng.random((m, n))
    Ug, Acc1 = blocking.graft_layer(G, U, Acc, B, 0.9, 1e-8)
    gs, us, accs = (blocking.block_layer(x, B)["full"] for x in (G, U, Acc))
    acc_ref, s_ref = shampoo.adam_graft(gs, us, accs, 0.9, 1e-8)
    assert np.allclose(blocking.block_layer(Acc1, B)["full"], acc_ref)
    assert np.allclose(blocking.block_layer(Ug, B)["full"], s_ref[:, None, None] * us)
    P = G / (1e-8 + np.sqrt(Acc1))
    assert np.isclose(np.linalg.norm(Ug[4:8, 8:12]), np.linalg.norm(P[4:8, 8:12]))
    # 1-D: pieces of B entries and a shorter last one
    g, u, a = rng.standard_normal(10), rng.standard_normal(10), rng.random(10)
    ug, a1 = blocking.graft_layer(g, u, a, 4, 0.9, 1e-8)
    p1 = g / (1e-8 + np.sqrt(a1))
    assert np.isclose(np.linalg.norm(ug[8:]), np.linalg.norm(p1[8:])) and np.allclose(ug[:4] / u[:4], ug[0] / u[0])
