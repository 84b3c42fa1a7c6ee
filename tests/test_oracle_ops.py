"""Pins of the oracle's GEMM, SDDMM, edge softmax, SPMM and projection steps.

Each is checked against the dense-matrix definition the paper writes (Sec. 2.1), on graphs small enough for
brute force, plus the invariants and the values the paper prints for its running example.
"""
import json
import os

import numpy as np
import pytest

import oracle as orc
import tango_inputs as ti
from dense_ref import from_dense, gat_backward, gat_forward, lrelu, mask, to_dense


@pytest.fixture(scope="module")
def paper(golden_dir):
    return json.load(open(os.path.join(golden_dir, "paper_worked_example.json")))


def small_graph(n=48, m=300, seed=5):
    return ti.toy_graph(n, m, seed)


def rand_i8(shape, seed):
    return np.random.default_rng(seed).integers(-127, 128, size=shape, dtype=np.int8)


# ------------------------------------------------------------------ GEMM
def test_fig3_dot_needs_int32(paper):
    ex = paper["fig3_int32_accumulation"]
    a = np.array([ex["row"]], np.int8)
    b = np.array(ex["col"], np.int8).reshape(-1, 1)
    acc = orc.igemm(a, b)
    assert acc.dtype == np.int32 and int(acc[0, 0]) == ex["dot"]
    assert abs(ex["dot"]) > 127


@pytest.mark.parametrize("ta,tb", [(False, False), (True, False), (False, True), (True, True)])
def test_igemm_matches_int64_matmul(ta, tb):
    M, N, K = 13, 9, 37
    A = rand_i8((K, M) if ta else (M, K), 1)
    B = rand_i8((N, K) if tb else (K, N), 2)
    want = (A.T if ta else A).astype(np.int64) @ (B.T if tb else B).astype(np.int64)
    got = orc.igemm(A, B, ta, tb)
    assert np.array_equal(got.astype(np.int64), want)


def test_igemm_reports_overflow():
    K = 140000  # 127*127*140000 > 2^31
    A = np.full((1, K), 127, np.int8)
    B = np.full((K, 1), 127, np.int8)
    with pytest.raises(OverflowError):
        orc.igemm(A, B)


def test_dequant_formula_and_absmax():
    acc = np.array([[11781, -3, 0], [7, -20000, 5]], np.int32)
    sa, sb = np.float32(0.0123), np.float32(0.0456)
    C, am = orc.dequant_i32(acc, sa, sb)
    sc = np.float32(sa * sb)  # scales first
    assert np.array_equal(C, acc.astype(np.float32) * sc)
    assert am == np.abs(C).max()
    # the abs-max of the dequantized result is the dequantized abs-max accumulator
    assert am == np.float32(np.float32(20000) * sc)


def test_qgemm_within_quantization_bound():
    rng = np.random.default_rng(3)
    M, K, N = 40, 64, 24
    A = rng.standard_normal((M, K)).astype(np.float32)
    B = rng.uniform(-0.3, 0.3, (K, N)).astype(np.float32)
    exact = A.astype(np.float64) @ B.astype(np.float64)
    r = orc.qgemm(A, B, orc.RN)
    # first-order bound for nearest rounding: sum_k (|a| sB/2 + |b| sA/2) + K sA sB / 4
    bound = (
        np.abs(A).astype(np.float64).sum(1)[:, None] * float(r["s_B"]) / 2
        + np.abs(B).astype(np.float64).sum(0)[None, :] * float(r["s_A"]) / 2
        + K * float(r["s_A"]) * float(r["s_B"]) / 4
    )
    assert (np.abs(r["C"] - exact) <= bound * (1 + 1e-4) + 1e-6).all()
    assert np.abs(r["C"] - exact).max() > 0  # it is a quantized product, not the exact one
    rs = orc.qgemm(A, B, orc.SR, seed=4)
    assert np.abs(rs["C"] - exact).max() <= 2 * bound.max()
    assert rs["absmax_C"] == np.abs(rs["C"]).max()


def test_qgemm_bwd_is_transposed_products():
    rng = np.random.default_rng(4)
    M, K, N = 30, 20, 12
    A_q, B_q = rand_i8((M, K), 5), rand_i8((K, N), 6)
    dC = rng.standard_normal((M, N)).astype(np.float32)
    r = orc.qgemm_bwd(A_q, np.float32(0.01), B_q, np.float32(0.02), dC, orc.RN)
    dCq = r["dC_q"].astype(np.int64)
    wantA = (dCq @ B_q.T.astype(np.int64)).astype(np.float32) * np.float32(r["s_dC"] * np.float32(0.02))
    wantB = (A_q.T.astype(np.int64) @ dCq).astype(np.float32) * np.float32(np.float32(0.01) * r["s_dC"])
    assert np.array_equal(r["dA"], wantA) and np.array_equal(r["dB"], wantB)
    # and they approximate the real gradients of C = A.B
    Af = 0.01 * A_q.astype(np.float64)
    Bf = 0.02 * B_q.astype(np.float64)
    assert np.allclose(r["dA"], dC.astype(np.float64) @ Bf.T, atol=0.02 * np.abs(dC @ Bf.T).max())
    assert np.allclose(r["dB"], Af.T @ dC.astype(np.float64), atol=0.02 * np.abs(Af.T @ dC).max())


# --------------------------------------------------------- head projections
def test_head_proj_paper_value(paper):
    ex = paper["step2_head_projection"]
    out = orc.head_proj(np.array([ex["Hp_v0"]], np.float32), np.array(ex["a_src"], np.float32))
    assert np.allclose(out[0], ex["S_v0"], atol=0.011)


def test_head_proj_matches_einsum():
    rng = np.random.default_rng(7)
    X = rng.standard_normal((50, 3 * 8)).astype(np.float32)
    a = rng.standard_normal((3, 8)).astype(np.float32)
    want = np.einsum("vhd,hd->vh", X.reshape(50, 3, 8).astype(np.float64), a.astype(np.float64))
    assert np.array_equal(orc.head_proj(X, a), want.astype(np.float32))


# ------------------------------------------------------------------ SDDMM
def test_sddmm_add_dense_definition():
    g = small_graph()
    heads = 3
    S_q, D_q = rand_i8((g.n_nodes, heads), 1), rand_i8((g.n_nodes, heads), 2)
    sS, sD, slope = np.float32(0.013), np.float32(0.007), 0.2
    E = orc.sddmm_add(g, S_q, sS, D_q, sD, slope)
    S = sS * S_q.astype(np.float32)
    D = sD * D_q.astype(np.float32)
    T = S.T[:, None, :] + D.T[:, :, None]  # [h, v, u] = S[u] + D[v], fp32
    dense = np.where(T > 0, T, np.float32(slope) * T) * mask(g)[None]
    assert np.array_equal(E, from_dense(g, dense))


def test_sddmm_add_paper_value(paper):
    ex = paper["step3_sddmm_add"]
    g = ti.graph_from_edges(4, [0], [3], self_loops=False)
    S = np.zeros((4, 2), np.float32)
    D = np.zeros((4, 2), np.float32)
    S[0] = ex["S_v0"]
    D[3] = ex["D_v3"]
    S_q, sS = orc.quantize(S, orc.RN)
    D_q, sD = orc.quantize(D, orc.RN)
    E = orc.sddmm_add(g, S_q, sS, D_q, sD, 0.0)  # the figure shows negative entries as 0
    assert np.allclose(E[0], ex["E_e3_after_lrelu"], atol=0.011 + float(sS) / 2 + float(sD) / 2)
    E = orc.sddmm_add(g, S_q, sS, D_q, sD, 1.0)  # slope 1 = no activation
    assert np.allclose(E[0], ex["E_e3_before_lrelu"], atol=0.011 + float(sS) / 2 + float(sD) / 2)


def test_sddmm_dot_dense_definition():
    g = small_graph()
    heads, dim = 2, 8
    Xd, Xs = rand_i8((g.n_nodes, heads * dim), 3), rand_i8((g.n_nodes, heads * dim), 4)
    out, acc = orc.sddmm_dot(g, Xd, np.float32(0.01), Xs, np.float32(0.03), heads, want_acc=True)
    dense = np.einsum(
        "vhd,uhd->hvu", Xd.reshape(-1, heads, dim).astype(np.int64), Xs.reshape(-1, heads, dim).astype(np.int64)
    )
    want_acc = from_dense(g, dense * mask(g)[None])
    assert np.array_equal(acc.astype(np.int64), want_acc)
    assert np.array_equal(out, want_acc.astype(np.float32) * np.float32(np.float32(0.01) * np.float32(0.03)))


def test_sddmm_dot_paper_value(paper):
    ex = paper["step5pp_sddmm_dot"]
    g = ti.graph_from_edges(2, [1], [0], self_loops=False)
    dH = np.zeros((2, 4), np.float32)
    Hp = np.zeros((2, 4), np.float32)
    dH[0] = ex["dH_v0"]
    Hp[1] = ex["Hp_v1"]
    dq, sd = orc.quantize(dH, orc.RN)
    hq, sh = orc.quantize(Hp, orc.RN)
    out = orc.sddmm_dot(g, dq, sd, hq, sh, heads=2)
    assert np.allclose(out[0], ex["dalpha_e0"], atol=0.02)


# ------------------------------------------------------------ edge softmax
def test_softmax_paper_value(paper):
    ex = paper["step4_softmax"]
    g = ti.graph_from_edges(4, [0, 2], [3, 3], self_loops=False)
    E = np.array([ex["E_e3"], ex["E_e4"]], np.float32)
    a = orc.edge_softmax(g, E)
    assert np.allclose(a[0], ex["alpha_e3"], atol=0.006) and np.allclose(a[1], ex["alpha_e4"], atol=0.006)


def test_softmax_dense_and_invariants():
    g = small_graph()
    heads = 3
    rng = np.random.default_rng(8)
    E = (4 * rng.standard_normal((g.n_edges, heads))).astype(np.float32)
    a = orc.edge_softmax(g, E)
    G = mask(g)
    Ed = to_dense(g, E.astype(np.float64))
    ex = np.where(G[None], np.exp(Ed), 0.0)  # the paper's formula, no max subtraction
    want = from_dense(g, ex / ex.sum(axis=2, keepdims=True))
    assert np.allclose(a, want, rtol=1e-6, atol=1e-9)
    sums = np.add.reduceat(a.astype(np.float64), g.in_ptr[:-1], axis=0)
    assert np.allclose(sums, 1.0, atol=1e-6)
    # adding a per-destination constant changes nothing (beyond fp32 rounding of the shifted input)
    shift = rng.standard_normal((g.n_nodes, heads)).astype(np.float32)[g.in_dst()]
    a2 = orc.edge_softmax(g, E + shift)
    assert np.allclose(a2, a, rtol=1e-5, atol=1e-7)
    # large scores do not overflow
    a3 = orc.edge_softmax(g, E + np.float32(1000.0))
    assert np.isfinite(a3).all() and np.allclose(a3, a, rtol=1e-3, atol=1e-6)


def test_softmax_single_in_edge_is_one():
    g = ti.graph_from_edges(3, [0, 1], [1, 2], self_loops=False)
    a = orc.edge_softmax(g, np.array([[3.0, -50.0], [0.1, 7.0]], np.float32))
    assert np.array_equal(a, np.ones((2, 2), np.float32))


def test_softmax_bwd_paper_value(paper):
    ex = paper["step4p_softmax_bwd"]
    g = ti.graph_from_edges(4, [0, 2], [3, 3], self_loops=False)
    alpha = np.array(ex["alpha"], np.float32).reshape(2, 1)
    dalpha = np.array(ex["dalpha"], np.float32).reshape(2, 1)
    dE = orc.edge_softmax_bwd(g, alpha, dalpha)
    P = float((alpha * dalpha).sum())
    assert abs(P - ex["P_v3"]) < 0.006
    assert abs(float(dE[0, 0]) - ex["dE_e3"]) < 0.006


def test_softmax_bwd_sums_to_zero_and_finite_difference():
    g = small_graph(24, 100, 9)
    heads = 2
    rng = np.random.default_rng(10)
    E = rng.standard_normal((g.n_edges, heads))
    up = rng.standard_normal((g.n_edges, heads))

    def soft(Ev):
        G = mask(g)
        ex = np.where(G[None], np.exp(to_dense(g, Ev)), 0.0)
        return from_dense(g, ex / ex.sum(axis=2, keepdims=True))

    alpha = soft(E)
    dE = orc.edge_softmax_bwd(g, alpha.astype(np.float32), up.astype(np.float32))
    sums = np.add.reduceat(dE.astype(np.float64), g.in_ptr[:-1], axis=0)
    assert np.abs(sums).max() < 1e-6
    # d/dE <up, softmax(E)> by central differences
    num = np.zeros_like(E)
    h = 1e-6
    for idx in rng.choice(E.size, 40, replace=False):
        e, k = divmod(int(idx), heads)
        Ep, Em = E.copy(), E.copy()
        Ep[e, k] += h
        Em[e, k] -= h
        num[e, k] = ((soft(Ep) - soft(Em)) * up).sum() / (2 * h)
        assert abs(num[e, k] - dE[e, k]) < 1e-5


# -------------------------------------------------------------------- SPMM
def test_spmm_dense_definition_both_directions():
    g = small_graph()
    heads, dim = 3, 4
    w = rand_i8((g.n_edges, heads), 11)
    X = rand_i8((g.n_nodes, heads * dim), 12)
    sw, sx = np.float32(1 / 127), np.float32(0.02)
    Wd = to_dense(g, w.astype(np.int64))  # [h, v, u]
    X3 = X.reshape(-1, heads, dim).astype(np.int64)
    out, am, acc = orc.spmm_in(g, w, sw, X, sx, want_acc=True)
    want = np.einsum("hvu,uhd->vhd", Wd, X3).reshape(g.n_nodes, -1)
    assert np.array_equal(acc.astype(np.int64), want)
    assert np.array_equal(out, want.astype(np.float32) * np.float32(sw * sx)) and am == np.abs(out).max()
    out, am, acc = orc.spmm_rev(g, w, sw, X, sx, want_acc=True)
    want = np.einsum("hvu,vhd->uhd", Wd, X3).reshape(g.n_nodes, -1)
    assert np.array_equal(acc.astype(np.int64), want)
    assert np.array_equal(out, want.astype(np.float32) * np.float32(sw * sx)) and am == np.abs(out).max()


def test_spmm_adjoint_identity_exact():
    g = small_graph(40, 250, 13)
    heads, dim = 2, 8
    w = rand_i8((g.n_edges, heads), 14)
    X = rand_i8((g.n_nodes, heads * dim), 15)
    Y = rand_i8((g.n_nodes, heads * dim), 16)
    one = np.float32(1.0)
    a = orc.spmm_in(g, w, one, X, one, want_acc=True)[2].astype(np.int64)
    b = orc.spmm_rev(g, w, one, Y, one, want_acc=True)[2].astype(np.int64)
    assert (a * Y.astype(np.int64)).sum() == (X.astype(np.int64) * b).sum()


def test_spmm_rev_paper_value(paper):
    ex = paper["step5p_spmm_reverse"]
    g = ti.graph_from_edges(3, [1, 1], [0, 2], self_loops=False)  # e0 = v1->v0, e2 = v1->v2
    alpha = np.ones((2, 2), np.float32)
    aq, sa = orc.quantize(alpha, orc.RN)
    assert (aq == 127).all()
    dH = np.zeros((3, 4), np.float32)
    dH[0] = ex["dH_v0"]
    dH[2] = ex["dH_v2"]
    gq, sg = orc.quantize(dH, orc.RN)
    out, _ = orc.spmm_rev(g, aq, sa, gq, sg)
    assert np.allclose(out[1], ex["dHp_v1"], atol=0.011 + float(sg))


def test_fp32_twins_dense_definitions():
    g = small_graph(40, 260, 17)
    heads, dim = 2, 4
    rng = np.random.default_rng(18)
    w = rng.standard_normal((g.n_edges, heads)).astype(np.float32)
    X = rng.standard_normal((g.n_nodes, heads * dim)).astype(np.float32)
    Y = rng.standard_normal((g.n_nodes, heads * dim)).astype(np.float32)
    Wd = to_dense(g, w.astype(np.float64))
    X3 = X.reshape(-1, heads, dim).astype(np.float64)
    Y3 = Y.reshape(-1, heads, dim).astype(np.float64)
    assert np.array_equal(orc.spmm_f32(g, w, X), np.einsum("hvu,uhd->vhd", Wd, X3).reshape(g.n_nodes, -1).astype(np.float32))
    assert np.array_equal(orc.spmm_f32(g, w, Y, reverse=True),
                          np.einsum("hvu,vhd->uhd", Wd, Y3).reshape(g.n_nodes, -1).astype(np.float32))
    dense = np.einsum("vhd,uhd->hvu", Y3, X3) * mask(g)[None]
    assert np.array_equal(orc.sddmm_dot_f32(g, Y, X, heads), from_dense(g, dense).astype(np.float32))


# ---------------------------------------------------- SDDMM-add backward / sums
def test_sddmm_add_bwd_dense_definition():
    g = small_graph()
    heads = 2
    S_q, D_q = rand_i8((g.n_nodes, heads), 21), rand_i8((g.n_nodes, heads), 22)
    sS, sD, slope = np.float32(0.02), np.float32(0.015), 0.2
    rng = np.random.default_rng(23)
    dEp = rng.standard_normal((g.n_edges, heads)).astype(np.float32)
    dE, dS, dD = orc.sddmm_add_bwd(g, S_q, sS, D_q, sD, slope, dEp)
    S = sS * S_q.astype(np.float32)
    D = sD * D_q.astype(np.float32)
    T = S.T[:, None, :] + D.T[:, :, None]
    dT = to_dense(g, dEp) * np.where(T > 0, np.float32(1.0), np.float32(slope)) * mask(g)[None]
    assert np.array_equal(dE, from_dense(g, dT))
    assert np.allclose(dD, dT.astype(np.float64).sum(axis=2).T, rtol=1e-6, atol=1e-7)
    assert np.allclose(dS, dT.astype(np.float64).sum(axis=1).T, rtol=1e-6, atol=1e-7)


def test_head_proj_bwd_definition():
    rng = np.random.default_rng(30)
    n, heads, dim = 37, 3, 8
    dS = rng.standard_normal((n, heads)).astype(np.float32)
    dD = rng.standard_normal((n, heads)).astype(np.float32)
    a_s = rng.standard_normal((heads, dim)).astype(np.float32)
    a_d = rng.standard_normal((heads, dim)).astype(np.float32)
    Xq = rand_i8((n, heads * dim), 31)
    sX = np.float32(0.017)
    agg = rng.standard_normal((n, heads * dim)).astype(np.float32)
    dX, am, da_s, da_d = orc.head_proj_bwd(dS, dD, a_s, a_d, Xq, sX, agg)
    att = (dS[:, :, None] * a_s[None] + dD[:, :, None] * a_d[None]).reshape(n, -1)  # fp32 ops, same order
    assert np.array_equal(dX, agg + att) and am == np.abs(dX).max()
    X = (sX * Xq.astype(np.float32)).astype(np.float64).reshape(n, heads, dim)
    assert np.allclose(da_s, np.einsum("vh,vhd->hd", dS.astype(np.float64), X), rtol=1e-6, atol=1e-6)
    assert np.allclose(da_d, np.einsum("vh,vhd->hd", dD.astype(np.float64), X), rtol=1e-6, atol=1e-6)


# ------------------------------------------------------------- whole layer
def rel_err(a, b):
    return np.linalg.norm(np.asarray(a, np.float64) - b) / np.linalg.norm(b)


def test_fp64_twin_gradients_by_finite_differences():
    """The dense fp64 layer used as yardstick below has a correct analytic backward."""
    g = small_graph(12, 40, 41)
    rng = np.random.default_rng(42)
    heads, dim, K = 2, 3, 5
    H = rng.standard_normal((g.n_nodes, K))
    W = rng.standard_normal((K, heads * dim)) * 0.5
    a_s = rng.standard_normal((heads, dim)) * 0.5
    a_d = rng.standard_normal((heads, dim)) * 0.5
    up = rng.standard_normal((g.n_nodes, heads * dim))
    f = gat_forward(g, H, W, a_s, a_d, 0.2)
    b = gat_backward(g, H, W, a_s, a_d, 0.2, f, up)

    def loss(H_, W_, as_, ad_):
        return (gat_forward(g, H_, W_, as_, ad_, 0.2)["out"] * up).sum()

    h = 1e-6
    for name, arr, grad in (("H", H, b["dH"]), ("W", W, b["dW"]), ("a_src", a_s, b["da_src"]), ("a_dst", a_d, b["da_dst"])):
        for idx in rng.choice(arr.size, min(12, arr.size), replace=False):
            i = np.unravel_index(int(idx), arr.shape)
            args = dict(H=H.copy(), W=W.copy(), a_src=a_s.copy(), a_dst=a_d.copy())
            args[name][i] += h
            up_ = loss(args["H"], args["W"], args["a_src"], args["a_dst"])
            args[name][i] -= 2 * h
            dn_ = loss(args["H"], args["W"], args["a_src"], args["a_dst"])
            assert abs((up_ - dn_) / (2 * h) - grad[i]) < 1e-5 * max(1.0, abs(grad[i])), name


@pytest.mark.parametrize("rounding", [orc.RN, orc.SR])
def test_quantized_gat_layer_close_to_fp64_layer(rounding):
    g = small_graph(64, 512, 43)
    li_seed = 44
    heads, dim, K = 2, 16, 32
    H = ti.normal((g.n_nodes, K), li_seed)
    W = ti.xavier_uniform(K, heads * dim, (K, heads * dim), li_seed + 1)
    a_s = ti.xavier_uniform(heads, dim, (heads, dim), li_seed + 2)
    a_d = ti.xavier_uniform(heads, dim, (heads, dim), li_seed + 3)
    up = ti.normal((g.n_nodes, heads * dim), li_seed + 4)
    f = orc.gat_layer_fwd(g, H, W, a_s, a_d, 0.2, rounding, seed=9)
    b = orc.gat_layer_bwd(g, f, a_s, a_d, up, 0.2, rounding, seed=9)
    rf = gat_forward(g, H, W, a_s, a_d, 0.2)
    rb = gat_backward(g, H, W, a_s, a_d, 0.2, rf, up)
    # a chain of up to five int8 quantizations; dS/dD are sums with heavy cancellation (sum of dE_sm over a
    # row is 0), so their relative error is several times larger.  A mis-wired composition gives O(1) errors.
    tol = 0.04 if rounding == orc.RN else 0.12
    assert rel_err(f["Hp"], rf["Hp"]) < tol
    assert rel_err(f["alpha"], from_dense(g, rf["alpha"])) < tol
    assert rel_err(f["out"], rf["out"]) < tol
    assert rel_err(b["dHp_agg"], rb["dHp_agg"]) < tol
    assert rel_err(b["dalpha"], from_dense(g, rb["dalpha"])) < tol
    assert rel_err(b["dS"], rb["dS"]) < 3 * tol and rel_err(b["dD"], rb["dD"]) < 3 * tol
    assert rel_err(b["dHp"], rb["dHp"]) < tol
    assert rel_err(b["dW"], rb["dW"]) < tol
    assert rel_err(b["dH"], rb["dH"]) < tol
    assert rel_err(b["da_src"], rb["da_src"]) < 3 * tol and rel_err(b["da_dst"], rb["da_dst"]) < 3 * tol


def test_quantized_gcn_layer_close_to_fp64_layer():
    g = small_graph(64, 512, 45)
    K, F = 32, 48
    H = ti.normal((g.n_nodes, K), 46)
    W = ti.xavier_uniform(K, F, (K, F), 47)
    up = ti.normal((g.n_nodes, F), 48)
    w = ti.gcn_edge_weights(g)
    w_q, s_w = orc.quantize(w, orc.SR, seed=3, stream=orc.SID_EW)
    f = orc.gcn_layer_fwd(g, H, W, w_q, s_w, orc.SR, seed=3)
    b = orc.gcn_layer_bwd(g, f, w_q, s_w, up, orc.SR, seed=3)
    A = to_dense(g, w.astype(np.float64))[0]  # [v, u]
    # edge weights are symmetric-normalised: 1/sqrt(d_out(u) d_in(v))
    d_in = np.diff(g.in_ptr)
    d_out = np.diff(g.out_ptr)
    assert np.allclose(A[mask(g)], (1 / np.sqrt(np.outer(d_in, d_out)))[mask(g)])
    out = A @ (H.astype(np.float64) @ W.astype(np.float64))
    dHp = A.T @ up.astype(np.float64)
    assert rel_err(f["out"], out) < 0.05
    assert rel_err(b["dHp"], dHp) < 0.05
    assert rel_err(b["dW"], H.astype(np.float64).T @ dHp) < 0.05
    assert rel_err(b["dH"], dHp @ W.astype(np.float64).T) < 0.05


# ----------------------------------------------------------------- typed-edge layers (GraphSAGE, relational GCN)
def typed_dense(tg, w):
    """A[t][v, u] = weight of the type-t edge u -> v (fp64)."""
    A = np.zeros((tg.n_types, tg.n_nodes, tg.n_nodes))
    A[tg.in_type, tg.in_dst(), tg.in_src] = np.asarray(w, np.float64).reshape(-1)
    return A


def test_typed_spmm_brute_force_and_adjoint():
    g = small_graph(23, 90, 51)
    tg, w = ti.rgcn_typed_graph(g, 3, 52)
    T, F = tg.n_types, 8
    w_q = rand_i8((tg.n_edges, 1), 53)
    Z_q = rand_i8((tg.n_nodes, T * F), 54)
    Y_q = rand_i8((tg.n_nodes, F), 55)
    _, _, acc = orc.typed_spmm_in(tg, w_q, 0.5, Z_q, 0.25, want_acc=True)
    _, _, racc = orc.typed_spmm_rev(tg, w_q, 0.5, Y_q, 0.25, want_acc=True)
    want = np.zeros((tg.n_nodes, F), np.int64)
    rwant = np.zeros((tg.n_nodes, T * F), np.int64)
    dst = tg.in_dst()
    for e in range(tg.n_edges):
        u, v, t = int(tg.in_src[e]), int(dst[e]), int(tg.in_type[e])
        for d in range(F):
            want[v, d] += int(w_q[e, 0]) * int(Z_q[u, t * F + d])
            rwant[u, t * F + d] += int(w_q[e, 0]) * int(Y_q[v, d])
    assert np.array_equal(acc, want) and np.array_equal(racc, rwant)
    # <A z, y> == <z, A^T y> exactly in integers
    assert int((acc.astype(np.int64) * Y_q).sum()) == int((racc.astype(np.int64) * Z_q).sum())
    out, am = orc.typed_spmm_in(tg, w_q, 0.5, Z_q, 0.25)
    assert np.array_equal(out, (want * 0.125).astype(np.float32)) and am == np.abs(out).max()


def test_typed_layer_with_one_type_is_the_gcn_layer():
    g = small_graph(64, 512, 56)
    K, F = 24, 16
    H, W, up = ti.normal((g.n_nodes, K), 57), ti.xavier_uniform(K, F, (K, F), 58), ti.normal((g.n_nodes, F), 59)
    w_q, s_w = orc.quantize(ti.gcn_edge_weights(g), orc.SR, seed=4, stream=orc.SID_EW)
    tg = ti.typed_graph_from_edges(g.n_nodes, 1, g.in_src, g.in_dst(), np.zeros(g.n_edges, np.int64))
    assert np.array_equal(tg.in_src, g.in_src) and np.array_equal(tg.in_ptr, g.in_ptr)
    f, ft = orc.gcn_layer_fwd(g, H, W, w_q, s_w, orc.SR, 4, 2), orc.typed_layer_fwd(tg, H, W, w_q, s_w, orc.SR, 4, 2)
    b = orc.gcn_layer_bwd(g, f, w_q, s_w, up, orc.SR, 4, 2)
    bt = orc.typed_layer_bwd(tg, ft, w_q, s_w, up, orc.SR, 4, 2)
    for a, c in ((f, ft), (b, bt)):
        assert a.keys() == c.keys()
        for k in a:
            assert np.array_equal(a[k], c[k]), k


@pytest.mark.parametrize("model", ["sage", "rgcn"])
def test_quantized_typed_layer_close_to_fp64_definition(model):
    g = small_graph(64, 600, 61)
    K, F = 32, 24
    tg, w = ti.sage_typed_graph(g) if model == "sage" else ti.rgcn_typed_graph(g, 3, 62)
    T = tg.n_types
    H = ti.normal((g.n_nodes, K), 63)
    Wc = ti.xavier_uniform(K, F, (K, T * F), 64)
    up = ti.normal((g.n_nodes, F), 65)
    w_q, s_w = orc.quantize(w, orc.SR, seed=5, stream=orc.SID_EW)
    f = orc.typed_layer_fwd(tg, H, Wc, w_q, s_w, orc.SR, seed=5)
    b = orc.typed_layer_bwd(tg, f, w_q, s_w, up, orc.SR, seed=5)
    A = typed_dense(tg, w)
    H64, W64, up64 = H.astype(np.float64), Wc.astype(np.float64), up.astype(np.float64)
    if model == "sage":
        # out = H.W_self + (row-normalised adjacency without the diagonal).H.W_neigh
        adj = (to_dense(g, np.ones((g.n_edges, 1)))[0] > 0).astype(np.float64)
        np.fill_diagonal(adj, 0.0)
        mean = adj / np.maximum(adj.sum(axis=1, keepdims=True), 1.0)
        assert np.array_equal(A[0], np.eye(g.n_nodes)) and np.allclose(A[1], mean)
    else:
        # every relation's weights of one destination sum to one (or the destination has no such edge)
        sums = A[1:].sum(axis=2)
        assert np.allclose(sums[sums > 0], 1.0) and np.array_equal(A[0], np.eye(g.n_nodes))
    out = sum(A[t] @ (H64 @ W64[:, t * F:(t + 1) * F]) for t in range(T))
    dZ = np.concatenate([A[t].T @ up64 for t in range(T)], axis=1)
    assert rel_err(f["out"], out) < 0.05
    assert rel_err(b["dHp"], dZ) < 0.05
    assert rel_err(b["dW"], H64.T @ dZ) < 0.05
    assert rel_err(b["dH"], dZ @ W64.T) < 0.05


def test_gat_layer_with_relu_output_is_relu_of_plain_layer():
    """relu_out: forward = max(0, plain output) (and its abs-max); backward = plain backward of the gradient with the
    entries zeroed where the output is not positive - the ReLU of the fp64 layer, by the chain rule."""
    g = small_graph(48, 400, 71)
    heads, dim, K = 2, 8, 12
    H = ti.normal((g.n_nodes, K), 72)
    W = ti.xavier_uniform(K, heads * dim, (K, heads * dim), 73)
    a_s = ti.xavier_uniform(heads, dim, (heads, dim), 74)
    a_d = ti.xavier_uniform(heads, dim, (heads, dim), 75)
    up = ti.normal((g.n_nodes, heads * dim), 76)
    plain = orc.gat_layer_fwd(g, H, W, a_s, a_d, 0.2, orc.SR, seed=11)
    act = orc.gat_layer_fwd(g, H, W, a_s, a_d, 0.2, orc.SR, seed=11, relu_out=True)
    assert np.array_equal(act["out"], np.where(plain["out"] > 0, plain["out"], 0).astype(np.float32))
    assert act["absmax_out"] == np.float32(max(plain["out"].max(), 0.0))
    assert (plain["out"] < 0).mean() > 0.2  # the case exercises the mask
    for k in plain:
        if k not in ("out", "absmax_out"):
            assert np.array_equal(plain[k], act[k]), k
    masked = np.where(plain["out"] > 0, up, 0).astype(np.float32)
    want = orc.gat_layer_bwd(g, plain, a_s, a_d, masked, 0.2, orc.SR, seed=11)
    got = orc.gat_layer_bwd(g, act, a_s, a_d, up, 0.2, orc.SR, seed=11, relu_out=True)
    for k in want:
        assert np.array_equal(want[k], got[k]), k
    # against the fp64 layer followed by a ReLU
    rf = gat_forward(g, H, W, a_s, a_d, 0.2)
    rb = gat_backward(g, H, W, a_s, a_d, 0.2, rf, np.where(rf["out"] > 0, up, 0.0))
    assert rel_err(act["out"], np.maximum(rf["out"], 0.0)) < 0.12
    assert rel_err(got["dW"], rb["dW"]) < 0.2 and rel_err(got["dH"], rb["dH"]) < 0.2
