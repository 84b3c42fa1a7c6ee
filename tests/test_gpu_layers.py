"""GPU parity of the whole-layer entry points (GAT and GCN, forward + backward).

Every stage is compared with the oracle primitive applied to the GPU's own inputs of that stage, so integer
results stay bit-exact all along the chain even though fp32 intermediates (S, D, alpha, dE ...) may differ from an
all-oracle run in the last bits.  The all-oracle chain is compared at the end as a whole."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import oracle as orc
import tango_inputs as ti
from gpu_util import assert_bit_exact, assert_close, dev, host


@pytest.fixture(scope="module")
def T():
    import torch

    import paper_2308_00890_amd as tango

    assert torch.cuda.is_available()
    tango.load_library()
    return tango


def gat_case(name):
    if name == "toy":  # configuration 1 exactly
        return ti.layer_inputs("toy"), 0.2
    if name == "rmat_h4":  # configuration-3 widths on a small skewed graph
        g = ti.rmat_graph(3000, 60000, seed=21)
        li = ti.layer_inputs("gat_dense", graph=g, k_in=602)
        return li, 0.2
    if name == "minibatch":  # six small sampled subgraphs handed over as one block-diagonal graph
        g = ti.minibatch_graph(6, 96, 700, seed=23)
        li = ti.layer_inputs("toy", graph=g, k_in=64)
        return li, 0.2
    if name == "rmat_h3":  # configuration-4 widths
        g = ti.rmat_graph(2000, 30000, seed=22)
        li = ti.layer_inputs("gat_products", graph=g, k_in=100)
        return li, 0.2
    raise KeyError(name)


def verify_gat_layer(o, g, feat, weight, a_src, a_dst, grad_out, slope, rounding, seed, layer_id, fused, chain=True,
                     relu_out=False, dH_keep=None):
    """Stage-by-stage check of one GAT layer's device tensors `o` (host copies) against the oracle primitives applied
    to the GPU's own inputs of each stage."""
    heads = a_src.shape[0]
    b = 16 * layer_id
    sc = lambda k: o[k][0]

    # ---- forward, stage by stage
    r = orc.qgemm(feat, weight, rounding, seed, b + orc.SID_H, b + orc.SID_W)
    assert sc("s_H") == r["s_A"] and sc("s_W") == r["s_B"]
    assert_bit_exact(o["H_q"], r["A_q"], "H_q")
    assert_bit_exact(o["W_q"], r["B_q"], "W_q")
    assert_bit_exact(o["Hp"], r["C"], "Hp")
    assert sc("absmax_Hp") == r["absmax_C"]
    assert_close(o["S"], orc.head_proj(o["Hp"], a_src), "S")
    assert_close(o["D"], orc.head_proj(o["Hp"], a_dst), "D")
    for name, src, sid, am in (("Hp_q", "Hp", orc.SID_HP, sc("absmax_Hp")), ("S_q", "S", orc.SID_S, None),
                               ("D_q", "D", orc.SID_D, None)):
        q, s = orc.quantize(o[src], rounding, seed, b + sid, am=am)
        assert_bit_exact(o[name], q, name)
        assert sc("s_" + name[:-2]) == s
    E = orc.sddmm_add(g, o["S_q"], sc("s_S"), o["D_q"], sc("s_D"), slope)
    if not fused:
        assert_bit_exact(o["E"], E, "E")
    assert_close(o["alpha"], orc.edge_softmax(g, E), "alpha")
    q, s = orc.quantize(o["alpha"], rounding, seed, b + orc.SID_ALPHA)
    if "alpha_q" in o:
        assert_bit_exact(o["alpha_q"], q, "alpha_q")
    else:  # the codes exist only inside the kernels: use the oracle's codes of the GPU's own alpha from here on
        o = dict(o, alpha_q=q)
    assert sc("s_alpha") == s
    out, am = orc.spmm_in(g, o["alpha_q"], sc("s_alpha"), o["Hp_q"], sc("s_Hp"))
    if relu_out:
        out = np.maximum(out, np.float32(0))
        am = orc.absmax(out)
    assert_bit_exact(o["out"], out, "out")
    assert sc("absmax_out") == am

    # ---- backward, stage by stage
    if relu_out:
        grad_out = np.where(o["out"] > 0, grad_out, np.float32(0)).astype(np.float32)
    q, s = orc.quantize(grad_out, rounding, seed, b + orc.SID_G)
    assert_bit_exact(o["g_q"], q, "g_q")
    assert sc("s_g") == s
    agg, _ = orc.spmm_rev(g, o["alpha_q"], sc("s_alpha"), o["g_q"], sc("s_g"))
    dalpha = orc.sddmm_dot(g, o["g_q"], sc("s_g"), o["Hp_q"], sc("s_Hp"), heads)
    dE_sm = orc.edge_softmax_bwd(g, o["alpha"], dalpha)
    if fused:  # dE is never written; dalpha is kept unless nothing at all is stored per edge
        if "dalpha" in o:
            assert_bit_exact(o["dalpha"], dalpha, "dalpha")
        _, dS, dD = orc.sddmm_add_bwd(g, o["S_q"], sc("s_S"), o["D_q"], sc("s_D"), slope, dE_sm)
    else:  # dalpha was overwritten by dE
        assert_close(o["dalpha"], dE_sm, "dE (softmax backward)")
        _, dS, dD = orc.sddmm_add_bwd(g, o["S_q"], sc("s_S"), o["D_q"], sc("s_D"), slope, o["dalpha"])
    assert_close(o["dS"], dS, "dS")
    assert_close(o["dD"], dD, "dD")
    dHp, am, da_s, da_d = orc.head_proj_bwd(o["dS"], o["dD"], a_src, a_dst, o["Hp_q"], sc("s_Hp"), agg)
    assert_bit_exact(o["dHp"], dHp, "dHp")
    assert sc("absmax_dHp") == am
    assert_close(o["da_src"], da_s, "da_src")
    assert_close(o["da_dst"], da_d, "da_dst")
    rb = orc.qgemm_bwd(o["H_q"], sc("s_H"), o["W_q"], sc("s_W"), o["dHp"], rounding, seed, b + orc.SID_DHP, am=am)
    assert_bit_exact(o["dHp_q"], rb["dC_q"], "dHp_q")
    assert sc("s_dHp") == rb["s_dC"]
    assert_bit_exact(o["dW"], rb["dB"], "dW")
    if dH_keep is None:
        assert_bit_exact(o["dH"], rb["dA"], "dH")
    else:  # the ReLU' of the layer below was applied on dH's way out of the GEMM
        want = np.where(dH_keep, rb["dA"], np.float32(0)).astype(np.float32)
        assert_bit_exact(o["dH"], want, "dH behind the lower layer's ReLU'")
        assert o["absmax_dH"][0] == orc.absmax(want)

    if not chain:
        return
    # ---- the all-oracle chain, as a whole: int8 codes may flip where an fp32 intermediate sits on a rounding
    # threshold, so this is a closeness check in norm plus a count of differing codes
    assert not relu_out  # (grad_out was masked with the GPU's own output above)
    f = orc.gat_layer_fwd(g, feat, weight, a_src, a_dst, slope, rounding, seed, layer_id)
    bw = orc.gat_layer_bwd(g, f, a_src, a_dst, grad_out, slope, rounding, seed, layer_id)
    rel = lambda a, c: np.linalg.norm(a.astype(np.float64) - c) / max(np.linalg.norm(c), 1e-30)
    for name, ref in (("out", f["out"]), ("dW", bw["dW"]), ("dH", bw["dH"]), ("da_src", bw["da_src"])):
        assert rel(o[name], ref) < 2e-2, name
    for name, ref in (("S_q", f["S_q"]), ("D_q", f["D_q"]), ("alpha_q", f["alpha_q"])):
        diff = o[name].astype(np.int32) - ref.astype(np.int32)
        assert np.abs(diff).max() <= 1 and (diff != 0).mean() < 1e-2, name


@pytest.mark.parametrize("case", ["toy", "rmat_h4", "rmat_h3", "minibatch"])
@pytest.mark.parametrize("rounding", [orc.SR, orc.RN])
@pytest.mark.parametrize("mode", ["fused, nothing stored per edge", "fused, edge caches kept", "primitive by primitive"])
def test_gat_layer_stagewise(T, case, rounding, mode):
    """Three ways through the layer: the production launch (what bench.py times: neither alpha_q nor dalpha exist, the
    backward pass recomputes the codes and forms the edge sums in two fused walks; alpha is dumped for this check only),
    the fused entry points with cached alpha_q and a stored dalpha, and the chain of primitives."""
    import torch

    li, slope = gat_case(case)
    g = li.graph
    seed, layer_id = li.sr_seed, 2
    G = T.Graph.from_host(g)
    fused = mode != "primitive by primitive"
    cached = mode != "fused, nothing stored per edge"
    L = T.GatLayer(G, dev(li.feat), dev(li.weight), dev(li.a_src), dev(li.a_dst), dev(li.grad_out), slope, rounding, seed,
                   layer_id, alias_E_alpha=False, fused=fused, keep_alpha=True, keep_alpha_q=cached, keep_dalpha=cached)
    assert cached or ("alpha_q" not in L.t and "dalpha" not in L.t)
    T.tango_gat_layer_fwd(L)
    T.tango_gat_layer_bwd(L)
    torch.cuda.synchronize()
    o = {k: host(v) for k, v in L.t.items() if k != "ws"}
    verify_gat_layer(o, g, li.feat, li.weight, li.a_src, li.a_dst, li.grad_out, slope, rounding, seed, layer_id, fused)


def test_three_layer_gat_chain(T):
    """Configuration-4 shape (K_in 100 -> 3 x 128 -> 3 x 128 -> 3 x 128) on a small skewed graph: three fused layers with
    ReLU between them, forward through all three and backward through all three; each layer is verified stage by
    stage on its own device inputs (the previous layer's activated output, the next layer's masked input gradient)."""
    import torch

    g = ti.rmat_graph(2500, 40000, seed=31)
    heads, dim, widths = 3, 128, [100, 384, 384]
    F = heads * dim
    seed, slope = 777, 0.2
    G = T.Graph.from_host(g)
    x0 = ti.normal((g.n_nodes, widths[0]), 32)
    up = ti.normal((g.n_nodes, F), 33)
    params = [(ti.xavier_uniform(k, F, (k, F), 40 + i), ti.xavier_uniform(heads, dim, (heads, dim), 50 + i),
               ti.xavier_uniform(heads, dim, (heads, dim), 60 + i)) for i, k in enumerate(widths)]
    feats = [dev(x0)]
    grads = [torch.empty((g.n_nodes, F), dtype=torch.float32, device="cuda:0") for _ in range(3)]
    grads[2].copy_(dev(up))
    layers = []
    for i in range(3):
        W, a_s, a_d = params[i]
        L = T.GatLayer(G, feats[i], dev(W), dev(a_s), dev(a_d), grads[i], slope, orc.SR, seed, i, fused=True, keep_alpha=True,
                       keep_alpha_q=True)
        T.tango_gat_layer_fwd(L)
        layers.append(L)
        if i < 2:
            act = torch.empty_like(L["out"])
            T.tango_relu(L["out"], act)
            feats.append(act)
    for i in (2, 1, 0):
        T.tango_gat_layer_bwd(layers[i])
        if i > 0:  # gradient w.r.t. the previous layer's pre-activation output
            T.tango_relu_bwd(layers[i - 1]["out"], layers[i]["dH"], grads[i - 1])
    torch.cuda.synchronize()
    for i in range(3):
        o = {k: host(v) for k, v in layers[i].t.items() if k != "ws"}
        W, a_s, a_d = params[i]
        feat = host(feats[i])
        gout = host(grads[i])
        if i > 0:
            prev_out = host(layers[i - 1]["out"])
            assert_bit_exact(feat, np.maximum(prev_out, 0), "relu")
        if i < 2:
            assert_bit_exact(gout, np.where(host(layers[i]["out"]) > 0, host(layers[i + 1]["dH"]), 0).astype(np.float32),
                             "relu backward")
        verify_gat_layer(o, g, feat, W, a_s, a_d, gout, slope, orc.SR, seed, i, True, chain=False)


@pytest.mark.parametrize("mode", ["fused", "fused, sign bits", "fused, sign bits, ReLU' where the gradient is produced",
                                  "primitive by primitive"])
def test_three_layer_gat_chain_activation_inside_the_layers(T, mode):
    """The same stack with the ReLU inside the layers: a layer writes max(0, aggregate) from its SPMM epilogue and
    hands its abs-max to the next layer's GEMM; the next layer's input gradient is the previous layer's grad_out, and
    ReLU' is applied while that gradient is quantized.  No activation kernel runs and no tensor sits between layers.
    With sign bits the forward epilogue also writes one bit per output element and the backward pass reads those
    instead of the fp32 output: same results, bit for bit."""
    import torch

    fused, bits = mode != "primitive by primitive", mode.startswith("fused, sign bits")
    at_producer = mode.endswith("produced")  # the upper layer's input-gradient GEMM masks dH and leaves its abs-max
    g = ti.rmat_graph(2500, 40000, seed=31)
    heads, dim, widths = 3, 128, [100, 384, 384]
    F = heads * dim
    seed, slope = 778, 0.2
    G = T.Graph.from_host(g)
    x0 = ti.normal((g.n_nodes, widths[0]), 32)
    up = ti.normal((g.n_nodes, F), 33)
    params = [(ti.xavier_uniform(k, F, (k, F), 40 + i), ti.xavier_uniform(heads, dim, (heads, dim), 50 + i),
               ti.xavier_uniform(heads, dim, (heads, dim), 60 + i)) for i, k in enumerate(widths)]
    grads = [torch.empty((g.n_nodes, F), dtype=torch.float32, device="cuda:0") for _ in range(3)]
    grads[2].copy_(dev(up))
    layers = []
    for i in range(3):
        W, a_s, a_d = params[i]
        feat = dev(x0) if i == 0 else layers[i - 1]["out"]
        L = T.GatLayer(G, feat, dev(W), dev(a_s), dev(a_d), grads[i], slope, orc.SR, seed, i, fused=fused, keep_alpha=True,
                       keep_alpha_q=True, alias_E_alpha=False, relu_out=(i < 2), relu_bits=bits,
                       absmax_H=(layers[i - 1]["absmax_out"] if i > 0 else None),
                       dH_keep_bits=(layers[i - 1]["relu_bits"] if at_producer and i > 0 else None))
        if bits and i < 2:
            L["relu_bits"].fill_(0xA5)  # stale contents must not survive the forward pass
        if i > 0:  # this layer's input gradient is the gradient behind the previous layer's ReLU
            L._bind("dH", grads[i - 1], torch.float32)
            if at_producer:
                layers[i - 1]._bind("absmax_grad_out", L["absmax_dH"], torch.float32)
        layers.append(L)
    for L in layers:
        T.tango_gat_layer_fwd(L)
    for L in reversed(layers):
        T.tango_gat_layer_bwd(L)
    torch.cuda.synchronize()
    for i in range(3):
        o = {k: host(v) for k, v in layers[i].t.items() if k not in ("ws", "absmax_H")}
        W, a_s, a_d = params[i]
        feat = x0 if i == 0 else host(layers[i - 1]["out"])
        assert i == 0 or feat.min() >= 0
        if bits and i < 2:
            got = np.unpackbits(o["relu_bits"], bitorder="little")[: g.n_nodes * F].reshape(g.n_nodes, F)
            assert_bit_exact(got, (o["out"] > 0).astype(np.uint8), "ReLU sign bits")
        keep = (host(layers[i - 1]["out"]) > 0) if at_producer and i > 0 else None
        verify_gat_layer(o, g, feat, W, a_s, a_d, host(grads[i]), slope, orc.SR, seed, i, fused, chain=False,
                         relu_out=(i < 2), dH_keep=keep)


@pytest.mark.parametrize("case", ["toy", "rmat_h4", "rmat_h3", "dense_h8", "hub_h1", "edgeless"])
def test_cached_source_codes_change_nothing(T, case):
    """With `src_codes` the first walk over the in-edges leaves S_q[src(e)] per edge and the later walks read that stream
    instead of gathering: the buffer holds exactly those codes and every output is the same bit for bit (fp32 edge sums
    included: the same values are added in the same order)."""
    import torch

    if case == "dense_h8":  # long rows (the row-by-row destination-side walk), eight heads
        g = ti.rmat_graph(600, 60000, seed=14)
        li = ti.layer_inputs("toy", graph=g, k_in=48)
        li.a_src = ti.xavier_uniform(8, 16, (8, 16), 71)
        li.a_dst = ti.xavier_uniform(8, 16, (8, 16), 72)
        li.weight = ti.xavier_uniform(48, 128, (48, 128), 73)
        li.grad_out = ti.normal((g.n_nodes, 128), 74)
        slope = 0.2
    elif case == "edgeless":  # no edge at all: every aggregate is zero, the layer must still run
        from test_gpu_graph_ops import graph

        li = ti.layer_inputs("toy", graph=graph("edgeless"), k_in=24)
        slope = 0.2
    elif case == "hub_h1":  # one head; two rows beyond the one-wave-per-row limit of the statistics pass
        from test_gpu_graph_ops import graph

        g = graph("hub")
        li = ti.layer_inputs("toy", graph=g, k_in=40)
        li.a_src = ti.xavier_uniform(1, 64, (1, 64), 75)
        li.a_dst = ti.xavier_uniform(1, 64, (1, 64), 76)
        li.weight = ti.xavier_uniform(40, 64, (40, 64), 77)
        li.grad_out = ti.normal((g.n_nodes, 64), 78)
        slope = 0.2
    else:
        li, slope = gat_case(case)
    G = T.Graph.from_host(li.graph)
    args = (G, dev(li.feat), dev(li.weight), dev(li.a_src), dev(li.a_dst), dev(li.grad_out), slope, orc.SR, li.sr_seed, 2)
    A = T.GatLayer(*args)
    B = T.GatLayer(*args, src_codes=True)
    B["src_codes"].fill_(99)
    for L in (A, B):
        T.tango_gat_layer_fwd(L)
        T.tango_gat_layer_bwd(L)
    torch.cuda.synchronize()
    assert_bit_exact(host(B["src_codes"]), host(B["S_q"])[li.graph.in_src], "S_q of every edge's source")
    if li.graph.n_edges == 0:
        assert not host(A["out"]).any() and host(A["s_alpha"])[0] == 1.0
    for name in ("out", "row_lse", "absmax_alpha", "s_alpha", "g_q", "dHp", "dS", "dD", "dW", "dH", "da_src", "da_dst"):
        assert_bit_exact(host(B[name]), host(A[name]), name)


def test_relu_sign_bits_are_ignored_for_narrow_rows(T):
    """Rows of at most 128 columns have no sign-bit path: the buffer is left alone and the results do not change."""
    import torch

    li, slope = gat_case("toy")
    G = T.Graph.from_host(li.graph)
    args = (G, dev(li.feat), dev(li.weight), dev(li.a_src), dev(li.a_dst), dev(li.grad_out), slope, orc.SR, li.sr_seed, 0)
    A = T.GatLayer(*args, relu_out=True)
    B = T.GatLayer(*args, relu_out=True, relu_bits=True)
    B["relu_bits"].fill_(0x5A)
    for L in (A, B):
        T.tango_gat_layer_fwd(L)
        T.tango_gat_layer_bwd(L)
    torch.cuda.synchronize()
    assert (host(B["relu_bits"]) == 0x5A).all()
    for name in ("out", "g_q", "dW", "dH"):
        assert_bit_exact(host(B[name]), host(A[name]), name)


def test_fused_gat_layer_without_edge_caches(T):
    """The production launch (what bench.py times) keeps neither alpha nor alpha_q: same results, bit for bit."""
    import torch

    li, slope = gat_case("rmat_h4")
    G = T.Graph.from_host(li.graph)
    args = (G, dev(li.feat), dev(li.weight), dev(li.a_src), dev(li.a_dst), dev(li.grad_out), slope, orc.SR, li.sr_seed, 1)
    A = T.GatLayer(*args, fused=True, keep_alpha=True, keep_alpha_q=True)
    B = T.GatLayer(*args, fused=True)
    for L in (A, B):
        T.tango_gat_layer_fwd(L)
        T.tango_gat_layer_bwd(L)
    torch.cuda.synchronize()
    assert "alpha_q" not in B.t and "alpha" not in B.t and "dalpha" not in B.t
    for name in ("out", "g_q"):
        assert_bit_exact(host(B[name]), host(A[name]), name)
    # the edge sums are formed in a different order (and dD as B - P*C): equal within the fp32 tolerance; what is
    # quantized from them may then differ by one code in a few places
    for name in ("dS", "dD", "dHp"):
        assert_close(host(B[name]), host(A[name]), name)
    diff = host(B["dHp_q"]).astype(np.int32) - host(A["dHp_q"]).astype(np.int32)
    assert np.abs(diff).max() <= 1 and (diff != 0).mean() < 1e-3
    rel = lambda x, y: np.linalg.norm(x.astype(np.float64) - y) / np.linalg.norm(y)
    for name in ("dW", "dH", "da_src", "da_dst"):  # sums over all nodes of the above (cancelling terms): in norm
        assert rel(host(B[name]), host(A[name]).astype(np.float64)) < 1e-3, name


@pytest.mark.parametrize("rounding", [orc.SR, orc.RN])
@pytest.mark.parametrize("src_order", [False, True])
def test_gcn_layer_stagewise(T, rounding, src_order):
    """src_order: the fixed edge weights are also handed over in source-major order (made once by
    tango_edge_to_src_order), and the backward pass's reverse SPMM reads them without the edge-id map."""
    import torch

    g = ti.rmat_graph(5000, 40000, seed=23)
    K, F = 128, 256  # configuration-2 widths
    H = ti.normal((g.n_nodes, K), 24)
    W = ti.xavier_uniform(K, F, (K, F), 25)
    up = ti.normal((g.n_nodes, F), 26)
    seed, layer_id = 99, 1
    b = 16 * layer_id
    w = ti.gcn_edge_weights(g)
    w_q, s_w = orc.quantize(w, rounding, seed, orc.SID_EW)
    G = T.Graph.from_host(g)
    from gpu_util import scalar

    w_src = None
    if src_order:
        w_src = torch.full((g.n_edges, 1), 99, dtype=torch.int8, device="cuda:0")
        T.tango_edge_to_src_order(G, 1, dev(w_q), w_src)
        torch.cuda.synchronize()
        assert_bit_exact(host(w_src), w_q[g.out_eid], "edge weights in source-major order")
    L = T.GcnLayer(G, dev(H), dev(W), dev(w_q), scalar(s_w), dev(up), rounding, seed, layer_id, w_q_src_order=w_src)
    T.tango_gcn_layer_fwd(L)
    T.tango_gcn_layer_bwd(L)
    torch.cuda.synchronize()
    o = {k: host(v) for k, v in L.t.items() if k not in ("ws", "w_q_src_order")}
    f = orc.gcn_layer_fwd(g, H, W, w_q, s_w, rounding, seed, layer_id)
    bw = orc.gcn_layer_bwd(g, f, w_q, s_w, up, rounding, seed, layer_id)
    # every stage is integer-exact given bit-identical inputs, so the whole chain is bit-exact
    for name in ("H_q", "W_q", "Hp", "Hp_q", "out"):
        assert_bit_exact(o[name], f[name], name)
    for name in ("g_q", "dHp", "dHp_q", "dW", "dH"):
        assert_bit_exact(o[name], bw[name], name)
    for name, ref in (("s_H", f["s_H"]), ("s_W", f["s_W"]), ("s_Hp", f["s_Hp"]), ("absmax_out", f["absmax_out"]),
                      ("s_g", bw["s_g"]), ("absmax_dHp", bw["absmax_dHp"]), ("s_dHp", bw["s_dHp"])):
        assert o[name][0] == ref, name


@pytest.mark.parametrize("model,rounding", [("sage", orc.SR), ("rgcn", orc.SR), ("rgcn", orc.RN), ("one_type", orc.SR)])
def test_typed_layer_stagewise(T, model, rounding):
    """GraphSAGE (mean) and relational GCN through the typed-edge GEMM + SPMM layer: every stage is integer-exact
    given bit-identical inputs, so the whole chain is bit-exact."""
    import torch

    from gpu_util import scalar

    g = ti.rmat_graph(4000, 36000, seed=31)
    K, F = 100, 64
    if model == "sage":
        tg, w = ti.sage_typed_graph(g)
    elif model == "rgcn":
        tg, w = ti.rgcn_typed_graph(g, 3, 32)
    else:
        tg = ti.typed_graph_from_edges(g.n_nodes, 1, g.in_src, g.in_dst(), np.zeros(g.n_edges, np.int64))
        w = ti.gcn_edge_weights(g)
    nt = tg.n_types
    H = ti.normal((g.n_nodes, K), 33)
    W = ti.xavier_uniform(K, F, (K, nt * F), 34)
    up = ti.normal((g.n_nodes, F), 35)
    seed, layer_id = 77, 2
    w_q, s_w = orc.quantize(w, rounding, seed, orc.SID_EW)
    G_dst, G_src = T.Graph.from_host(tg.dst_view()), T.Graph.from_host(tg.src_view())
    w_src = None
    if model == "rgcn":  # also with the weights handed over in the source view's order
        w_src = torch.empty((tg.n_edges, 1), dtype=torch.int8, device="cuda:0")
        T.tango_edge_to_src_order(G_src, 1, dev(w_q), w_src)
    L = T.TypedLayer(G_dst, G_src, nt, dev(H), dev(W), dev(w_q), scalar(s_w), dev(up), rounding, seed, layer_id,
                     w_q_src_order=w_src)
    T.tango_typed_layer_fwd(L)
    T.tango_typed_layer_bwd(L)
    torch.cuda.synchronize()
    o = {k: host(v) for k, v in L.t.items() if k not in ("ws", "w_q_src_order")}
    f = orc.typed_layer_fwd(tg, H, W, w_q, s_w, rounding, seed, layer_id)
    bw = orc.typed_layer_bwd(tg, f, w_q, s_w, up, rounding, seed, layer_id)
    for name in ("H_q", "W_q", "Hp", "Hp_q", "out"):
        assert_bit_exact(o[name], f[name], name)
    for name in ("g_q", "dHp", "dHp_q", "dW", "dH"):
        assert_bit_exact(o[name], bw[name], name)
    for name, ref in (("s_H", f["s_H"]), ("s_W", f["s_W"]), ("s_Hp", f["s_Hp"]), ("absmax_out", f["absmax_out"]),
                      ("s_g", bw["s_g"]), ("absmax_dHp", bw["absmax_dHp"]), ("s_dHp", bw["s_dHp"])):
        assert o[name][0] == ref, name


def test_typed_layer_rejects_mismatched_views(T):
    import torch

    from gpu_util import scalar

    g = ti.rmat_graph(300, 2000, seed=36)
    tg, w = ti.sage_typed_graph(g)
    K, F = 16, 8
    H, W, up = ti.normal((g.n_nodes, K), 37), ti.normal((K, 2 * F), 38), ti.normal((g.n_nodes, F), 39)
    w_q, s_w = orc.quantize(w, orc.RN, 0, orc.SID_EW)
    G_dst = T.Graph.from_host(tg.dst_view())
    G_bad = T.Graph.from_host(g)  # n rows instead of n * n_types
    L = T.TypedLayer(G_dst, G_bad, 2, dev(H), dev(W), dev(w_q), scalar(s_w), dev(up), orc.RN, 0, 0)
    T.tango_typed_layer_fwd(L)
    with pytest.raises(T.TangoError):
        T.tango_typed_layer_bwd(L)
    L2 = T.TypedLayer(G_dst, None, 2, dev(H), dev(W), dev(w_q), scalar(s_w), dev(up), orc.RN, 0, 0)
    with pytest.raises(T.TangoError):
        T.tango_typed_layer_bwd(L2)
    torch.cuda.synchronize()
