"""GPU parity of the fused attention forward against the oracle's step-by-step composition."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import oracle as orc
import tango_inputs as ti
from gpu_util import assert_bit_exact, assert_close, dev, empty, host, scalar, workspace
from test_gpu_graph_ops import graph, rand_i8


@pytest.fixture(scope="module")
def T():
    import torch

    import paper_2308_00890_amd as tango

    assert torch.cuda.is_available()
    tango.load_library()
    return tango


@pytest.mark.parametrize("gname,heads,dim", [("toy", 2, 32), ("rmat", 4, 64), ("rmat", 3, 128), ("sparse", 1, 64),
                                             ("sparse", 8, 16), ("holes", 2, 32), ("one", 4, 64),
                                             ("dense", 4, 64), ("dense", 3, 128), ("dense", 8, 16), ("dense", 1, 32),
                                             ("sparse", 2, 128), ("hub", 4, 64), ("hub", 3, 128), ("hub", 1, 32),
                                             ("edgeless", 4, 64)])
@pytest.mark.parametrize("rounding", [orc.SR, orc.RN])
def test_fused_attention_forward_backward(T, gname, heads, dim, rounding):
    import torch

    g = graph(gname)
    G = T.Graph.from_host(g)
    F = heads * dim
    Sq, Dq = rand_i8((g.n_nodes, heads), 8), rand_i8((g.n_nodes, heads), 9)
    Xq = rand_i8((g.n_nodes, F), 10)
    sS, sD, sX, slope = np.float32(0.021), np.float32(0.013), np.float32(0.017), 0.2
    seed, sid = 4242, 38
    row_lse = empty((g.n_nodes, heads), torch.float32)
    am_alpha = scalar(-1)
    alpha_q = empty((g.n_edges, heads), torch.int8)
    dump = empty((g.n_edges, heads), torch.float32)
    s_alpha, am = scalar(-1), scalar(-1)
    out = empty((g.n_nodes, F), torch.float32)
    ws = workspace(T.tango_gat_attention_workspace_bytes(g.n_nodes, g.n_edges, heads))
    T.tango_gat_attention_fwd(G, heads, dim, dev(Sq), scalar(sS), dev(Dq), scalar(sD), slope, dev(Xq), scalar(sX), rounding,
                              seed, sid, row_lse, alpha_q, s_alpha, am_alpha, dump, out, am, ws)
    torch.cuda.synchronize()
    E = orc.sddmm_add(g, Sq, sS, Dq, sD, slope)
    alpha = orc.edge_softmax(g, E)
    assert_close(host(dump), alpha, "alpha (fp32 dump)")
    # the int8 attention is the quantization of exactly those fp32 values
    q, s = orc.quantize(host(dump), rounding, seed, sid)
    assert_bit_exact(host(alpha_q), q, "alpha_q")
    if g.n_edges:
        assert host(s_alpha)[0] == s
    want, want_am = orc.spmm_in(g, host(alpha_q), host(s_alpha)[0], Xq, sX)
    assert_bit_exact(host(out), want, "out")
    assert host(am)[0] == want_am
    # row statistics: log-sum-exp of the activated scores
    nonempty = np.diff(g.in_ptr) > 0
    starts = g.in_ptr[:-1][nonempty]
    if g.n_edges:
        m = np.maximum.reduceat(E, starts, axis=0).astype(np.float64)
        den = np.add.reduceat(np.exp(E.astype(np.float64) - np.repeat(m, np.diff(g.in_ptr)[nonempty], axis=0)), starts, axis=0)
        assert_close(host(row_lse)[nonempty], m + np.log(den), "row log-sum-exp", rtol=1e-6, atol=1e-6)
        assert host(am_alpha)[0] == host(dump).max()

    # ---- backward from the caches of the fused forward
    dOq = rand_i8((g.n_nodes, F), 11)
    s_dO = np.float32(0.0041)
    dX = empty((g.n_nodes, F), torch.float32)
    dal = empty((g.n_edges, heads), torch.float32)
    dS, dD = empty((g.n_nodes, heads), torch.float32), empty((g.n_nodes, heads), torch.float32)
    amx = scalar(-1)
    wsb = workspace(T.tango_gat_attention_bwd_workspace_bytes(g.n_nodes, g.n_edges, heads))
    T.tango_gat_attention_bwd(G, heads, dim, dev(Sq), scalar(sS), dev(Dq), scalar(sD), slope, row_lse, alpha_q, s_alpha,
                              am_alpha, rounding, seed, sid, dev(Xq), scalar(sX), dev(dOq), scalar(s_dO), dX, amx, dal, dS, dD,
                              wsb)
    torch.cuda.synchronize()
    # without the cached alpha_q the reverse SPMM recomputes the same int8 codes
    dX2 = empty((g.n_nodes, F), torch.float32)
    amx2 = scalar(-1)
    T.tango_gat_attention_bwd(G, heads, dim, dev(Sq), scalar(sS), dev(Dq), scalar(sD), slope, row_lse, None, s_alpha,
                              am_alpha, rounding, seed, sid, dev(Xq), scalar(sX), dev(dOq), scalar(s_dO), dX2, amx2,
                              empty((g.n_edges, heads), torch.float32), empty((g.n_nodes, heads), torch.float32),
                              empty((g.n_nodes, heads), torch.float32), wsb)
    torch.cuda.synchronize()
    assert_bit_exact(host(dX2), host(dX), "dX_agg with recomputed attention codes")
    assert host(amx2)[0] == host(amx)[0]
    w_dX, w_am = orc.spmm_rev(g, host(alpha_q), host(s_alpha)[0], dOq, s_dO)
    assert_bit_exact(host(dX), w_dX, "dX_agg")
    assert host(amx)[0] == w_am
    w_dal = orc.sddmm_dot(g, dOq, s_dO, Xq, sX, heads)
    assert_bit_exact(host(dal), w_dal, "dalpha")
    # the backward recomputes exactly the fp32 alpha the forward dumped
    dE_sm = orc.edge_softmax_bwd(g, host(dump), w_dal)
    _, w_dS, w_dD = orc.sddmm_add_bwd(g, Sq, sS, Dq, sD, slope, dE_sm)
    assert_close(host(dD), w_dD, "dD")
    assert_close(host(dS), w_dS, "dS")

    # ---- no edge tensor at all (dalpha = None): two fused walks; and the same as its two halves called separately
    dX3, dS3, dD3 = empty((g.n_nodes, F), torch.float32), empty((g.n_nodes, heads), torch.float32), empty((g.n_nodes, heads), torch.float32)
    for t in (dX3, dS3, dD3):
        t.fill_(float("nan"))
    amx3 = scalar(-1)
    T.tango_gat_attention_bwd(G, heads, dim, dev(Sq), scalar(sS), dev(Dq), scalar(sD), slope, row_lse, None, s_alpha,
                              am_alpha, rounding, seed, sid, dev(Xq), scalar(sX), dev(dOq), scalar(s_dO), dX3, amx3, None, dS3, dD3,
                              wsb)
    torch.cuda.synchronize()
    assert_bit_exact(host(dX3), w_dX, "dX_agg (no edge tensor)")
    assert host(amx3)[0] == w_am
    assert_close(host(dD3), w_dD, "dD (no edge tensor)")
    assert_close(host(dS3), w_dS, "dS (no edge tensor)")
    rec = workspace(T.tango_gat_attention_bwd_rec_bytes(g.n_nodes, heads))
    dX4, dS4, dD4 = empty((g.n_nodes, F), torch.float32), empty((g.n_nodes, heads), torch.float32), empty((g.n_nodes, heads), torch.float32)
    T.tango_gat_attention_bwd_dst(G, heads, dim, dev(Sq), scalar(sS), dev(Dq), scalar(sD), slope, row_lse, dev(Xq), scalar(sX),
                                  dev(dOq), scalar(s_dO), rec, dD4, workspace(T.tango_gat_attention_bwd_dst_workspace_bytes(g.n_nodes, heads)))
    T.tango_gat_attention_bwd_src(G, heads, dim, dev(Sq), scalar(sS), dev(Dq), scalar(sD), slope, row_lse, s_alpha, am_alpha,
                                  rounding, seed, sid, dev(Xq), scalar(sX), dev(dOq), scalar(s_dO), rec, dX4, None, dS4,
                                  workspace(T.tango_gat_attention_bwd_src_workspace_bytes(g.n_nodes, heads)))
    torch.cuda.synchronize()
    assert_bit_exact(host(dX4), w_dX, "dX_agg (halves)")
    assert_close(host(dD4), w_dD, "dD (halves)")
    assert_close(host(dS4), w_dS, "dS (halves)")
