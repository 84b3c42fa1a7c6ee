"""GPU parity of the graph primitives (SPMM both directions, SDDMM add/dot and backward, edge softmax
forward/backward) against the CPU oracle, through the C ABI, on seeded synthetic graphs that span many
chunks/tiles, contain hub rows, ragged tails and (in one case) empty rows."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import oracle as orc
import tango_inputs as ti
from gpu_util import assert_bit_exact, assert_close, dev, empty, host, scalar


@pytest.fixture(scope="module")
def T():
    import torch

    import paper_2308_00890_amd as tango

    assert torch.cuda.is_available()
    tango.load_library()
    return tango


_graphs = {}


def graph(name):
    if name not in _graphs:
        if name == "toy":
            g = ti.config_graph("toy")
        elif name == "rmat":  # skewed: hub rows cut by many chunk boundaries, many short rows
            g = ti.rmat_graph(20000, 400000, seed=11)
        elif name == "sparse":  # mean degree ~4 incl. self-loop
            g = ti.rmat_graph(30011, 90000, seed=12)
        elif name == "holes":  # no self-loops: nodes without in-edges and nodes without out-edges
            g = ti.rmat_graph(5000, 20000, seed=13, self_loops=False)
        elif name == "dense":  # mean degree ~100: the kernels that switch on the mean degree take their long-row paths
            g = ti.rmat_graph(600, 60000, seed=14)
        elif name == "hub":  # two nodes with ~6,000 in- and out-edges each (beyond the 4,096-edge limit of the one-wave-per-row
            # walks) among short rows
            n = 6000
            rng = np.random.default_rng(15)
            everyone = np.arange(n)
            src = np.concatenate([everyone, everyone, np.full(n, 5), np.full(n, 4321), rng.integers(0, n, 30000)])
            dst = np.concatenate([np.full(n, 5), np.full(n, 4321), everyone, everyone, rng.integers(0, n, 30000)])
            g = ti.graph_from_edges(n, src, dst)
        elif name == "wide":  # more than 2^19 nodes, mean degree ~4: the large-graph split of the plain SPMM (rows of up to
            # 4 or 8 edges to the tiny-row kernel, the rest to the chunked one); no self-loops, so some rows are empty
            g = ti.rmat_graph(540000, 1700000, seed=16, self_loops=False)
        elif name == "edgeless":  # nodes only
            g = ti.graph_from_edges(37, [], [], self_loops=False)
        elif name == "one":
            g = ti.graph_from_edges(1, [], [], self_loops=True)
        else:
            raise KeyError(name)
        _graphs[name] = g
    return _graphs[name]


def rand_i8(shape, seed):
    return np.random.default_rng(seed).integers(-127, 128, size=shape, dtype=np.int8)


CASES = [
    ("toy", 2, 32),
    ("rmat", 4, 64),
    ("rmat", 3, 128),
    ("rmat", 1, 256),
    ("sparse", 1, 32),
    ("sparse", 1, 64),
    ("sparse", 1, 128),
    ("sparse", 1, 512),
    ("sparse", 8, 16),
    ("holes", 2, 32),
    ("holes", 1, 1024),
    ("one", 4, 64),
    ("hub", 4, 64),
    ("hub", 3, 128),
    ("edgeless", 2, 32),
    ("wide", 1, 32),
    ("wide", 1, 128),
    ("wide", 4, 16),
    ("wide", 8, 8),
    ("wide", 2, 32),
    ("wide", 3, 128),
    ("wide", 1, 512),
]


@pytest.mark.parametrize("gname,heads,dim", CASES)
@pytest.mark.parametrize("direction", [0, 1, 2])
def test_qspmm(T, gname, heads, dim, direction):
    """direction 2 = TANGO_OUT_SRC_ORDER: the reversed graph with the weights handed over in source-major order (put
    there by tango_edge_to_src_order); the result is that of direction 1."""
    import torch

    g = graph(gname)
    G = T.Graph.from_host(g)
    F = heads * dim
    w = rand_i8((g.n_edges, heads), 1)
    X = rand_i8((g.n_nodes, F), 2)
    sw, sx = np.float32(1.0 / 127), np.float32(0.0213)
    out = empty((g.n_nodes, F), torch.float32)
    out.fill_(float("nan"))
    am = scalar(-1)
    wd = dev(w)
    if direction == 2:
        w_src = empty((g.n_edges, heads), torch.int8)
        w_src.fill_(55)
        T.tango_edge_to_src_order(G, heads, wd, w_src)
        torch.cuda.synchronize()
        assert_bit_exact(host(w_src), w[g.out_eid], "weights in source-major order")
        wd = w_src
    T.tango_qspmm(G, direction, heads, dim, wd, scalar(sw), dev(X), scalar(sx), out, am)
    torch.cuda.synchronize()
    fn = orc.spmm_in if direction == 0 else orc.spmm_rev
    want, want_am = fn(g, w, sw, X, sx)
    assert_bit_exact(host(out), want, "spmm %s h%d d%d dir%d" % (gname, heads, dim, direction))
    assert host(am)[0] == want_am


@pytest.mark.parametrize("gname,heads,dim", CASES)
def test_qsddmm_dot(T, gname, heads, dim):
    import torch

    g = graph(gname)
    G = T.Graph.from_host(g)
    F = heads * dim
    Xd = rand_i8((g.n_nodes, F), 3)
    Xs = rand_i8((g.n_nodes, F), 4)
    sd, ss = np.float32(0.011), np.float32(0.023)
    out = empty((g.n_edges, heads), torch.float32)
    out.fill_(float("nan"))
    T.tango_qsddmm(G, T.SDDMM_DOT, heads, dim, dev(Xs), scalar(ss), dev(Xd), scalar(sd), 0.0, out)
    torch.cuda.synchronize()
    want = orc.sddmm_dot(g, Xd, sd, Xs, ss, heads)
    assert_bit_exact(host(out), want, "sddmm-dot %s h%d d%d" % (gname, heads, dim))


@pytest.mark.parametrize("gname,heads,dim", [("toy", 2, 32), ("rmat", 4, 64), ("holes", 1, 128)])
def test_qspmm_bwd_is_reverse_spmm_plus_sddmm_dot(T, gname, heads, dim):
    import torch

    g = graph(gname)
    G = T.Graph.from_host(g)
    F = heads * dim
    w, X, dO = rand_i8((g.n_edges, heads), 5), rand_i8((g.n_nodes, F), 6), rand_i8((g.n_nodes, F), 7)
    sw, sx, sg = np.float32(1 / 127), np.float32(0.02), np.float32(0.003)
    dX = empty((g.n_nodes, F), torch.float32)
    dW = empty((g.n_edges, heads), torch.float32)
    am = scalar(-1)
    T.tango_qspmm_bwd(G, heads, dim, dev(w), scalar(sw), dev(X), scalar(sx), dev(dO), scalar(sg), dX, am, dW)
    torch.cuda.synchronize()
    want_dX, want_am = orc.spmm_rev(g, w, sw, dO, sg)
    want_dW = orc.sddmm_dot(g, dO, sg, X, sx, heads)
    assert_bit_exact(host(dX), want_dX, "dX")
    assert_bit_exact(host(dW), want_dW, "dW")
    assert host(am)[0] == want_am


EDGE_CASES = [("toy", 2), ("rmat", 4), ("rmat", 3), ("rmat", 1), ("sparse", 1), ("sparse", 8), ("holes", 2), ("one", 4),
              ("hub", 4), ("hub", 3), ("dense", 2), ("edgeless", 2)]


@pytest.mark.parametrize("gname,heads", EDGE_CASES)
def test_qsddmm_add_and_backward(T, gname, heads):
    import torch

    g = graph(gname)
    G = T.Graph.from_host(g)
    Sq, Dq = rand_i8((g.n_nodes, heads), 8), rand_i8((g.n_nodes, heads), 9)
    sS, sD, slope = np.float32(0.0131), np.float32(0.0077), 0.2
    E = empty((g.n_edges, heads), torch.float32)
    T.tango_qsddmm(G, T.SDDMM_ADD_LEAKYRELU, heads, 1, dev(Sq), scalar(sS), dev(Dq), scalar(sD), slope, E)
    torch.cuda.synchronize()
    assert_bit_exact(host(E), orc.sddmm_add(g, Sq, sS, Dq, sD, slope), "sddmm-add")

    dEp = ti.normal((g.n_edges, heads), 10)
    dE = empty((g.n_edges, heads), torch.float32)
    dS = empty((g.n_nodes, heads), torch.float32)
    dD = empty((g.n_nodes, heads), torch.float32)
    T.tango_qsddmm_bwd(G, heads, dev(Sq), scalar(sS), dev(Dq), scalar(sD), slope, dev(dEp), dE, dS, dD)
    torch.cuda.synchronize()
    w_dE, w_dS, w_dD = orc.sddmm_add_bwd(g, Sq, sS, Dq, sD, slope, dEp)
    assert_bit_exact(host(dE), w_dE, "dE_pre")
    assert_close(host(dS), w_dS, "dS")
    assert_close(host(dD), w_dD, "dD")


@pytest.mark.parametrize("gname,heads", EDGE_CASES)
def test_edge_softmax_forward_backward(T, gname, heads):
    import torch

    g = graph(gname)
    G = T.Graph.from_host(g)
    E = (3.0 * ti.normal((g.n_edges, heads), 20)).astype(np.float32)
    alpha = empty((g.n_edges, heads), torch.float32)
    am = scalar(-1)
    T.tango_edge_softmax(G, heads, dev(E), alpha, am)
    torch.cuda.synchronize()
    want = orc.edge_softmax(g, E)
    assert_close(host(alpha), want, "alpha")
    if g.n_edges:
        assert host(am)[0] == host(alpha).max()
        sums = np.add.reduceat(host(alpha).astype(np.float64), g.in_ptr[:-1][np.diff(g.in_ptr) > 0], axis=0)
        assert np.abs(sums - 1.0).max() < 1e-5

    dalpha = ti.normal((g.n_edges, heads), 21)
    dE = empty((g.n_edges, heads), torch.float32)
    T.tango_edge_softmax_bwd(G, heads, dev(want), dev(dalpha), dE)
    torch.cuda.synchronize()
    assert_close(host(dE), orc.edge_softmax_bwd(g, want, dalpha), "dE")


def test_unsupported_shapes_are_refused(T):
    import torch

    g = graph("toy")
    G = T.Graph.from_host(g)
    out = empty((g.n_nodes, 6), torch.float32)
    with pytest.raises(T.TangoError):  # dim not a multiple of 4
        T.tango_qspmm(G, 0, 2, 3, dev(rand_i8((g.n_edges, 2), 1)), scalar(1), dev(rand_i8((g.n_nodes, 6), 2)), scalar(1), out, None)
    with pytest.raises(T.TangoError):  # bad direction
        T.tango_qspmm(G, 7, 2, 32, dev(rand_i8((g.n_edges, 2), 1)), scalar(1), dev(rand_i8((g.n_nodes, 64), 2)), scalar(1),
                      empty((g.n_nodes, 64), torch.float32), None)


@pytest.mark.parametrize("gname,heads,dim", [("toy", 2, 32), ("rmat", 4, 64), ("rmat", 1, 256), ("sparse", 1, 32),
                                             ("sparse", 1, 128), ("sparse", 1, 512), ("holes", 2, 16), ("one", 1, 64)])
def test_fp32_twins(T, gname, heads, dim):
    """The full-precision comparison kernels against fp64-accumulating CPU versions (fp32 sums: 1e-5 relative to the
    largest term magnitude of a row, which for N(0,1) inputs and the longest rows here is covered by atol 2e-4)."""
    import torch

    g = graph(gname)
    G = T.Graph.from_host(g)
    F = heads * dim
    w = ti.normal((g.n_edges, heads), 31)
    X = ti.normal((g.n_nodes, F), 32)
    Y = ti.normal((g.n_nodes, F), 33)
    out = empty((g.n_nodes, F), torch.float32)
    out.fill_(float("nan"))
    T.tango_spmm_f32(G, T.IN, heads, dim, dev(w), dev(X), out)
    torch.cuda.synchronize()
    assert_close(host(out), orc.spmm_f32(g, w, X), "spmm f32 in", rtol=1e-5, atol=2e-4)
    T.tango_spmm_f32(G, T.OUT, heads, dim, dev(w), dev(Y), out)
    torch.cuda.synchronize()
    assert_close(host(out), orc.spmm_f32(g, w, Y, reverse=True), "spmm f32 out", rtol=1e-5, atol=2e-4)
    E = empty((g.n_edges, heads), torch.float32)
    T.tango_sddmm_dot_f32(G, heads, dim, dev(X), dev(Y), E)
    torch.cuda.synchronize()
    assert_close(host(E), orc.sddmm_dot_f32(g, Y, X, heads), "sddmm-dot f32", rtol=1e-5, atol=2e-5)
