"""GPU parity of the 4-bit paths (packed quantizer, SPMM on a packed table, SDDMM-dot on packed tables) against the
CPU oracle, through the C ABI.  The oracle unpacks the nibbles and runs its int8 routines on the codes."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import oracle as orc
import tango_inputs as ti
from gpu_util import assert_bit_exact, dev, empty, host, scalar, workspace


@pytest.fixture(scope="module")
def T():
    import torch

    import paper_2308_00890_amd as tango

    assert torch.cuda.is_available()
    tango.load_library()
    return tango


@pytest.mark.parametrize("n", [8, 2, 14, 4096, 100006, 1 << 20])
@pytest.mark.parametrize("rounding", [orc.RN, orc.SR])
def test_quantize_i4(T, n, rounding):
    import torch

    x = ti.normal((n,), 700 + n)
    q4 = empty((n // 2,), torch.uint8)
    q4.fill_(0xAA)
    s = scalar(-1)
    T.tango_quantize_i4(dev(x), rounding, 2308, 5, None, q4, s, workspace(256))
    torch.cuda.synchronize()
    want_q, want_s = orc.quantize_bits(x, 4, rounding, 2308, 5)
    assert host(s)[0] == want_s
    assert_bit_exact(host(q4), orc.pack_int4(want_q), "packed codes")
    # cached abs-max
    q4b = empty((n // 2,), torch.uint8)
    T.tango_quantize_i4(dev(x), rounding, 2308, 5, scalar(orc.absmax(x)), q4b, s, None)
    torch.cuda.synchronize()
    assert_bit_exact(host(q4b), orc.pack_int4(want_q), "packed codes (cached abs-max)")


_graphs = {}


def graph(name):
    if name not in _graphs:
        _graphs[name] = {
            "toy": lambda: ti.config_graph("toy"),
            "rmat": lambda: ti.rmat_graph(20000, 400000, seed=11),
            "sparse": lambda: ti.rmat_graph(30011, 90000, seed=12),
            "holes": lambda: ti.rmat_graph(5000, 20000, seed=13, self_loops=False),
        }[name]()
    return _graphs[name]


def rand_i4(shape, seed):
    return np.random.default_rng(seed).integers(-7, 8, size=shape, dtype=np.int8)


CASES = [("toy", 2, 32), ("rmat", 4, 64), ("rmat", 1, 256), ("rmat", 3, 128), ("sparse", 1, 64), ("sparse", 1, 512),
         ("sparse", 8, 16), ("sparse", 1, 1024), ("holes", 2, 8), ("holes", 1, 128)]


@pytest.mark.parametrize("gname,heads,dim", CASES)
@pytest.mark.parametrize("direction", [0, 1])
def test_qspmm_i4(T, gname, heads, dim, direction):
    import torch

    g = graph(gname)
    G = T.Graph.from_host(g)
    F = heads * dim
    w = np.random.default_rng(1).integers(-127, 128, size=(g.n_edges, heads), dtype=np.int8)
    X = rand_i4((g.n_nodes, F), 2)
    sw, sx = np.float32(1.0 / 127), np.float32(0.31)
    out = empty((g.n_nodes, F), torch.float32)
    out.fill_(float("nan"))
    am = scalar(-1)
    T.tango_qspmm_i4(G, direction, heads, dim, dev(w), scalar(sw), dev(orc.pack_int4(X)), scalar(sx), out, am)
    torch.cuda.synchronize()
    fn = orc.spmm_in if direction == 0 else orc.spmm_rev
    want, want_am = fn(g, w, sw, X, sx)
    assert_bit_exact(host(out), want, "spmm i4 %s h%d d%d dir%d" % (gname, heads, dim, direction))
    assert host(am)[0] == want_am


@pytest.mark.parametrize("gname,heads,dim", CASES + [("sparse", 2, 1024)])
def test_qsddmm_dot_i4(T, gname, heads, dim):
    import torch

    g = graph(gname)
    G = T.Graph.from_host(g)
    F = heads * dim
    Xd, Xs = rand_i4((g.n_nodes, F), 3), rand_i4((g.n_nodes, F), 4)
    Xd[0, :], Xs[:, 0] = -7, 7  # extreme codes on a row and a column
    sd, ss = np.float32(0.11), np.float32(0.23)
    E = empty((g.n_edges, heads), torch.float32)
    E.fill_(float("nan"))
    T.tango_qsddmm_dot_i4(G, heads, dim, dev(orc.pack_int4(Xs)), scalar(ss), dev(orc.pack_int4(Xd)), scalar(sd), E)
    torch.cuda.synchronize()
    assert_bit_exact(host(E), orc.sddmm_dot(g, Xd, sd, Xs, ss, heads), "sddmm-dot i4 %s h%d d%d" % (gname, heads, dim))


def test_i4_bad_shapes(T):
    import torch

    g = graph("toy")
    G = T.Graph.from_host(g)
    with pytest.raises(T.TangoError):  # dim not a multiple of 8
        T.tango_qspmm_i4(G, 0, 2, 12, empty((g.n_edges, 2), torch.int8), scalar(1), empty((g.n_nodes, 12), torch.uint8), scalar(1),
                         empty((g.n_nodes, 24), torch.float32), None)
    with pytest.raises(T.TangoError):  # odd element count
        T.tango_quantize_i4(empty((7,), torch.float32), T.SR, 0, 0, scalar(1), empty((4,), torch.uint8), scalar(), None)
