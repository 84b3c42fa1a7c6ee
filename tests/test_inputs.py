"""Host-side checks of the seeded graph builders (no method arithmetic involved)."""
import numpy as np
import pytest

import tango_inputs as ti


def check_graph(g):
    N, nnz = g.n_nodes, g.n_edges
    assert g.in_ptr[0] == 0 and g.in_ptr[-1] == nnz and g.out_ptr[0] == 0 and g.out_ptr[-1] == nnz
    assert (np.diff(g.in_ptr) >= 1).all() and (np.diff(g.out_ptr) >= 1).all()  # the self-loop
    dst = g.in_dst().astype(np.int64)
    src = g.in_src.astype(np.int64)
    keys = dst * N + src
    assert (np.diff(keys) > 0).all()  # sorted, no duplicate edges
    assert np.isin(np.arange(N) * (N + 1), keys).all()  # every self-loop present
    # out_* is the transpose: same edges, source-major, eid maps back
    assert np.array_equal(np.sort(g.out_eid), np.arange(nnz))
    osrc = np.repeat(np.arange(N), np.diff(g.out_ptr))
    assert np.array_equal(src[g.out_eid], osrc)
    assert np.array_equal(dst[g.out_eid], g.out_dst)
    okeys = osrc.astype(np.int64) * N + g.out_dst
    assert (np.diff(okeys) > 0).all()


def test_toy_graph_shape():
    g = ti.config_graph("toy")
    assert g.n_nodes == 1024 and g.n_edges == 16384 + 1024
    check_graph(g)


def test_rmat_graph_counts_and_skew():
    g = ti.rmat_graph(5000, 60000, seed=3)
    assert g.n_edges == 65000
    check_graph(g)
    deg = np.diff(g.in_ptr)
    assert deg.max() > 20 * np.median(deg)  # power-law skew
    g2 = ti.rmat_graph(5000, 60000, seed=3)
    assert np.array_equal(g.in_src, g2.in_src) and np.array_equal(g.out_eid, g2.out_eid)
    g3 = ti.rmat_graph(5000, 60000, seed=4)
    assert not np.array_equal(g.in_src, g3.in_src)


def test_config2_graph_counts():
    g = ti.config_graph("gcn_arxiv")
    assert g.n_nodes == 169343 and g.n_edges == 1166243 + 169343
    assert np.array_equal(np.sort(g.out_eid), np.arange(g.n_edges))


def test_values_are_seeded():
    a = ti.normal((100, 8), 5)
    assert a.dtype == np.float32 and np.array_equal(a, ti.normal((100, 8), 5))
    w = ti.xavier_uniform(64, 64, (64, 64), 6)
    assert np.abs(w).max() <= np.sqrt(6 / 128)
    li = ti.layer_inputs("toy")
    assert li.feat.shape == (1024, 64) and li.weight.shape == (64, 64) and li.a_src.shape == (2, 32)


def test_batched_minibatch_graph_is_block_diagonal():
    parts = [ti.toy_graph(50 + 7 * k, 300 + 11 * k, seed=100 + k) for k in range(5)]
    g = ti.batch_graphs(parts)
    assert g.n_nodes == sum(p.n_nodes for p in parts) and g.n_edges == sum(p.n_edges for p in parts)
    off = 0
    dst = g.in_dst()
    for p in parts:
        lo, hi = g.in_ptr[off], g.in_ptr[off + p.n_nodes]
        assert hi - lo == p.n_edges
        assert np.array_equal(g.in_src[lo:hi] - off, p.in_src)  # same edges, same destination-major order, shifted ids
        assert dst[lo:hi].min() >= off and dst[lo:hi].max() < off + p.n_nodes
        assert np.array_equal(np.diff(g.out_ptr[off:off + p.n_nodes + 1]), np.diff(p.out_ptr))
        off += p.n_nodes
    assert np.array_equal(np.sort(g.out_eid), np.arange(g.n_edges))
    m = ti.minibatch_graph(3, 40, 200, seed=5)
    assert m.n_nodes == 120 and m.n_edges == 3 * 240


@pytest.mark.parametrize("kind", ["sage", "rgcn"])
def test_typed_graph_views(kind):
    g = ti.rmat_graph(400, 3000, seed=9)
    tg, w = ti.sage_typed_graph(g) if kind == "sage" else ti.rgcn_typed_graph(g, 4, 10)
    N, T, nnz = tg.n_nodes, tg.n_types, tg.n_edges
    assert nnz == g.n_edges and w.shape == (nnz, 1) and T == (2 if kind == "sage" else 5)
    assert tg.in_ptr[0] == 0 and tg.in_ptr[-1] == nnz and tg.out_ptr.shape == (N * T + 1,) and tg.out_ptr[-1] == nnz
    dst, key = tg.in_dst().astype(np.int64), tg.in_key().astype(np.int64)
    assert (np.diff(dst * N * T + key) > 0).all()  # destination-major, no duplicate (src, dst, type)
    # the same (src, dst) pairs as the untyped graph; type 0 exactly on the self-connections
    assert np.array_equal(np.sort(dst * N + tg.in_src), np.sort(g.in_dst().astype(np.int64) * N + g.in_src))
    assert np.array_equal(tg.in_type == 0, tg.in_src == dst)
    # source-major view: rows are (source, type) pairs, eid maps back
    assert np.array_equal(np.sort(tg.out_eid), np.arange(nnz))
    orow = np.repeat(np.arange(N * T), np.diff(tg.out_ptr))
    assert np.array_equal(key[tg.out_eid], orow) and np.array_equal(dst[tg.out_eid], tg.out_dst)
    # weights of one destination and type sum to one
    sums = np.bincount(dst * T + tg.in_type, weights=w.reshape(-1).astype(np.float64), minlength=N * T)
    assert np.allclose(sums[sums > 0], 1.0, atol=1e-5)
    dv, sv = tg.dst_view(), tg.src_view()
    assert dv.n_nodes == N and sv.n_nodes == N * T and np.array_equal(dv.in_src, key)
