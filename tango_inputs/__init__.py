"""Seeded synthetic inputs for the quantized GNN-layer primitives.

This package only *generates inputs* (graphs, feature matrices, weights,
upstream gradients).  It contains none of the method's arithmetic and is the
one module that both the CPU oracle's tests and the GPU path's tests/bench may
share.  Everything is a pure function of its seed.

Graphs are returned as a ``Graph`` of int32 numpy arrays:

* ``in_ptr[N+1]``, ``in_src[nnz]``   destination-major (CSC): in-edges of v are
  positions ``in_ptr[v] .. in_ptr[v+1]-1``; edge tensors are indexed by this
  position.
* ``out_ptr[N+1]``, ``out_dst[nnz]``, ``out_eid[nnz]``  source-major (CSR) view
  of the same edges; ``out_eid[j]`` is the destination-major position of
  out-edge ``j``.

The graphs are simple (no duplicate edges) and every node has a self-loop
(the paper's preprocessing adds self-connections, Sec. 4.1 "Datasets").
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gen.c")
_LIB = os.path.join(_HERE, "libtango_inputs.so")
_lib = None

BASE_SEED = 2308008900


def build(force: bool = False) -> str:
    """Compile gen.c with gcc (host code only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-std=c11", "-o", tmp, _SRC]
        )
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.ti_rmat_keys.restype = None
        _lib.ti_unique_sorted.restype = ctypes.c_int64
        _lib.ti_select.restype = None
        _lib.ti_csc_from_sorted_keys.restype = None
        _lib.ti_csr_from_csc.restype = None
    return _lib


def _p(a: np.ndarray):
    return ctypes.c_void_p(a.ctypes.data)


@dataclass
class Graph:
    n_nodes: int
    n_edges: int
    in_ptr: np.ndarray
    in_src: np.ndarray
    out_ptr: np.ndarray
    out_dst: np.ndarray
    out_eid: np.ndarray

    def in_dst(self) -> np.ndarray:
        """Destination of every edge in destination-major order."""
        return np.repeat(np.arange(self.n_nodes, dtype=np.int32), np.diff(self.in_ptr))


def graph_from_keys(n_nodes: int, keys: np.ndarray) -> Graph:
    """``keys`` = unique ``(dst << 32) | src`` values, any order."""
    lib = _load()
    keys = np.sort(np.ascontiguousarray(keys, dtype=np.uint64))
    nnz = int(keys.shape[0])
    if nnz >= 2**31:
        raise ValueError("n_edges must be below 2^31")
    in_ptr = np.empty(n_nodes + 1, np.int32)
    in_src = np.empty(nnz, np.int32)
    lib.ti_csc_from_sorted_keys(ctypes.c_int64(n_nodes), ctypes.c_int64(nnz), _p(keys), _p(in_ptr), _p(in_src))
    del keys
    out_ptr = np.empty(n_nodes + 1, np.int32)
    out_dst = np.empty(nnz, np.int32)
    out_eid = np.empty(nnz, np.int32)
    lib.ti_csr_from_csc(
        ctypes.c_int64(n_nodes), ctypes.c_int64(nnz), _p(in_ptr), _p(in_src), _p(out_ptr), _p(out_dst), _p(out_eid)
    )
    return Graph(n_nodes, nnz, in_ptr, in_src, out_ptr, out_dst, out_eid)


def graph_from_edges(n_nodes: int, src, dst, self_loops: bool = True) -> Graph:
    """Simple graph from an explicit edge list (duplicates removed)."""
    src = np.asarray(src, dtype=np.uint64)
    dst = np.asarray(dst, dtype=np.uint64)
    keys = (dst << np.uint64(32)) | src
    if self_loops:
        ids = np.arange(n_nodes, dtype=np.uint64)
        keys = np.concatenate([keys, (ids << np.uint64(32)) | ids])
    return graph_from_keys(n_nodes, np.unique(keys))


def toy_graph(n_nodes: int = 1024, n_edges: int = 16384, seed: int = BASE_SEED + 1) -> Graph:
    """``n_edges`` distinct ordered pairs u != v, uniform, plus one self-loop per node."""
    rng = np.random.default_rng(seed)
    total = n_nodes * (n_nodes - 1)
    if n_edges > total:
        raise ValueError("too many edges for a simple graph")
    # index into the list of ordered pairs without the diagonal
    pick = rng.choice(total, size=n_edges, replace=False)
    u = pick // (n_nodes - 1)
    r = pick % (n_nodes - 1)
    v = r + (r >= u)
    return graph_from_edges(n_nodes, u, v, self_loops=True)


def batch_graphs(graphs) -> Graph:
    """Block-diagonal union of several graphs (the usual way a mini-batch of sampled subgraphs is handed to the
    primitives as one graph): node ids of graph k are shifted by the node count of graphs 0..k-1."""
    srcs, dsts, off = [], [], 0
    for g in graphs:
        srcs.append(g.in_src.astype(np.uint64) + np.uint64(off))
        dsts.append(g.in_dst().astype(np.uint64) + np.uint64(off))
        off += g.n_nodes
    return graph_from_edges(off, np.concatenate(srcs), np.concatenate(dsts), self_loops=False)


def minibatch_graph(n_graphs: int, nodes_each: int, edges_each: int, seed: int) -> Graph:
    """``n_graphs`` uniform random subgraphs (self-loops included in each), batched block-diagonally."""
    return batch_graphs([toy_graph(nodes_each, edges_each, seed + k) for k in range(n_graphs)])


def rmat_graph(
    n_nodes: int,
    n_edges: int,
    seed: int,
    a: float = 0.57,
    b: float = 0.19,
    c: float = 0.19,
    permute: bool = True,
    self_loops: bool = True,
) -> Graph:
    """R-MAT graph with exactly ``n_edges`` distinct directed edges u != v (+ self-loops).

    scale = ceil(log2 n_nodes); candidates with an endpoint >= n_nodes, self
    pairs and duplicates are dropped and more candidates are drawn until the
    count is met; the surplus of the last batch is cut by a seeded choice.
    Node ids are randomly permuted (seeded) unless ``permute`` is False.
    """
    lib = _load()
    scale = max(1, int(np.ceil(np.log2(max(n_nodes, 2)))))
    thr = np.array(
        [round(a * 65536), round((a + b) * 65536), round((a + b + c) * 65536)], dtype=np.uint32
    )
    rng = np.random.default_rng(seed)
    perm = rng.permutation(n_nodes).astype(np.int32) if permute else None
    have = np.empty(0, np.uint64)
    first = 0
    while have.shape[0] < n_edges:
        batch = 2 * (n_edges - have.shape[0]) + 1024
        keys = np.empty(have.shape[0] + batch, np.uint64)
        keys[: have.shape[0]] = have
        lib.ti_rmat_keys(
            ctypes.c_int(scale),
            ctypes.c_uint64(n_nodes),
            ctypes.c_uint64(batch),
            ctypes.c_uint64(seed),
            ctypes.c_uint64(first),
            _p(thr),
            _p(perm) if perm is not None else None,
            ctypes.c_void_p(keys.ctypes.data + 8 * have.shape[0]),
        )
        first += batch
        keys.sort()
        m = lib.ti_unique_sorted(_p(keys), ctypes.c_int64(keys.shape[0]))
        if m > n_edges:
            lib.ti_select(_p(keys), ctypes.c_int64(m), ctypes.c_int64(n_edges), ctypes.c_uint64(seed + 77))
            m = n_edges
        have = keys[:m].copy()
        del keys
    if self_loops:
        ids = np.arange(n_nodes, dtype=np.uint64)
        have = np.concatenate([have, (ids << np.uint64(32)) | ids])
    return graph_from_keys(n_nodes, have)


@dataclass
class TypedGraph:
    """Multigraph whose edges carry a type in ``0 .. n_types-1`` (relation types of a relational GCN; self / neighbour
    for GraphSAGE).  Destination-major edge order, ties by (source, type).  The source-major view has one row per
    (source, type) pair, row index ``source * n_types + type``: a layer that keeps one block of ``F`` columns per type
    in a row-major ``N x (n_types*F)`` table then sees the table as ``(N*n_types) x F`` and the typed graph as an
    ordinary bipartite graph from these rows to the N destinations."""

    n_nodes: int
    n_types: int
    n_edges: int
    in_ptr: np.ndarray  # N + 1
    in_src: np.ndarray  # nnz, source node
    in_type: np.ndarray  # nnz
    out_ptr: np.ndarray  # N * n_types + 1
    out_dst: np.ndarray  # nnz
    out_eid: np.ndarray  # nnz

    def in_dst(self) -> np.ndarray:
        return np.repeat(np.arange(self.n_nodes, dtype=np.int32), np.diff(self.in_ptr))

    def in_key(self) -> np.ndarray:
        """Row of the (source, type) pair of every edge."""
        return (self.in_src.astype(np.int64) * self.n_types + self.in_type).astype(np.int32)

    def dst_view(self) -> Graph:
        """N destination rows gathering from N*n_types table rows (forward direction only)."""
        return Graph(self.n_nodes, self.n_edges, self.in_ptr, self.in_key(), None, None, None)

    def src_view(self) -> Graph:
        """N*n_types (source, type) rows gathering from N destination rows (reverse direction only)."""
        return Graph(self.n_nodes * self.n_types, self.n_edges, None, None, self.out_ptr, self.out_dst, self.out_eid)


def typed_graph_from_edges(n_nodes: int, n_types: int, src, dst, etype) -> TypedGraph:
    """Typed multigraph from an edge list; duplicate (src, dst, type) triples are removed."""
    if n_nodes * n_types >= 2**31:
        raise ValueError("n_nodes * n_types must be below 2^31")
    key = np.asarray(src, dtype=np.uint64) * np.uint64(n_types) + np.asarray(etype, dtype=np.uint64)
    keys = np.unique((np.asarray(dst, dtype=np.uint64) << np.uint64(32)) | key)
    nnz = int(keys.shape[0])
    in_dst = (keys >> np.uint64(32)).astype(np.int64)
    in_key = (keys & np.uint64(0xFFFFFFFF)).astype(np.int64)
    in_ptr = np.zeros(n_nodes + 1, np.int64)
    np.cumsum(np.bincount(in_dst, minlength=n_nodes), out=in_ptr[1:])
    order = np.argsort(in_key, kind="stable")  # source-major, ties keep the destination order
    out_ptr = np.zeros(n_nodes * n_types + 1, np.int64)
    np.cumsum(np.bincount(in_key, minlength=n_nodes * n_types), out=out_ptr[1:])
    return TypedGraph(
        n_nodes, n_types, nnz, in_ptr.astype(np.int32), (in_key // n_types).astype(np.int32),
        (in_key % n_types).astype(np.int32), out_ptr.astype(np.int32), in_dst[order].astype(np.int32),
        order.astype(np.int32),
    )


def sage_typed_graph(g: Graph):
    """GraphSAGE with the mean aggregator as a two-type graph: type 0 = the node itself (weight 1), type 1 = its
    in-neighbours other than itself (weight 1/their number).  Returns (TypedGraph, fp32 weights nnz x 1)."""
    src, dst = g.in_src.astype(np.int64), g.in_dst().astype(np.int64)
    keep = src != dst
    ids = np.arange(g.n_nodes, dtype=np.int64)
    tg = typed_graph_from_edges(
        g.n_nodes, 2, np.concatenate([src[keep], ids]), np.concatenate([dst[keep], ids]),
        np.concatenate([np.ones(int(keep.sum()), np.int64), np.zeros(g.n_nodes, np.int64)]),
    )
    n_neigh = np.bincount(tg.in_dst()[tg.in_type == 1], minlength=g.n_nodes).astype(np.float64)
    w = np.where(tg.in_type == 0, 1.0, 1.0 / np.maximum(n_neigh[tg.in_dst()], 1.0))
    return tg, w.astype(np.float32).reshape(-1, 1)


def rgcn_typed_graph(g: Graph, n_relations: int, seed: int):
    """Relational GCN input: every non-self edge of ``g`` gets one of ``n_relations`` relation types (uniform, seeded;
    types 1..n_relations), weight 1/c with c = the number of in-edges of its destination under that relation; type 0
    is the self-connection with weight 1.  Returns (TypedGraph, fp32 weights nnz x 1)."""
    rng = np.random.default_rng(seed)
    src, dst = g.in_src.astype(np.int64), g.in_dst().astype(np.int64)
    keep = src != dst
    rel = 1 + rng.integers(0, n_relations, size=int(keep.sum()))
    ids = np.arange(g.n_nodes, dtype=np.int64)
    T = n_relations + 1
    tg = typed_graph_from_edges(
        g.n_nodes, T, np.concatenate([src[keep], ids]), np.concatenate([dst[keep], ids]),
        np.concatenate([rel, np.zeros(g.n_nodes, np.int64)]),
    )
    slot = tg.in_dst().astype(np.int64) * T + tg.in_type
    c = np.bincount(slot, minlength=g.n_nodes * T).astype(np.float64)
    w = np.where(tg.in_type == 0, 1.0, 1.0 / c[slot])
    return tg, w.astype(np.float32).reshape(-1, 1)


def normal(shape, seed: int) -> np.ndarray:
    """i.i.d. N(0,1) fp32."""
    rng = np.random.default_rng(seed)
    return rng.standard_normal(size=shape, dtype=np.float32)


def xavier_uniform(fan_in: int, fan_out: int, shape, seed: int) -> np.ndarray:
    """U(-b, b) with b = sqrt(6 / (fan_in + fan_out)), fp32."""
    rng = np.random.default_rng(seed)
    bound = np.sqrt(6.0 / (fan_in + fan_out))
    return rng.uniform(-bound, bound, size=shape).astype(np.float32)


def gcn_edge_weights(g: Graph) -> np.ndarray:
    """Fixed GCN edge weights 1/sqrt(d_out(src) * d_in(dst)), degrees counted with self-loops.

    These are *inputs* of the GCN layer's SPMM (they are not learned).
    """
    d_in = np.diff(g.in_ptr).astype(np.float64)
    d_out = np.diff(g.out_ptr).astype(np.float64)
    w = 1.0 / np.sqrt(d_out[g.in_src] * d_in[g.in_dst()])
    return w.astype(np.float32).reshape(-1, 1)


@dataclass
class LayerInputs:
    graph: Graph
    feat: np.ndarray  # N x K_in
    weight: np.ndarray  # K_in x F
    a_src: np.ndarray  # heads x dim (GAT only)
    a_dst: np.ndarray
    grad_out: np.ndarray  # N x F
    heads: int
    dim: int
    sr_seed: int


# name -> (n_nodes, directed edges without self-loops, K_in, heads, dim, kind)
CONFIGS = {
    "toy": dict(config=1, n_nodes=1024, n_edges=16384, k_in=64, heads=2, dim=32, kind="gat", graph="uniform"),
    "gcn_arxiv": dict(config=2, n_nodes=169343, n_edges=1166243, k_in=128, heads=1, dim=256, kind="gcn", graph="rmat"),
    "gat_dense": dict(config=3, n_nodes=232965, n_edges=114615892, k_in=602, heads=4, dim=64, kind="gat", graph="rmat"),
    "gat_products": dict(config=4, n_nodes=2449029, n_edges=61859140, k_in=100, heads=3, dim=128, kind="gat", graph="rmat"),
    "sweep22": dict(config=5, n_nodes=4194304, n_edges=4194304 * 15, k_in=0, heads=1, dim=0, kind="sweep", graph="rmat"),
}


def config_graph(name: str, scale_down: int = 1) -> Graph:
    """Graph of a named configuration; ``scale_down`` divides nodes and edges (same mean degree)."""
    c = CONFIGS[name]
    seed = BASE_SEED + c["config"]
    n = max(2, c["n_nodes"] // scale_down)
    m = c["n_edges"] // scale_down
    if c["graph"] == "uniform":
        return toy_graph(n, m, seed)
    return rmat_graph(n, m, seed)


def layer_inputs(name: str, scale_down: int = 1, graph: Graph | None = None, k_in: int | None = None) -> LayerInputs:
    """All tensors of one layer of a named configuration (seeds fixed per configuration)."""
    c = CONFIGS[name]
    seed = BASE_SEED + c["config"]
    g = graph if graph is not None else config_graph(name, scale_down)
    k = c["k_in"] if k_in is None else k_in
    heads, dim = c["heads"], c["dim"]
    f = heads * dim
    feat = normal((g.n_nodes, k), seed + 100)
    weight = xavier_uniform(k, f, (k, f), seed + 200)
    a_src = xavier_uniform(heads, dim, (heads, dim), seed + 201)
    a_dst = xavier_uniform(heads, dim, (heads, dim), seed + 202)
    grad = normal((g.n_nodes, f), seed + 300)
    return LayerInputs(g, feat, weight, a_src, a_dst, grad, heads, dim, seed + 400)


def stack_weights(li: LayerInputs, n_layers: int = 3):
    """Weights of ``n_layers`` stacked layers on the inputs of one configuration (configuration 4: three layers,
    K_in -> F -> F -> F): per layer a Xavier-uniform ``W`` (seeded per layer); the attention vectors of ``li`` are
    used by every layer.  Returns (list of W, list of a_src, list of a_dst)."""
    f = li.heads * li.dim
    ws = []
    for i in range(n_layers):
        k = li.feat.shape[1] if i == 0 else f
        ws.append(xavier_uniform(k, f, (k, f), li.sr_seed + 10 + i))
    return ws, [li.a_src] * n_layers, [li.a_dst] * n_layers
