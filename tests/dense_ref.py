"""Dense-matrix (numpy, fp64/int64) formulations of the layer's steps, for pinning the oracle on tiny graphs.

Everything here works on the dense adjacency mask G[v, u] = 1 iff there is an edge u -> v, exactly as the
paper writes the primitives (Sec. 2.1): SDDMM = G (.) (S (+) D^T), SPMM = (G (.) alpha) . H', etc.
Edge tensors are converted with ``to_dense`` / ``from_dense`` using the destination-major edge positions.
"""
import numpy as np


def mask(g):
    G = np.zeros((g.n_nodes, g.n_nodes), dtype=bool)
    G[g.in_dst(), g.in_src] = True
    return G


def to_dense(g, edge_vals):
    """edge_vals (nnz, heads) -> (heads, N_dst, N_src)"""
    edge_vals = np.asarray(edge_vals)
    heads = edge_vals.shape[1]
    out = np.zeros((heads, g.n_nodes, g.n_nodes), dtype=edge_vals.dtype)
    out[:, g.in_dst(), g.in_src] = edge_vals.T
    return out


def from_dense(g, dense):
    """(heads, N_dst, N_src) -> (nnz, heads)"""
    return np.ascontiguousarray(dense[:, g.in_dst(), g.in_src].T)


def lrelu(x, slope):
    return np.where(x > 0, x, slope * x)


def gat_forward(g, H, W, a_src, a_dst, slope):
    """Unquantized fp64 GAT layer (Fig. 1a). Returns dict of dense intermediates."""
    H = H.astype(np.float64)
    W = W.astype(np.float64)
    heads, dim = a_src.shape
    N = g.n_nodes
    G = mask(g)
    Hp = H @ W
    Hp3 = Hp.reshape(N, heads, dim)
    S = np.einsum("vhd,hd->vh", Hp3, a_src.astype(np.float64))
    D = np.einsum("vhd,hd->vh", Hp3, a_dst.astype(np.float64))
    # T[h, v, u] = S[u, h] + D[v, h]
    T = S.T[:, None, :] + D.T[:, :, None]
    E = lrelu(T, slope)
    Em = np.where(G[None], E, -np.inf)
    Em = Em - Em.max(axis=2, keepdims=True)
    ex = np.where(G[None], np.exp(Em), 0.0)
    alpha = ex / ex.sum(axis=2, keepdims=True)
    out = np.einsum("hvu,uhd->vhd", alpha, Hp3).reshape(N, heads * dim)
    return dict(Hp=Hp, S=S, D=D, T=T, E=E, alpha=alpha, out=out, G=G)


def gat_backward(g, H, W, a_src, a_dst, slope, fwd, grad_out):
    """Analytic fp64 backward of gat_forward (Fig. 1b)."""
    heads, dim = a_src.shape
    N = g.n_nodes
    G = fwd["G"]
    go = grad_out.astype(np.float64).reshape(N, heads, dim)
    Hp3 = fwd["Hp"].reshape(N, heads, dim)
    alpha = fwd["alpha"]
    dHp_agg = np.einsum("hvu,vhd->uhd", alpha, go)
    dalpha = np.einsum("vhd,uhd->hvu", go, Hp3) * G[None]
    P = (dalpha * alpha).sum(axis=2, keepdims=True)
    dE_sm = alpha * (dalpha - P)
    dT = dE_sm * np.where(fwd["T"] > 0, 1.0, slope)
    dD = dT.sum(axis=2).T  # (N, heads): over sources
    dS = dT.sum(axis=1).T  # over destinations
    dHp_att = dS[:, :, None] * a_src[None].astype(np.float64) + dD[:, :, None] * a_dst[None].astype(np.float64)
    da_src = np.einsum("vh,vhd->hd", dS, Hp3)
    da_dst = np.einsum("vh,vhd->hd", dD, Hp3)
    dHp = (dHp_agg + dHp_att).reshape(N, heads * dim)
    dW = H.astype(np.float64).T @ dHp
    dH = dHp @ W.astype(np.float64).T
    return dict(dHp_agg=dHp_agg.reshape(N, -1), dalpha=dalpha, dE_sm=dE_sm, dT=dT, dS=dS, dD=dD, dHp=dHp,
                da_src=da_src, da_dst=da_dst, dW=dW, dH=dH)
