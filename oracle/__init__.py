"""CPU oracle for the quantized GNN-layer primitives -- TEST INFRASTRUCTURE ONLY.

Thin numpy/ctypes front end of ``tango_oracle.c`` plus the layer-level
compositions (one GAT layer, one GCN layer and one typed-edge GEMM+SPMM layer
that covers GraphSAGE and the relational GCN, forward and backward, with the
quantized tensors cached between primitives as in Sec. 3.3 "Inter-primitive
optimization").  Only tests, the smoke check and the benchmark's CPU-baseline
leg may import this package; it shares no code with the GPU library and the
GPU library never falls back to it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tango_oracle.c")
_LIB = os.path.join(_HERE, "libtango_oracle.so")
_lib = None

RN = 0  # round to nearest, ties to even
SR = 1  # stochastic rounding

# random-stream ids of the tensors quantized in one layer (layer l uses 16*l + id)
SID_H, SID_W, SID_HP, SID_S, SID_D, SID_ALPHA, SID_G, SID_DHP, SID_EW = 1, 2, 3, 4, 5, 6, 7, 8, 9


def build(force: bool = False) -> str:
    """Compile the oracle with gcc: no fast-math, no FMA contraction."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-ffp-contract=off", "-std=c11", "-shared", "-fPIC", "-o", tmp, _SRC, "-lm"]
        )
        os.replace(tmp, _LIB)
    return _LIB


def _L():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        lib.orc_sr_bits16.restype = ctypes.c_uint32
        lib.orc_absmax.restype = ctypes.c_float
        lib.orc_igemm.restype = ctypes.c_int64
        lib.orc_dequant_i32.restype = ctypes.c_float
        lib.orc_sddmm_dot.restype = ctypes.c_int64
        lib.orc_spmm_in.restype = ctypes.c_int64
        lib.orc_spmm_rev.restype = ctypes.c_int64
        lib.orc_head_proj_bwd.restype = ctypes.c_float
        lib.orc_error_x.restype = ctypes.c_double
        lib.orc_splitmix64.restype = ctypes.c_uint64
        lib.orc_xoshiro256pp_next.restype = ctypes.c_uint64
        for name in (
            "orc_philox4x32_10",
            "orc_scale_from_absmax",
            "orc_quantize",
            "orc_dequantize",
            "orc_head_proj",
            "orc_sddmm_add",
            "orc_sddmm_add_bwd",
            "orc_edge_softmax",
            "orc_edge_softmax_bwd",
            "orc_spmm_f32",
            "orc_sddmm_dot_f32",
            "orc_quantize_bits",
            "orc_quantize_xoshiro",
            "orc_pack_int4",
            "orc_unpack_int4",
        ):
            getattr(lib, name).restype = None
        _lib = lib
    return _lib


def _p(a):
    return None if a is None else ctypes.c_void_p(a.ctypes.data)


def _c(a, dtype):
    return np.ascontiguousarray(a, dtype=dtype)


_i64 = ctypes.c_int64
_f32 = ctypes.c_float
_u64 = ctypes.c_uint64


# ----------------------------------------------------------------- RNG
def philox4x32_10(ctr, key) -> np.ndarray:
    c = _c(ctr, np.uint32)
    k = _c(key, np.uint32)
    out = np.empty(4, np.uint32)
    _L().orc_philox4x32_10(_p(c), _p(k), _p(out))
    return out


def sr_bits16(seed: int, stream: int, i: int) -> int:
    return int(_L().orc_sr_bits16(_u64(seed), _u64(stream), _u64(i)))


# ------------------------------------------------------------ quantize
def absmax(x) -> np.float32:
    x = _c(x, np.float32)
    return np.float32(_L().orc_absmax(_p(x), ctypes.c_size_t(x.size)))


def scale_from_absmax(am):
    s = _f32()
    inv = _f32()
    _L().orc_scale_from_absmax(_f32(float(am)), ctypes.byref(s), ctypes.byref(inv))
    return np.float32(s.value), np.float32(inv.value)


def quantize(x, rounding: int = SR, seed: int = 0, stream: int = 0, am=None, first: int = 0):
    """Returns (q int8 same shape, scale fp32).  ``am`` overrides the abs-max (a cached one, or that of the
    whole tensor when ``x`` is a window of it starting at flat element ``first``)."""
    x = _c(x, np.float32)
    if am is None:
        am = absmax(x)
    q = np.empty(x.shape, np.int8)
    _L().orc_quantize(_p(x), ctypes.c_size_t(x.size), _u64(first), _f32(float(am)), ctypes.c_int(rounding), _u64(seed),
                      _u64(stream), _p(q))
    return q, scale_from_absmax(am)[0]


def quantize_bits(x, bits: int, rounding: int = SR, seed: int = 0, stream: int = 0, am=None, first: int = 0):
    """B-bit quantizer: (codes int8 in +-(2^(B-1)-1), scale fp32 = absmax/qmax)."""
    x = _c(x, np.float32)
    if am is None:
        am = absmax(x)
    q = np.empty(x.shape, np.int8)
    _L().orc_quantize_bits(_p(x), ctypes.c_size_t(x.size), _u64(first), _f32(float(am)), ctypes.c_int(bits), ctypes.c_int(rounding),
                           _u64(seed), _u64(stream), _p(q))
    qmax = np.float32((1 << (bits - 1)) - 1)
    s = np.float32(am) / qmax if am > 0 else np.float32(1.0)
    return q, np.float32(s)


def pack_int4(q) -> np.ndarray:
    """Two 4-bit codes per byte along the last axis (even element in the low nibble)."""
    q = _c(q, np.int8)
    assert q.shape[-1] % 2 == 0
    p = np.empty(q.shape[:-1] + (q.shape[-1] // 2,), np.uint8)
    _L().orc_pack_int4(_p(q), ctypes.c_size_t(q.size), _p(p))
    return p


def unpack_int4(p) -> np.ndarray:
    p = _c(p, np.uint8)
    q = np.empty(p.shape[:-1] + (p.shape[-1] * 2,), np.int8)
    _L().orc_unpack_int4(_p(p), ctypes.c_size_t(q.size), _p(q))
    return q


def xoshiro256pp(state, count: int):
    """`count` outputs of xoshiro256++ from the four-word state (list of ints)."""
    st = (ctypes.c_uint64 * 4)(*state)
    return [int(_L().orc_xoshiro256pp_next(st)) for _ in range(count)]


def splitmix64(x: int, count: int):
    xs = ctypes.c_uint64(x)
    return [int(_L().orc_splitmix64(ctypes.byref(xs))) for _ in range(count)]


def quantize_xoshiro(x, seed: int = 0, stream: int = 0, am=None):
    """Stochastic-rounding quantizer with the stateful generator as the source of bits: (q int8, scale)."""
    x = _c(x, np.float32)
    if am is None:
        am = absmax(x)
    q = np.empty(x.shape, np.int8)
    _L().orc_quantize_xoshiro(_p(x), ctypes.c_size_t(x.size), _f32(float(am)), _u64(seed), _u64(stream), _p(q))
    return q, scale_from_absmax(am)[0]


def error_x(x, bits: int, rounding: int = SR, seed: int = 0, stream: int = 0) -> float:
    """Quantization-error metric of Eq. 4 for a B-bit symmetric per-tensor quantizer."""
    x = _c(x, np.float32)
    return float(_L().orc_error_x(_p(x), ctypes.c_size_t(x.size), ctypes.c_int(bits), _f32(float(absmax(x))),
                                  ctypes.c_int(rounding), _u64(seed), _u64(stream)))


def select_bits(x, candidates=(4, 6, 8), threshold: float = 0.3, rounding: int = SR, seed: int = 0, stream: int = 0):
    """Smallest candidate bit count whose Error_X is below the threshold (the largest candidate if none is);
    returns (bits, [Error_X per candidate])."""
    errs = [error_x(x, b, rounding, seed, stream) for b in candidates]
    for b, e in zip(candidates, errs):
        if e < threshold:
            return b, errs
    return candidates[-1], errs


def dequantize(q, s) -> np.ndarray:
    q = _c(q, np.int8)
    x = np.empty(q.shape, np.float32)
    _L().orc_dequantize(_p(q), ctypes.c_size_t(q.size), _f32(float(s)), _p(x))
    return x


# ---------------------------------------------------------------- GEMM
def igemm(A, B, transA: bool = False, transB: bool = False) -> np.ndarray:
    """int32 = op(A) . op(B) for int8 row-major A, B; raises if a sum leaves int32."""
    A = _c(A, np.int8)
    B = _c(B, np.int8)
    if transA:
        K, M = A.shape
        ars, acs = 1, A.shape[1]
    else:
        M, K = A.shape
        ars, acs = A.shape[1], 1
    if transB:
        N, K2 = B.shape
        brs, bcs = 1, B.shape[1]
    else:
        K2, N = B.shape
        brs, bcs = B.shape[1], 1
    assert K == K2
    acc = np.empty((M, N), np.int32)
    bad = _L().orc_igemm(_i64(M), _i64(N), _i64(K), _p(A), _i64(ars), _i64(acs), _p(B), _i64(brs), _i64(bcs), _p(acc))
    if bad:
        raise OverflowError("%d accumulators do not fit int32: the test input is out of the method's range" % bad)
    return acc


def dequant_i32(acc, sa, sb):
    """(C fp32, absmax) with C = (float)acc * (sa*sb)."""
    acc = _c(acc, np.int32)
    C = np.empty(acc.shape, np.float32)
    am = _L().orc_dequant_i32(_p(acc), ctypes.c_size_t(acc.size), _f32(float(sa)), _f32(float(sb)), _p(C))
    return C, np.float32(am)


def qgemm(A, B, rounding=SR, seed=0, sid_a=SID_H, sid_b=SID_W):
    """Forward quantized GEMM: quantize both fp32 operands, int8 GEMM, dequantize.

    Returns dict(A_q, s_A, B_q, s_B, acc, C, absmax_C).
    """
    A_q, s_A = quantize(A, rounding, seed, sid_a)
    B_q, s_B = quantize(B, rounding, seed, sid_b)
    acc = igemm(A_q, B_q)
    C, am = dequant_i32(acc, s_A, s_B)
    return dict(A_q=A_q, s_A=s_A, B_q=B_q, s_B=s_B, acc=acc, C=C, absmax_C=am)


def qgemm_bwd(A_q, s_A, B_q, s_B, dC, rounding=SR, seed=0, sid=SID_DHP, am=None):
    """Backward of C = A.B with cached quantized A, B: dA = dC_q.B_q^T, dB = A_q^T.dC_q."""
    dC_q, s_dC = quantize(dC, rounding, seed, sid, am=am)
    dA, am_dA = dequant_i32(igemm(dC_q, B_q, transB=True), s_dC, s_B)
    dB, am_dB = dequant_i32(igemm(A_q, dC_q, transA=True), s_A, s_dC)
    return dict(dC_q=dC_q, s_dC=s_dC, dA=dA, absmax_dA=am_dA, dB=dB, absmax_dB=am_dB)


# ------------------------------------------------------- graph kernels
def head_proj(X, a) -> np.ndarray:
    X = _c(X, np.float32)
    a = _c(a, np.float32)
    heads, dim = a.shape
    n = X.shape[0]
    out = np.empty((n, heads), np.float32)
    _L().orc_head_proj(_i64(n), ctypes.c_int(heads), ctypes.c_int(dim), _p(X), _p(a), _p(out))
    return out


def sddmm_add(g, S_q, s_S, D_q, s_D, slope) -> np.ndarray:
    S_q = _c(S_q, np.int8)
    D_q = _c(D_q, np.int8)
    heads = S_q.shape[1]
    E = np.empty((g.n_edges, heads), np.float32)
    _L().orc_sddmm_add(
        _i64(g.n_nodes), _p(g.in_ptr), _p(g.in_src), ctypes.c_int(heads), _p(S_q), _f32(float(s_S)), _p(D_q),
        _f32(float(s_D)), _f32(float(slope)), _p(E),
    )
    return E


def sddmm_add_bwd(g, S_q, s_S, D_q, s_D, slope, dE_post):
    """Returns (dE_pre, dS, dD)."""
    S_q = _c(S_q, np.int8)
    D_q = _c(D_q, np.int8)
    dE_post = _c(dE_post, np.float32)
    heads = S_q.shape[1]
    dE_pre = np.empty((g.n_edges, heads), np.float32)
    dS = np.empty((g.n_nodes, heads), np.float32)
    dD = np.empty((g.n_nodes, heads), np.float32)
    _L().orc_sddmm_add_bwd(
        _i64(g.n_nodes), _p(g.in_ptr), _p(g.in_src), ctypes.c_int(heads), _p(S_q), _f32(float(s_S)), _p(D_q),
        _f32(float(s_D)), _f32(float(slope)), _p(dE_post), _p(dE_pre), _p(dS), _p(dD),
    )
    return dE_pre, dS, dD


def sddmm_dot(g, Xdst_q, s_dst, Xsrc_q, s_src, heads: int, want_acc: bool = False):
    Xdst_q = _c(Xdst_q, np.int8)
    Xsrc_q = _c(Xsrc_q, np.int8)
    F = Xdst_q.shape[1]
    dim = F // heads
    out = np.empty((g.n_edges, heads), np.float32)
    acc = np.empty((g.n_edges, heads), np.int32) if want_acc else None
    bad = _L().orc_sddmm_dot(
        _i64(g.n_nodes), _p(g.in_ptr), _p(g.in_src), ctypes.c_int(heads), ctypes.c_int(dim), _p(Xdst_q),
        _f32(float(s_dst)), _p(Xsrc_q), _f32(float(s_src)), _p(out), _p(acc),
    )
    if bad:
        raise OverflowError("int32 overflow in SDDMM-dot")
    return (out, acc) if want_acc else out


def edge_softmax(g, E) -> np.ndarray:
    E = _c(E, np.float32)
    alpha = np.empty_like(E)
    _L().orc_edge_softmax(_i64(g.n_nodes), _p(g.in_ptr), ctypes.c_int(E.shape[1]), _p(E), _p(alpha))
    return alpha


def edge_softmax_bwd(g, alpha, dalpha) -> np.ndarray:
    alpha = _c(alpha, np.float32)
    dalpha = _c(dalpha, np.float32)
    dE = np.empty_like(alpha)
    _L().orc_edge_softmax_bwd(_i64(g.n_nodes), _p(g.in_ptr), ctypes.c_int(alpha.shape[1]), _p(alpha), _p(dalpha), _p(dE))
    return dE


def _spmm(fn, g, w_q, s_w, X_q, s_X, want_acc):
    w_q = _c(w_q, np.int8)
    X_q = _c(X_q, np.int8)
    heads = w_q.shape[1]
    F = X_q.shape[1]
    dim = F // heads
    out = np.empty((g.n_nodes, F), np.float32)
    acc = np.empty((g.n_nodes, F), np.int32) if want_acc else None
    am = _f32()
    bad = fn(
        _i64(g.n_nodes), _p(g.in_ptr), _p(g.in_src), ctypes.c_int(heads), ctypes.c_int(dim), _p(w_q),
        _f32(float(s_w)), _p(X_q), _f32(float(s_X)), _p(out), ctypes.byref(am), _p(acc),
    )
    if bad:
        raise OverflowError("int32 overflow in SPMM")
    return (out, np.float32(am.value), acc) if want_acc else (out, np.float32(am.value))


def spmm_in(g, w_q, s_w, X_q, s_X, want_acc: bool = False):
    """out[v] = sum over in-edges (u->v) of w[e] * X[u]; returns (out, absmax[, acc])."""
    return _spmm(_L().orc_spmm_in, g, w_q, s_w, X_q, s_X, want_acc)


def spmm_rev(g, w_q, s_w, Y_q, s_Y, want_acc: bool = False):
    """out[u] = sum over out-edges (u->v) of w[e] * Y[v]; returns (out, absmax[, acc])."""
    return _spmm(_L().orc_spmm_rev, g, w_q, s_w, Y_q, s_Y, want_acc)


def spmm_f32(g, w, X, reverse: bool = False) -> np.ndarray:
    """fp32 twin of the SPMM: out[v] = sum over in-edges of w[e]*X[src] (reverse: out[u] = sum over out-edges of w[e]*X[dst])."""
    w = _c(w, np.float32)
    X = _c(X, np.float32)
    heads = w.shape[1]
    F = X.shape[1]
    out = np.empty((g.n_nodes, F), np.float32)
    _L().orc_spmm_f32(_i64(g.n_nodes), _p(g.in_ptr), _p(g.in_src), ctypes.c_int(heads), ctypes.c_int(F // heads), _p(w), _p(X),
                      ctypes.c_int(1 if reverse else 0), _p(out))
    return out


def sddmm_dot_f32(g, X_dst, X_src, heads: int) -> np.ndarray:
    """fp32 twin of the SDDMM-dot: out[e][h] = X_dst[dst(e)][h] . X_src[src(e)][h]."""
    X_dst = _c(X_dst, np.float32)
    X_src = _c(X_src, np.float32)
    F = X_dst.shape[1]
    out = np.empty((g.n_edges, heads), np.float32)
    _L().orc_sddmm_dot_f32(_i64(g.n_nodes), _p(g.in_ptr), _p(g.in_src), ctypes.c_int(heads), ctypes.c_int(F // heads),
                           _p(X_dst), _p(X_src), _p(out))
    return out


def head_proj_bwd(dS, dD, a_src, a_dst, X_q, s_X, dX_agg):
    """Returns (dX = dX_agg + dX_att, absmax(dX), da_src, da_dst)."""
    dS = _c(dS, np.float32)
    dD = _c(dD, np.float32)
    a_src = _c(a_src, np.float32)
    a_dst = _c(a_dst, np.float32)
    X_q = _c(X_q, np.int8)
    dX_agg = _c(dX_agg, np.float32)
    heads, dim = a_src.shape
    n = X_q.shape[0]
    dX = np.empty_like(dX_agg)
    da_s = np.empty((heads, dim), np.float32)
    da_d = np.empty((heads, dim), np.float32)
    am = _L().orc_head_proj_bwd(
        _i64(n), ctypes.c_int(heads), ctypes.c_int(dim), _p(dS), _p(dD), _p(a_src), _p(a_dst), _p(X_q),
        _f32(float(s_X)), _p(dX_agg), _p(dX), _p(da_s), _p(da_d),
    )
    return dX, np.float32(am), da_s, da_d


# ------------------------------------------------------------- layers
def gat_layer_fwd(g, H, W, a_src, a_dst, slope=0.2, rounding=SR, seed=0, layer=0, relu_out=False):
    """One quantized GAT layer forward (Fig. 1a steps 1-5); returns every intermediate."""
    b = 16 * layer
    r = qgemm(H, W, rounding, seed, b + SID_H, b + SID_W)
    Hp = r["C"]
    S = head_proj(Hp, a_src)
    D = head_proj(Hp, a_dst)
    Hp_q, s_Hp = quantize(Hp, rounding, seed, b + SID_HP, am=r["absmax_C"])
    S_q, s_S = quantize(S, rounding, seed, b + SID_S)
    D_q, s_D = quantize(D, rounding, seed, b + SID_D)
    E = sddmm_add(g, S_q, s_S, D_q, s_D, slope)
    alpha = edge_softmax(g, E)
    alpha_q, s_alpha = quantize(alpha, rounding, seed, b + SID_ALPHA)
    out, am_out = spmm_in(g, alpha_q, s_alpha, Hp_q, s_Hp)
    if relu_out:  # ReLU between stacked layers (the paper leaves the activation open): out = max(0, aggregate)
        out = np.maximum(out, np.float32(0))
        am_out = absmax(out)
    return dict(
        H_q=r["A_q"], s_H=r["s_A"], W_q=r["B_q"], s_W=r["s_B"], Hp=Hp, absmax_Hp=r["absmax_C"], S=S, D=D,
        Hp_q=Hp_q, s_Hp=s_Hp, S_q=S_q, s_S=s_S, D_q=D_q, s_D=s_D, E=E, alpha=alpha, alpha_q=alpha_q,
        s_alpha=s_alpha, out=out, absmax_out=am_out,
    )


def gat_layer_bwd(g, fwd, a_src, a_dst, grad_out, slope=0.2, rounding=SR, seed=0, layer=0, relu_out=False):
    """Backward of gat_layer_fwd (Fig. 1b steps 5', 5'', 4', 3', 3'', 2', 1')."""
    b = 16 * layer
    heads = a_src.shape[0]
    if relu_out:  # grad_out is the gradient behind the ReLU: its derivative is 1 where the output is positive, else 0
        grad_out = np.where(fwd["out"] > 0, grad_out, np.float32(0)).astype(np.float32)
    g_q, s_g = quantize(grad_out, rounding, seed, b + SID_G)
    dHp_agg, _ = spmm_rev(g, fwd["alpha_q"], fwd["s_alpha"], g_q, s_g)
    dalpha = sddmm_dot(g, g_q, s_g, fwd["Hp_q"], fwd["s_Hp"], heads)
    dE_sm = edge_softmax_bwd(g, fwd["alpha"], dalpha)
    dE_pre, dS, dD = sddmm_add_bwd(g, fwd["S_q"], fwd["s_S"], fwd["D_q"], fwd["s_D"], slope, dE_sm)
    dHp, am_dHp, da_src, da_dst = head_proj_bwd(dS, dD, a_src, a_dst, fwd["Hp_q"], fwd["s_Hp"], dHp_agg)
    r = qgemm_bwd(fwd["H_q"], fwd["s_H"], fwd["W_q"], fwd["s_W"], dHp, rounding, seed, b + SID_DHP, am=am_dHp)
    return dict(
        g_q=g_q, s_g=s_g, dHp_agg=dHp_agg, dalpha=dalpha, dE_sm=dE_sm, dE=dE_pre, dS=dS, dD=dD, dHp=dHp,
        absmax_dHp=am_dHp, da_src=da_src, da_dst=da_dst, dHp_q=r["dC_q"], s_dHp=r["s_dC"], dW=r["dB"], dH=r["dA"],
    )


def gcn_layer_fwd(g, H, W, w_q, s_w, rounding=SR, seed=0, layer=0):
    """One quantized GCN layer: transform (GEMM) then aggregate (SPMM) with fixed quantized edge weights."""
    b = 16 * layer
    r = qgemm(H, W, rounding, seed, b + SID_H, b + SID_W)
    Hp_q, s_Hp = quantize(r["C"], rounding, seed, b + SID_HP, am=r["absmax_C"])
    out, am_out = spmm_in(g, w_q, s_w, Hp_q, s_Hp)
    return dict(
        H_q=r["A_q"], s_H=r["s_A"], W_q=r["B_q"], s_W=r["s_B"], Hp=r["C"], absmax_Hp=r["absmax_C"], Hp_q=Hp_q,
        s_Hp=s_Hp, out=out, absmax_out=am_out,
    )


def gcn_layer_bwd(g, fwd, w_q, s_w, grad_out, rounding=SR, seed=0, layer=0):
    b = 16 * layer
    g_q, s_g = quantize(grad_out, rounding, seed, b + SID_G)
    dHp, am_dHp = spmm_rev(g, w_q, s_w, g_q, s_g)
    r = qgemm_bwd(fwd["H_q"], fwd["s_H"], fwd["W_q"], fwd["s_W"], dHp, rounding, seed, b + SID_DHP, am=am_dHp)
    return dict(g_q=g_q, s_g=s_g, dHp=dHp, absmax_dHp=am_dHp, dHp_q=r["dC_q"], s_dHp=r["s_dC"], dW=r["dB"], dH=r["dA"])


# ------------------------------------------------ layers built from GEMM + SPMM over typed edges
# Sec. 2.2 lists GraphSAGE and the relational GCN as models made of the same GEMM and SPMM primitives and gives no
# formulas; the usual definitions are taken (the tests pin them to their dense fp64 forms, to brute force and, with
# one type, to the GCN layer above):
#   relational GCN   out[v] = H[v].W_0 + sum_r sum_{u ->_r v} (1/c_{v,r}) H[u].W_r
#   GraphSAGE (mean) out[v] = H[v].W_self + mean_{u -> v} H[u] . W_neigh
# Both are one layer over edges that carry a type t(e) and a fixed weight w(e):
#   Z = H.[W_0 | W_1 | ... | W_{T-1}]   (one quantized GEMM),   out[v] = sum_{e: u -> v} w(e) * Z[u, block t(e)].
# ``tg`` needs n_nodes, n_types, in_src, in_type, in_dst() in destination-major edge order.
def typed_spmm_in(tg, w_q, s_w, Z_q, s_Z, want_acc: bool = False):
    """out[v, :] = (s_w*s_Z) * sum over in-edges e=(u->v) of w_q[e] * Z_q[u, t(e)*F : (t(e)+1)*F]."""
    T = tg.n_types
    Zb = _c(Z_q, np.int8).reshape(tg.n_nodes, T, -1).astype(np.int64)
    acc = np.zeros((tg.n_nodes, Zb.shape[2]), np.int64)
    w = _c(w_q, np.int8).reshape(-1).astype(np.int64)
    np.add.at(acc, tg.in_dst(), w[:, None] * Zb[tg.in_src, tg.in_type])
    if np.abs(acc).max(initial=0) >= 2**31:
        raise OverflowError("int32 overflow in typed SPMM")
    out, am = dequant_i32(acc.astype(np.int32), s_w, s_Z)
    return (out, am, acc.astype(np.int32)) if want_acc else (out, am)


def typed_spmm_rev(tg, w_q, s_w, Y_q, s_Y, want_acc: bool = False):
    """dZ[u, t*F:(t+1)*F] = (s_w*s_Y) * sum over out-edges e=(u->v) of type t of w_q[e] * Y_q[v, :]."""
    T = tg.n_types
    Y = _c(Y_q, np.int8).astype(np.int64)
    acc = np.zeros((tg.n_nodes, T, Y.shape[1]), np.int64)
    w = _c(w_q, np.int8).reshape(-1).astype(np.int64)
    np.add.at(acc, (tg.in_src, tg.in_type), w[:, None] * Y[tg.in_dst()])
    if np.abs(acc).max(initial=0) >= 2**31:
        raise OverflowError("int32 overflow in typed SPMM")
    acc = acc.reshape(tg.n_nodes, -1).astype(np.int32)
    out, am = dequant_i32(acc, s_w, s_Y)
    return (out, am, acc) if want_acc else (out, am)


def typed_layer_fwd(tg, H, W_cat, w_q, s_w, rounding=SR, seed=0, layer=0):
    """Transform with all type blocks in one GEMM, quantize, aggregate over the typed edges."""
    b = 16 * layer
    r = qgemm(H, W_cat, rounding, seed, b + SID_H, b + SID_W)
    Z_q, s_Z = quantize(r["C"], rounding, seed, b + SID_HP, am=r["absmax_C"])
    out, am_out = typed_spmm_in(tg, w_q, s_w, Z_q, s_Z)
    return dict(
        H_q=r["A_q"], s_H=r["s_A"], W_q=r["B_q"], s_W=r["s_B"], Hp=r["C"], absmax_Hp=r["absmax_C"], Hp_q=Z_q,
        s_Hp=s_Z, out=out, absmax_out=am_out,
    )


def typed_layer_bwd(tg, fwd, w_q, s_w, grad_out, rounding=SR, seed=0, layer=0):
    b = 16 * layer
    g_q, s_g = quantize(grad_out, rounding, seed, b + SID_G)
    dZ, am_dZ = typed_spmm_rev(tg, w_q, s_w, g_q, s_g)
    r = qgemm_bwd(fwd["H_q"], fwd["s_H"], fwd["W_q"], fwd["s_W"], dZ, rounding, seed, b + SID_DHP, am=am_dZ)
    return dict(g_q=g_q, s_g=s_g, dHp=dZ, absmax_dHp=am_dZ, dHp_q=r["dC_q"], s_dHp=r["s_dC"], dW=r["dB"], dH=r["dA"])
