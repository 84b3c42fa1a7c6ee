"""ctypes binding of libtango.so: argument marshalling only.

Every function has the name of the C entry point it calls (see include/tango.h) and takes torch
tensors that already live on the GPU (inputs and outputs alike); the binding extracts raw device
pointers and the current HIP stream.  There is no CPU fallback: if the library is not built, or a
tensor is not on the GPU, the call raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtango.so")

RN, SR = 0, 1
SDDMM_ADD_LEAKYRELU, SDDMM_DOT = 0, 1
IN, OUT, OUT_SRC_ORDER = 0, 1, 2

_lib = None


class TangoError(RuntimeError):
    pass


class tango_graph(ctypes.Structure):
    _fields_ = [
        ("n_nodes", ctypes.c_int32),
        ("n_edges", ctypes.c_int64),
        ("in_ptr", ctypes.c_void_p),
        ("in_src", ctypes.c_void_p),
        ("out_ptr", ctypes.c_void_p),
        ("out_dst", ctypes.c_void_p),
        ("out_eid", ctypes.c_void_p),
    ]


_vp, _sz, _i64, _u64, _int, _f32 = (
    ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int64, ctypes.c_uint64, ctypes.c_int, ctypes.c_float,
)
_gp = ctypes.POINTER(tango_graph)

# name -> (restype, argtypes); must list every symbol include/tango.h declares
SIGNATURES = {
    "tango_version": (_int, []),
    "tango_status_string": (ctypes.c_char_p, [_int]),
    "tango_absmax": (_int, [_vp, _sz, _vp, _vp]),
    "tango_quantize_workspace_bytes": (_sz, [_sz]),
    "tango_quantize": (_int, [_vp, _sz, _int, _u64, _u64, _vp, _vp, _vp, _vp, _sz, _vp]),
    "tango_dequantize": (_int, [_vp, _sz, _vp, _vp, _vp]),
    "tango_quantize_relu_bwd": (_int, [_vp, _vp, _sz, _int, _u64, _u64, _vp, _vp, _vp, _sz, _vp]),
    "tango_qgemm_workspace_bytes": (_sz, [_i64, _i64, _i64]),
    "tango_qgemm": (_int, [_i64, _i64, _i64, _vp, _vp, _int, _u64, _u64, _u64, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "tango_qgemm_static": (_int, [_i64, _i64, _i64, _vp, _vp, _int, _u64, _u64, _u64, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "tango_qgemm_i8": (_int, [_i64, _i64, _i64, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "tango_gat_attention_bwd_rec_bytes": (_sz, [_i64, _int]),
    "tango_gat_attention_bwd_dst_workspace_bytes": (_sz, [_i64, _int]),
    "tango_gat_attention_bwd_src_workspace_bytes": (_sz, [_i64, _int]),
    "tango_gat_attention_bwd_dst": (_int, [_gp, _int, _int, _vp, _vp, _vp, _vp, ctypes.c_float, _vp, _vp, _vp, _vp, _vp, _vp, _vp,
                                           _vp, _sz, _vp]),
    "tango_gat_attention_bwd_src": (_int, [_gp, _int, _int, _vp, _vp, _vp, _vp, ctypes.c_float, _vp, _vp, _vp, _int, _u64, _u64,
                                           _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "tango_quantize_xoshiro": (_int, [_vp, _sz, _u64, _u64, _vp, _vp, _vp, _vp, _sz, _vp]),
    "tango_quantize_i4": (_int, [_vp, _sz, _int, _u64, _u64, _vp, _vp, _vp, _vp, _sz, _vp]),
    "tango_qspmm_i4": (_int, [_gp, _int, _int, _int, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "tango_qsddmm_dot_i4": (_int, [_gp, _int, _int, _vp, _vp, _vp, _vp, _vp, _vp]),
    "tango_qgemm_bwd_workspace_bytes": (_sz, [_i64, _i64, _i64]),
    "tango_qgemm_bwd": (_int, [_i64, _i64, _i64, _vp, _vp, _vp, _vp, _vp, _int, _u64, _u64, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "tango_head_proj": (_int, [_i64, _int, _int, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "tango_head_proj_bwd_workspace_bytes": (_sz, [_i64, _int, _int]),
    "tango_head_proj_bwd": (_int, [_i64, _int, _int, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "tango_qsddmm": (_int, [_gp, _int, _int, _int, _vp, _vp, _vp, _vp, _f32, _vp, _vp]),
    "tango_qsddmm_bwd": (_int, [_gp, _int, _vp, _vp, _vp, _vp, _f32, _vp, _vp, _vp, _vp, _vp]),
    "tango_edge_softmax": (_int, [_gp, _int, _vp, _vp, _vp, _vp]),
    "tango_edge_softmax_bwd": (_int, [_gp, _int, _vp, _vp, _vp, _vp]),
    "tango_qspmm": (_int, [_gp, _int, _int, _int, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "tango_qspmm_bwd": (_int, [_gp, _int, _int, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "tango_edge_to_src_order": (_int, [_gp, _int, _vp, _vp, _vp]),
}


def load_library(path: str = LIB_PATH):
    """Load libtango.so; raises if it has not been built (there is no fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(path):
            raise TangoError(
                "libtango.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                "(there is no CPU fallback)"
            )
        lib = ctypes.CDLL(path)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(lib, name)  # AttributeError if a declared symbol is missing
            fn.restype = res
            fn.argtypes = args
        _lib = lib
    return _lib


def _ptr(t, dtype=None):
    if t is None:
        return None
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TangoError("expected a GPU tensor, got %r" % (type(t),))
    if not t.is_contiguous():
        raise TangoError("tensor must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise TangoError("expected dtype %s, got %s" % (dtype, t.dtype))
    return t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def _check(rc: int, what: str):
    if rc != 0:
        raise TangoError("%s failed: %s (%d)" % (what, load_library().tango_status_string(rc).decode(), rc))


class Graph:
    """Device copy of the graph index arrays + the C struct that points at them."""

    def __init__(self, n_nodes, in_ptr, in_src, out_ptr=None, out_dst=None, out_eid=None):
        self.n_nodes = int(n_nodes)
        self.n_edges = int((in_src if in_src is not None else out_dst).numel())
        self.in_ptr, self.in_src = in_ptr, in_src
        self.out_ptr, self.out_dst, self.out_eid = out_ptr, out_dst, out_eid
        self.c = tango_graph(
            self.n_nodes, self.n_edges, _ptr(in_ptr, torch.int32), _ptr(in_src, torch.int32),
            _ptr(out_ptr, torch.int32), _ptr(out_dst, torch.int32), _ptr(out_eid, torch.int32),
        )

    @classmethod
    def from_host(cls, g, device="cuda:0"):
        """``g``: object with numpy int32 arrays n_nodes, in_ptr, in_src, out_ptr, out_dst, out_eid."""
        dev = lambda a: None if a is None else torch.from_numpy(a).to(device)
        return cls(g.n_nodes, dev(g.in_ptr), dev(g.in_src), dev(g.out_ptr), dev(g.out_dst), dev(g.out_eid))

    def ref(self):
        return ctypes.byref(self.c)


# --------------------------------------------------------------------- quantization
def tango_version() -> int:
    return load_library().tango_version()


def tango_status_string(status: int) -> str:
    return load_library().tango_status_string(status).decode()


def tango_absmax(x, absmax_out):
    _check(load_library().tango_absmax(_ptr(x, torch.float32), x.numel(), _ptr(absmax_out, torch.float32), _stream()),
           "tango_absmax")


def tango_quantize_workspace_bytes(n: int) -> int:
    return load_library().tango_quantize_workspace_bytes(n)


def tango_quantize(x, rounding, seed, stream_id, absmax_in, q, scale_out, ws):
    _check(
        load_library().tango_quantize(
            _ptr(x, torch.float32), x.numel(), rounding, seed, stream_id, _ptr(absmax_in, torch.float32),
            _ptr(q, torch.int8), _ptr(scale_out, torch.float32), _ptr(ws), 0 if ws is None else ws.numel() * ws.element_size(),
            _stream(),
        ),
        "tango_quantize",
    )


def tango_dequantize(q, scale, x):
    _check(load_library().tango_dequantize(_ptr(q, torch.int8), q.numel(), _ptr(scale, torch.float32),
                                           _ptr(x, torch.float32), _stream()), "tango_dequantize")


SIGNATURES.update({
    "tango_relu": (_int, [_vp, _sz, _vp, _vp, _vp]),
    "tango_relu_bwd": (_int, [_vp, _vp, _sz, _vp, _vp]),
})


SIGNATURES.update({
    "tango_error_x_workspace_bytes": (_sz, []),
    "tango_error_x": (_int, [_vp, _sz, ctypes.POINTER(ctypes.c_int), _int, _f32, _int, _u64, _u64, _vp, _vp, _vp, _vp, _sz, _vp]),
})


def tango_quantize_relu_bwd(x, y, rounding, seed, stream_id, q, scale_out, ws):
    _check(
        load_library().tango_quantize_relu_bwd(
            _ptr(x, torch.float32), _ptr(y, torch.float32), x.numel(), rounding, seed, stream_id, _ptr(q, torch.int8),
            _ptr(scale_out, torch.float32), _ptr(ws), ws.numel() * ws.element_size(), _stream(),
        ),
        "tango_quantize_relu_bwd",
    )


def tango_error_x_workspace_bytes() -> int:
    return load_library().tango_error_x_workspace_bytes()


def tango_error_x(x, candidate_bits, threshold, rounding, seed, stream_id, absmax_in, error_out, bits_out, ws):
    cand = (ctypes.c_int * len(candidate_bits))(*candidate_bits)
    _check(
        load_library().tango_error_x(
            _ptr(x, torch.float32), x.numel(), cand, len(candidate_bits), threshold, rounding, seed, stream_id,
            _ptr(absmax_in, torch.float32), _ptr(error_out, torch.float64), _ptr(bits_out, torch.int32), _ptr(ws),
            ws.numel() * ws.element_size(), _stream(),
        ),
        "tango_error_x",
    )


def tango_relu(x, y, absmax_y=None):
    _check(load_library().tango_relu(_ptr(x, torch.float32), x.numel(), _ptr(y, torch.float32), _ptr(absmax_y, torch.float32),
                                     _stream()), "tango_relu")


def tango_relu_bwd(x, dy, dx):
    _check(load_library().tango_relu_bwd(_ptr(x, torch.float32), _ptr(dy, torch.float32), x.numel(), _ptr(dx, torch.float32),
                                         _stream()), "tango_relu_bwd")


# ----------------------------------------------------------------------------- GEMM
def tango_qgemm_workspace_bytes(M, N, K) -> int:
    return load_library().tango_qgemm_workspace_bytes(M, N, K)


def tango_qgemm(A, B, rounding, seed, sid_A, sid_B, A_q, s_A, B_q, s_B, C, absmax_C, ws):
    M, K = A.shape
    K2, N = B.shape
    if K != K2:
        raise TangoError("inner dimensions differ")
    _check(
        load_library().tango_qgemm(
            M, N, K, _ptr(A, torch.float32), _ptr(B, torch.float32), rounding, seed, sid_A, sid_B,
            _ptr(A_q, torch.int8), _ptr(s_A, torch.float32), _ptr(B_q, torch.int8), _ptr(s_B, torch.float32),
            _ptr(C, torch.float32), _ptr(absmax_C, torch.float32), _ptr(ws), ws.numel() * ws.element_size(), _stream(),
        ),
        "tango_qgemm",
    )


QGEMM_STATIC_SCRATCH_BYTES = 256 + (2 << 20)  # TANGO_QGEMM_STATIC_SCRATCH_BYTES of tango.h


def tango_qgemm_static(A, B, rounding, seed, sid_A, sid_B, A_q, s_A, B_q, s_B, C, absmax_C):
    M, K = A.shape
    K2, N = B.shape
    if K != K2:
        raise TangoError("inner dimensions differ")
    _check(
        load_library().tango_qgemm_static(
            M, N, K, _ptr(A, torch.float32), _ptr(B, torch.float32), rounding, seed, sid_A, sid_B,
            _ptr(A_q, torch.int8), _ptr(s_A, torch.float32), _ptr(B_q, torch.int8), _ptr(s_B, torch.float32),
            _ptr(C, torch.float32), _ptr(absmax_C, torch.float32), _stream(),
        ),
        "tango_qgemm_static",
    )


def tango_qgemm_i8(A_q, s_A, BT_q, s_B, C, absmax_C):
    M, K = A_q.shape
    N, K2 = BT_q.shape
    if K != K2 or tuple(C.shape) != (M, N):
        raise TangoError("shape mismatch")
    _check(
        load_library().tango_qgemm_i8(
            M, N, K, _ptr(A_q, torch.int8), _ptr(s_A, torch.float32), _ptr(BT_q, torch.int8), _ptr(s_B, torch.float32),
            _ptr(C, torch.float32), _ptr(absmax_C, torch.float32), _stream(),
        ),
        "tango_qgemm_i8",
    )


def tango_qgemm_bwd_workspace_bytes(M, N, K) -> int:
    return load_library().tango_qgemm_bwd_workspace_bytes(M, N, K)


def tango_qgemm_bwd(A_q, s_A, B_q, s_B, dC, rounding, seed, sid_dC, absmax_dC_in, dC_q, s_dC, dA, dB, ws):
    M, K = A_q.shape
    K2, N = B_q.shape
    if K != K2 or tuple(dC.shape) != (M, N):
        raise TangoError("shape mismatch")
    _check(
        load_library().tango_qgemm_bwd(
            M, N, K, _ptr(A_q, torch.int8), _ptr(s_A, torch.float32), _ptr(B_q, torch.int8), _ptr(s_B, torch.float32),
            _ptr(dC, torch.float32), rounding, seed, sid_dC, _ptr(absmax_dC_in, torch.float32), _ptr(dC_q, torch.int8),
            _ptr(s_dC, torch.float32), _ptr(dA, torch.float32), _ptr(dB, torch.float32), _ptr(ws),
            ws.numel() * ws.element_size(), _stream(),
        ),
        "tango_qgemm_bwd",
    )


# --------------------------------------------------------------------- projections
def tango_head_proj(X, a_src, a_dst, S, D, absmax_S, absmax_D):
    heads, dim = a_src.shape
    _check(
        load_library().tango_head_proj(
            X.shape[0], heads, dim, _ptr(X, torch.float32), _ptr(a_src, torch.float32), _ptr(a_dst, torch.float32),
            _ptr(S, torch.float32), _ptr(D, torch.float32), _ptr(absmax_S, torch.float32), _ptr(absmax_D, torch.float32),
            _stream(),
        ),
        "tango_head_proj",
    )


def tango_head_proj_bwd_workspace_bytes(n, heads, dim) -> int:
    return load_library().tango_head_proj_bwd_workspace_bytes(n, heads, dim)


def tango_head_proj_bwd(dS, dD, a_src, a_dst, X_q, s_X, dX_agg, dX, absmax_dX, da_src, da_dst, ws):
    heads, dim = a_src.shape
    _check(
        load_library().tango_head_proj_bwd(
            X_q.shape[0], heads, dim, _ptr(dS, torch.float32), _ptr(dD, torch.float32), _ptr(a_src, torch.float32),
            _ptr(a_dst, torch.float32), _ptr(X_q, torch.int8), _ptr(s_X, torch.float32), _ptr(dX_agg, torch.float32),
            _ptr(dX, torch.float32), _ptr(absmax_dX, torch.float32), _ptr(da_src, torch.float32),
            _ptr(da_dst, torch.float32), _ptr(ws), ws.numel() * ws.element_size(), _stream(),
        ),
        "tango_head_proj_bwd",
    )


# ---------------------------------------------------------------------- graph ops
def tango_qsddmm(g, op, heads, dim, X_src, s_src, X_dst, s_dst, slope, E):
    _check(
        load_library().tango_qsddmm(
            g.ref(), op, heads, dim, _ptr(X_src, torch.int8), _ptr(s_src, torch.float32), _ptr(X_dst, torch.int8),
            _ptr(s_dst, torch.float32), slope, _ptr(E, torch.float32), _stream(),
        ),
        "tango_qsddmm",
    )


def tango_qsddmm_bwd(g, heads, X_src, s_src, X_dst, s_dst, slope, dE, dE_pre, dS, dD):
    _check(
        load_library().tango_qsddmm_bwd(
            g.ref(), heads, _ptr(X_src, torch.int8), _ptr(s_src, torch.float32), _ptr(X_dst, torch.int8),
            _ptr(s_dst, torch.float32), slope, _ptr(dE, torch.float32), _ptr(dE_pre, torch.float32),
            _ptr(dS, torch.float32), _ptr(dD, torch.float32), _stream(),
        ),
        "tango_qsddmm_bwd",
    )


def tango_edge_softmax(g, heads, E, alpha, absmax_alpha):
    _check(load_library().tango_edge_softmax(g.ref(), heads, _ptr(E, torch.float32), _ptr(alpha, torch.float32),
                                             _ptr(absmax_alpha, torch.float32), _stream()), "tango_edge_softmax")


def tango_edge_softmax_bwd(g, heads, alpha, dalpha, dE):
    _check(load_library().tango_edge_softmax_bwd(g.ref(), heads, _ptr(alpha, torch.float32), _ptr(dalpha, torch.float32),
                                                 _ptr(dE, torch.float32), _stream()), "tango_edge_softmax_bwd")


def tango_qspmm(g, direction, heads, dim, w_q, s_w, X_q, s_X, out, absmax_out):
    _check(
        load_library().tango_qspmm(
            g.ref(), direction, heads, dim, _ptr(w_q, torch.int8), _ptr(s_w, torch.float32), _ptr(X_q, torch.int8),
            _ptr(s_X, torch.float32), _ptr(out, torch.float32), _ptr(absmax_out, torch.float32), _stream(),
        ),
        "tango_qspmm",
    )


def tango_edge_to_src_order(g, heads, w_q, w_q_src):
    _check(load_library().tango_edge_to_src_order(g.ref(), heads, _ptr(w_q, torch.int8), _ptr(w_q_src, torch.int8), _stream()),
           "tango_edge_to_src_order")


def tango_gat_attention_bwd_rec_bytes(n_nodes, heads) -> int:
    return load_library().tango_gat_attention_bwd_rec_bytes(n_nodes, heads)


def tango_gat_attention_bwd_dst_workspace_bytes(n_nodes, heads) -> int:
    return load_library().tango_gat_attention_bwd_dst_workspace_bytes(n_nodes, heads)


def tango_gat_attention_bwd_src_workspace_bytes(n_nodes, heads) -> int:
    return load_library().tango_gat_attention_bwd_src_workspace_bytes(n_nodes, heads)


def tango_gat_attention_bwd_dst(g, heads, dim, S_q, s_S, D_q, s_D, slope, row_lse, X_q, s_X, dOut_q, s_dOut, rec, dD, ws):
    f32, i8 = torch.float32, torch.int8
    _check(
        load_library().tango_gat_attention_bwd_dst(
            g.ref(), heads, dim, _ptr(S_q, i8), _ptr(s_S, f32), _ptr(D_q, i8), _ptr(s_D, f32), slope, _ptr(row_lse, f32),
            _ptr(X_q, i8), _ptr(s_X, f32), _ptr(dOut_q, i8), _ptr(s_dOut, f32), _ptr(rec), _ptr(dD, f32), _ptr(ws),
            ws.numel() * ws.element_size(), _stream(),
        ),
        "tango_gat_attention_bwd_dst",
    )


def tango_gat_attention_bwd_src(g, heads, dim, S_q, s_S, D_q, s_D, slope, row_lse, s_alpha, absmax_alpha, rounding, seed,
                                sid_alpha, X_q, s_X, dOut_q, s_dOut, rec, dX_agg, absmax_dX, dS, ws):
    f32, i8 = torch.float32, torch.int8
    _check(
        load_library().tango_gat_attention_bwd_src(
            g.ref(), heads, dim, _ptr(S_q, i8), _ptr(s_S, f32), _ptr(D_q, i8), _ptr(s_D, f32), slope, _ptr(row_lse, f32),
            _ptr(s_alpha, f32), _ptr(absmax_alpha, f32), rounding, seed, sid_alpha, _ptr(X_q, i8), _ptr(s_X, f32),
            _ptr(dOut_q, i8), _ptr(s_dOut, f32), _ptr(rec), _ptr(dX_agg, f32), _ptr(absmax_dX, f32), _ptr(dS, f32), _ptr(ws),
            ws.numel() * ws.element_size(), _stream(),
        ),
        "tango_gat_attention_bwd_src",
    )


def tango_quantize_xoshiro(x, seed, stream_id, absmax_in, q, scale_out, ws):
    _check(
        load_library().tango_quantize_xoshiro(
            _ptr(x, torch.float32), x.numel(), seed, stream_id, _ptr(absmax_in, torch.float32), _ptr(q, torch.int8),
            _ptr(scale_out, torch.float32), _ptr(ws), 0 if ws is None else ws.numel() * ws.element_size(), _stream(),
        ),
        "tango_quantize_xoshiro",
    )


def tango_quantize_i4(x, rounding, seed, stream_id, absmax_in, q4, scale_out, ws):
    _check(
        load_library().tango_quantize_i4(
            _ptr(x, torch.float32), x.numel(), rounding, seed, stream_id, _ptr(absmax_in, torch.float32), _ptr(q4, torch.uint8),
            _ptr(scale_out, torch.float32), _ptr(ws), 0 if ws is None else ws.numel() * ws.element_size(), _stream(),
        ),
        "tango_quantize_i4",
    )


def tango_qspmm_i4(g, direction, heads, dim, w_q, s_w, X_q4, s_X, out, absmax_out):
    _check(
        load_library().tango_qspmm_i4(
            g.ref(), direction, heads, dim, _ptr(w_q, torch.int8), _ptr(s_w, torch.float32), _ptr(X_q4, torch.uint8),
            _ptr(s_X, torch.float32), _ptr(out, torch.float32), _ptr(absmax_out, torch.float32), _stream(),
        ),
        "tango_qspmm_i4",
    )


def tango_qsddmm_dot_i4(g, heads, dim, X_src4, s_src, X_dst4, s_dst, E):
    _check(
        load_library().tango_qsddmm_dot_i4(
            g.ref(), heads, dim, _ptr(X_src4, torch.uint8), _ptr(s_src, torch.float32), _ptr(X_dst4, torch.uint8),
            _ptr(s_dst, torch.float32), _ptr(E, torch.float32), _stream(),
        ),
        "tango_qsddmm_dot_i4",
    )


def tango_qspmm_bwd(g, heads, dim, w_q, s_w, X_q, s_X, dOut_q, s_dOut, dX, absmax_dX, dW):
    _check(
        load_library().tango_qspmm_bwd(
            g.ref(), heads, dim, _ptr(w_q, torch.int8), _ptr(s_w, torch.float32), _ptr(X_q, torch.int8),
            _ptr(s_X, torch.float32), _ptr(dOut_q, torch.int8), _ptr(s_dOut, torch.float32), _ptr(dX, torch.float32),
            _ptr(absmax_dX, torch.float32), _ptr(dW, torch.float32), _stream(),
        ),
        "tango_qspmm_bwd",
    )


# ---------------------------------------------------------------- fused attention
SIGNATURES.update({
    "tango_gat_attention_workspace_bytes": (_sz, [_i64, _i64, _int]),
    "tango_gat_attention_fwd": (_int, [_gp, _int, _int, _vp, _vp, _vp, _vp, _f32, _vp, _vp, _int, _u64, _u64] + [_vp] * 8
                                + [_sz, _vp]),
})


def tango_gat_attention_workspace_bytes(n_nodes, n_edges, heads) -> int:
    return load_library().tango_gat_attention_workspace_bytes(n_nodes, n_edges, heads)


def tango_gat_attention_fwd(g, heads, dim, S_q, s_S, D_q, s_D, slope, X_q, s_X, rounding, seed, sid_alpha, row_lse,
                            alpha_q, s_alpha, absmax_alpha, alpha_dump, out, absmax_out, ws):
    _check(
        load_library().tango_gat_attention_fwd(
            g.ref(), heads, dim, _ptr(S_q, torch.int8), _ptr(s_S, torch.float32), _ptr(D_q, torch.int8),
            _ptr(s_D, torch.float32), slope, _ptr(X_q, torch.int8), _ptr(s_X, torch.float32), rounding, seed, sid_alpha,
            _ptr(row_lse, torch.float32), _ptr(alpha_q, torch.int8), _ptr(s_alpha, torch.float32),
            _ptr(absmax_alpha, torch.float32), _ptr(alpha_dump, torch.float32), _ptr(out, torch.float32),
            _ptr(absmax_out, torch.float32), _ptr(ws), ws.numel() * ws.element_size(), _stream(),
        ),
        "tango_gat_attention_fwd",
    )


SIGNATURES.update({
    "tango_gat_attention_bwd_workspace_bytes": (_sz, [_i64, _i64, _int]),
    "tango_gat_attention_bwd": (_int, [_gp, _int, _int, _vp, _vp, _vp, _vp, _f32, _vp, _vp, _vp, _vp, _int, _u64, _u64]
                                + [_vp] * 10 + [_sz, _vp]),
})


def tango_gat_attention_bwd_workspace_bytes(n_nodes, n_edges, heads) -> int:
    return load_library().tango_gat_attention_bwd_workspace_bytes(n_nodes, n_edges, heads)


def tango_gat_attention_bwd(g, heads, dim, S_q, s_S, D_q, s_D, slope, row_lse, alpha_q, s_alpha, absmax_alpha, rounding,
                            seed, sid_alpha, X_q, s_X, dOut_q, s_dOut, dX_agg, absmax_dX, dalpha, dS, dD, ws):
    f32, i8 = torch.float32, torch.int8
    _check(
        load_library().tango_gat_attention_bwd(
            g.ref(), heads, dim, _ptr(S_q, i8), _ptr(s_S, f32), _ptr(D_q, i8), _ptr(s_D, f32), slope, _ptr(row_lse, f32),
            _ptr(alpha_q, i8), _ptr(s_alpha, f32), _ptr(absmax_alpha, f32), rounding, seed, sid_alpha, _ptr(X_q, i8),
            _ptr(s_X, f32), _ptr(dOut_q, i8),
            _ptr(s_dOut, f32), _ptr(dX_agg, f32), _ptr(absmax_dX, f32), _ptr(dalpha, f32), _ptr(dS, f32), _ptr(dD, f32),
            _ptr(ws), ws.numel() * ws.element_size(), _stream(),
        ),
        "tango_gat_attention_bwd",
    )


SIGNATURES.update({
    "tango_spmm_f32": (_int, [_gp, _int, _int, _int, _vp, _vp, _vp, _vp]),
    "tango_sddmm_dot_f32": (_int, [_gp, _int, _int, _vp, _vp, _vp, _vp]),
})


def tango_spmm_f32(g, direction, heads, dim, w, X, out):
    f32 = torch.float32
    _check(load_library().tango_spmm_f32(g.ref(), direction, heads, dim, _ptr(w, f32), _ptr(X, f32), _ptr(out, f32), _stream()),
           "tango_spmm_f32")


def tango_sddmm_dot_f32(g, heads, dim, X_src, X_dst, E):
    f32 = torch.float32
    _check(load_library().tango_sddmm_dot_f32(g.ref(), heads, dim, _ptr(X_src, f32), _ptr(X_dst, f32), _ptr(E, f32), _stream()),
           "tango_sddmm_dot_f32")


# ------------------------------------------------------------------- whole layers
class tango_gat_layer(ctypes.Structure):
    _fields_ = (
        [("g", _gp), ("k_in", _int), ("heads", _int), ("dim", _int), ("slope", _f32), ("rounding", _int),
         ("seed", _u64), ("layer_id", _u64)]
        + [(n, _vp) for n in (
            "H", "W", "a_src", "a_dst", "H_q", "s_H", "W_q", "s_W", "Hp", "absmax_Hp", "Hp_q", "s_Hp", "S", "D",
            "S_q", "s_S", "D_q", "s_D", "E", "alpha", "alpha_q", "s_alpha", "out", "absmax_out", "grad_out", "g_q",
            "s_g", "dHp", "absmax_dHp", "dalpha", "dS", "dD", "dHp_q", "s_dHp", "dW", "dH", "da_src", "da_dst")]
        + [("fused", _int), ("row_lse", _vp), ("absmax_alpha", _vp), ("ws", _vp), ("ws_bytes", _sz),
           ("relu_out", _int), ("absmax_H", _vp), ("relu_bits", _vp), ("src_codes", _vp),
           ("dH_keep_bits", _vp), ("absmax_dH", _vp), ("absmax_grad_out", _vp)]
    )


class tango_gcn_layer(ctypes.Structure):
    _fields_ = (
        [("g", _gp), ("k_in", _int), ("f_out", _int), ("rounding", _int), ("seed", _u64), ("layer_id", _u64)]
        + [(n, _vp) for n in (
            "H", "W", "w_q", "s_w", "H_q", "s_H", "W_q", "s_W", "Hp", "absmax_Hp", "Hp_q", "s_Hp", "out",
            "absmax_out", "grad_out", "g_q", "s_g", "dHp", "absmax_dHp", "dHp_q", "s_dHp", "dW", "dH", "ws")]
        + [("ws_bytes", _sz), ("w_q_src_order", _vp)]
    )


class tango_typed_layer(ctypes.Structure):
    _fields_ = (
        [("g_dst", _gp), ("g_src", _gp), ("n_types", _int), ("k_in", _int), ("f_out", _int), ("rounding", _int),
         ("seed", _u64), ("layer_id", _u64)]
        + [(n, _vp) for n in (
            "H", "W", "w_q", "s_w", "H_q", "s_H", "W_q", "s_W", "Hp", "absmax_Hp", "Hp_q", "s_Hp", "out",
            "absmax_out", "grad_out", "g_q", "s_g", "dHp", "absmax_dHp", "dHp_q", "s_dHp", "dW", "dH", "ws")]
        + [("ws_bytes", _sz), ("w_q_src_order", _vp)]
    )


SIGNATURES.update({
    "tango_typed_layer_workspace_bytes": (_sz, [_i64, _i64, _int, _int, _int]),
    "tango_typed_layer_fwd": (_int, [ctypes.POINTER(tango_typed_layer), _vp]),
    "tango_typed_layer_bwd": (_int, [ctypes.POINTER(tango_typed_layer), _vp]),
    "tango_gat_layer_workspace_bytes": (_sz, [_i64, _i64, _int, _int, _int]),
    "tango_gat_layer_fwd": (_int, [ctypes.POINTER(tango_gat_layer), _vp]),
    "tango_gat_layer_bwd": (_int, [ctypes.POINTER(tango_gat_layer), _vp]),
    "tango_gcn_layer_workspace_bytes": (_sz, [_i64, _i64, _int, _int]),
    "tango_gcn_layer_fwd": (_int, [ctypes.POINTER(tango_gcn_layer), _vp]),
    "tango_gcn_layer_bwd": (_int, [ctypes.POINTER(tango_gcn_layer), _vp]),
})


def tango_gat_layer_workspace_bytes(n_nodes, n_edges, k_in, heads, dim) -> int:
    return load_library().tango_gat_layer_workspace_bytes(n_nodes, n_edges, k_in, heads, dim)


def tango_gcn_layer_workspace_bytes(n_nodes, n_edges, k_in, f_out) -> int:
    return load_library().tango_gcn_layer_workspace_bytes(n_nodes, n_edges, k_in, f_out)


class _LayerBuffers:
    """Owns the device tensors one layer struct points at (allocation only; no arithmetic)."""

    _struct = None
    _spec = {}  # field -> (shape fn, dtype)

    def __init__(self):
        self.t = {}
        self.c = self._struct()

    def _alloc(self, name, shape, dtype):
        t = torch.empty(shape, dtype=dtype, device=self.device)
        self.t[name] = t
        setattr(self.c, name, t.data_ptr())
        return t

    def _bind(self, name, tensor, dtype):
        self.t[name] = tensor
        setattr(self.c, name, _ptr(tensor, dtype))

    def __getitem__(self, name):
        return self.t[name]

    def ref(self):
        return ctypes.byref(self.c)


class GatLayer(_LayerBuffers):
    _struct = tango_gat_layer

    def __init__(self, graph: "Graph", H, W, a_src, a_dst, grad_out=None, slope=0.2, rounding=SR, seed=0, layer_id=0,
                 want_dH=True, alias_E_alpha=True, fused=True, keep_alpha=False, keep_alpha_q=False, keep_dalpha=False,
                 relu_out=False, absmax_H=None, relu_bits=False, src_codes=False, dH_keep_bits=None,
                 absmax_grad_out=None):
        super().__init__()
        self.device = H.device
        self.graph = graph
        n, k_in = H.shape
        heads, dim = a_src.shape
        F = heads * dim
        nnz = graph.n_edges
        c = self.c
        c.g = ctypes.pointer(graph.c)
        c.k_in, c.heads, c.dim, c.slope, c.rounding, c.seed, c.layer_id = k_in, heads, dim, slope, rounding, seed, layer_id
        f32, i8 = torch.float32, torch.int8
        for name, tensor in (("H", H), ("W", W), ("a_src", a_src), ("a_dst", a_dst)):
            self._bind(name, tensor, f32)
        for name in ("s_H", "s_W", "absmax_Hp", "s_Hp", "s_S", "s_D", "s_alpha", "absmax_out", "s_g", "absmax_dHp", "s_dHp"):
            self._alloc(name, (1,), f32)
        self._alloc("H_q", (n, k_in), i8)
        self._alloc("W_q", (k_in, F), i8)
        self._alloc("Hp", (n, F), f32)
        self._alloc("Hp_q", (n, F), i8)
        for name in ("S", "D", "dS", "dD"):
            self._alloc(name, (n, heads), f32)
        self._alloc("S_q", (n, heads), i8)
        self._alloc("D_q", (n, heads), i8)
        c.relu_out = 1 if relu_out else 0
        if relu_out and relu_bits:
            self._alloc("relu_bits", ((n * F + 63) // 64 * 8,), torch.uint8)
        if absmax_H is not None:
            self._bind("absmax_H", absmax_H, f32)
        if absmax_grad_out is not None:
            self._bind("absmax_grad_out", absmax_grad_out, f32)
        if dH_keep_bits is not None:  # the relu_bits of the layer below: dH leaves with its ReLU' applied, and its abs-max
            self._bind("dH_keep_bits", dH_keep_bits, torch.uint8)
            self._alloc("absmax_dH", (1,), f32)
        c.fused = 1 if fused else 0
        if fused:
            if src_codes:
                self._alloc("src_codes", (nnz, heads), i8)
            self._alloc("row_lse", (n, heads), f32)
            self._alloc("absmax_alpha", (1,), f32)
            if keep_alpha:
                self._alloc("alpha", (nnz, heads), f32)
            if keep_alpha_q:
                self._alloc("alpha_q", (nnz, heads), i8)
        else:
            self._alloc("alpha", (nnz, heads), f32)
            if alias_E_alpha:
                self._bind("E", self.t["alpha"], f32)
            else:
                self._alloc("E", (nnz, heads), f32)
            self._alloc("alpha_q", (nnz, heads), i8)
        self._alloc("out", (n, F), f32)
        if grad_out is not None:
            self._bind("grad_out", grad_out, f32)
            self._alloc("g_q", (n, F), i8)
            self._alloc("dHp", (n, F), f32)
            if keep_dalpha or not fused or keep_alpha_q:
                self._alloc("dalpha", (nnz, heads), f32)
            self._alloc("dHp_q", (n, F), i8)
            self._alloc("dW", (k_in, F), f32)
            if want_dH:
                self._alloc("dH", (n, k_in), f32)
            self._alloc("da_src", (heads, dim), f32)
            self._alloc("da_dst", (heads, dim), f32)
        nbytes = tango_gat_layer_workspace_bytes(n, nnz, k_in, heads, dim)
        self._alloc("ws", (nbytes,), torch.uint8)
        c.ws_bytes = nbytes


class GatStack:
    """Stacked GAT layers in the configuration the stacked-layer workloads run (allocation and pointer wiring only): the
    ReLU between layers sits inside the layers (`relu_out`, sign bits kept in `relu_bits`), a layer's output is the next
    layer's input with its abs-max handed over (`absmax_H`), a layer's input gradient is written straight into the
    lower layer's `grad_out` with that layer's ReLU' applied (`dH_keep_bits`) and its abs-max handed down
    (`absmax_grad_out`), the sources' S_q codes are kept as an edge-ordered stream (`src_codes`), and nothing else is
    stored per edge unless `keep_alpha` asks for the fp32 attention that was quantized (verification only)."""

    def __init__(self, graph: "Graph", feat, weights, a_src, a_dst, grad_out, slope=0.2, rounding=SR, seed=0,
                 keep_alpha=False):
        n = feat.shape[0]
        last = len(weights) - 1
        self.layers = []
        for i, W in enumerate(weights):
            F = W.shape[1]
            below = self.layers[i - 1] if i > 0 else None
            grad = grad_out if i == last else torch.empty((n, F), dtype=torch.float32, device=feat.device)
            self.layers.append(GatLayer(
                graph, feat if i == 0 else below["out"], W, a_src[i], a_dst[i], grad, slope, rounding, seed, i,
                want_dH=False, relu_out=(i < last), relu_bits=True, src_codes=True, keep_alpha=keep_alpha,
                absmax_H=(below["absmax_out"] if below else None),
                dH_keep_bits=(below["relu_bits"] if below else None)))
        for i in range(1, len(weights)):
            self.layers[i]._bind("dH", self.layers[i - 1]["grad_out"], torch.float32)
            self.layers[i - 1]._bind("absmax_grad_out", self.layers[i]["absmax_dH"], torch.float32)

    def __getitem__(self, i):
        return self.layers[i]

    def __len__(self):
        return len(self.layers)

    def step(self):
        """Forward through every layer, then backward through every layer."""
        for L in self.layers:
            tango_gat_layer_fwd(L)
        for L in reversed(self.layers):
            tango_gat_layer_bwd(L)


class GcnLayer(_LayerBuffers):
    _struct = tango_gcn_layer

    def __init__(self, graph: "Graph", H, W, w_q, s_w, grad_out=None, rounding=SR, seed=0, layer_id=0, want_dH=True,
                 w_q_src_order=None):
        super().__init__()
        self.device = H.device
        self.graph = graph
        if w_q_src_order is not None:  # the fixed edge weights in source-major order (tango_edge_to_src_order), optional
            self._bind("w_q_src_order", w_q_src_order, torch.int8)
        n, k_in = H.shape
        f_out = W.shape[1]
        c = self.c
        c.g = ctypes.pointer(graph.c)
        c.k_in, c.f_out, c.rounding, c.seed, c.layer_id = k_in, f_out, rounding, seed, layer_id
        f32, i8 = torch.float32, torch.int8
        self._bind("H", H, f32)
        self._bind("W", W, f32)
        self._bind("w_q", w_q, i8)
        self._bind("s_w", s_w, f32)
        for name in ("s_H", "s_W", "absmax_Hp", "s_Hp", "absmax_out", "s_g", "absmax_dHp", "s_dHp"):
            self._alloc(name, (1,), f32)
        self._alloc("H_q", (n, k_in), i8)
        self._alloc("W_q", (k_in, f_out), i8)
        self._alloc("Hp", (n, f_out), f32)
        self._alloc("Hp_q", (n, f_out), i8)
        self._alloc("out", (n, f_out), f32)
        if grad_out is not None:
            self._bind("grad_out", grad_out, f32)
            self._alloc("g_q", (n, f_out), i8)
            self._alloc("dHp", (n, f_out), f32)
            self._alloc("dHp_q", (n, f_out), i8)
            self._alloc("dW", (k_in, f_out), f32)
            if want_dH:
                self._alloc("dH", (n, k_in), f32)
        nbytes = tango_gcn_layer_workspace_bytes(n, graph.n_edges, k_in, f_out)
        self._alloc("ws", (nbytes,), torch.uint8)
        c.ws_bytes = nbytes


class TypedLayer(_LayerBuffers):
    """GEMM + SPMM layer over typed edges (GraphSAGE mean aggregator, relational GCN)."""

    _struct = tango_typed_layer

    def __init__(self, g_dst: "Graph", g_src: "Graph", n_types, H, W, w_q, s_w, grad_out=None, rounding=SR, seed=0,
                 layer_id=0, want_dH=True, w_q_src_order=None):
        super().__init__()
        self.device = H.device
        self.g_dst, self.g_src = g_dst, g_src
        if w_q_src_order is not None:
            self._bind("w_q_src_order", w_q_src_order, torch.int8)
        n, k_in = H.shape
        f_cat = W.shape[1]
        f_out = f_cat // n_types
        c = self.c
        c.g_dst = ctypes.pointer(g_dst.c)
        if g_src is not None:
            c.g_src = ctypes.pointer(g_src.c)
        c.n_types, c.k_in, c.f_out, c.rounding, c.seed, c.layer_id = n_types, k_in, f_out, rounding, seed, layer_id
        f32, i8 = torch.float32, torch.int8
        self._bind("H", H, f32)
        self._bind("W", W, f32)
        self._bind("w_q", w_q, i8)
        self._bind("s_w", s_w, f32)
        for name in ("s_H", "s_W", "absmax_Hp", "s_Hp", "absmax_out", "s_g", "absmax_dHp", "s_dHp"):
            self._alloc(name, (1,), f32)
        self._alloc("H_q", (n, k_in), i8)
        self._alloc("W_q", (k_in, f_cat), i8)
        self._alloc("Hp", (n, f_cat), f32)
        self._alloc("Hp_q", (n, f_cat), i8)
        self._alloc("out", (n, f_out), f32)
        if grad_out is not None:
            self._bind("grad_out", grad_out, f32)
            self._alloc("g_q", (n, f_out), i8)
            self._alloc("dHp", (n, f_cat), f32)
            self._alloc("dHp_q", (n, f_cat), i8)
            self._alloc("dW", (k_in, f_cat), f32)
            if want_dH:
                self._alloc("dH", (n, k_in), f32)
        nbytes = load_library().tango_typed_layer_workspace_bytes(n, g_dst.n_edges, n_types, k_in, f_out)
        self._alloc("ws", (nbytes,), torch.uint8)
        c.ws_bytes = nbytes


def tango_typed_layer_workspace_bytes(n_nodes, n_edges, n_types, k_in, f_out) -> int:
    return load_library().tango_typed_layer_workspace_bytes(n_nodes, n_edges, n_types, k_in, f_out)


def tango_typed_layer_fwd(layer: TypedLayer):
    _check(load_library().tango_typed_layer_fwd(layer.ref(), _stream()), "tango_typed_layer_fwd")


def tango_typed_layer_bwd(layer: TypedLayer):
    _check(load_library().tango_typed_layer_bwd(layer.ref(), _stream()), "tango_typed_layer_bwd")


def tango_gat_layer_fwd(layer: GatLayer):
    _check(load_library().tango_gat_layer_fwd(layer.ref(), _stream()), "tango_gat_layer_fwd")


def tango_gat_layer_bwd(layer: GatLayer):
    _check(load_library().tango_gat_layer_bwd(layer.ref(), _stream()), "tango_gat_layer_bwd")


def tango_gcn_layer_fwd(layer: GcnLayer):
    _check(load_library().tango_gcn_layer_fwd(layer.ref(), _stream()), "tango_gcn_layer_fwd")


def tango_gcn_layer_bwd(layer: GcnLayer):
    _check(load_library().tango_gcn_layer_bwd(layer.ref(), _stream()), "tango_gcn_layer_bwd")
