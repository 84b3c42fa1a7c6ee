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
IN, OUT = 0, 1

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
    "tango_qgemm_workspace_bytes": (_sz, [_i64, _i64, _i64]),
    "tango_qgemm": (_int, [_i64, _i64, _i64, _vp, _vp, _int, _u64, _u64, _u64, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
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
        self.n_edges = int(in_src.numel())
        self.in_ptr, self.in_src = in_ptr, in_src
        self.out_ptr, self.out_dst, self.out_eid = out_ptr, out_dst, out_eid
        self.c = tango_graph(
            self.n_nodes, self.n_edges, _ptr(in_ptr, torch.int32), _ptr(in_src, torch.int32),
            _ptr(out_ptr, torch.int32), _ptr(out_dst, torch.int32), _ptr(out_eid, torch.int32),
        )

    @classmethod
    def from_host(cls, g, device="cuda:0"):
        """``g``: object with numpy int32 arrays n_nodes, in_ptr, in_src, out_ptr, out_dst, out_eid."""
        dev = lambda a: torch.from_numpy(a).to(device)
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


def tango_qspmm_bwd(g, heads, dim, w_q, s_w, X_q, s_X, dOut_q, s_dOut, dX, absmax_dX, dW):
    _check(
        load_library().tango_qspmm_bwd(
            g.ref(), heads, dim, _ptr(w_q, torch.int8), _ptr(s_w, torch.float32), _ptr(X_q, torch.int8),
            _ptr(s_X, torch.float32), _ptr(dOut_q, torch.int8), _ptr(s_dOut, torch.float32), _ptr(dX, torch.float32),
            _ptr(absmax_dX, torch.float32), _ptr(dW, torch.float32), _stream(),
        ),
        "tango_qspmm_bwd",
    )
