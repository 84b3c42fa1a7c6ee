"""ctypes binding of libtango_benchaid.so: the measurement aids of the benchmark harness (include/tango_benchaid.h).

Not part of the method.  As a program it runs the plain streaming copy a few times, which is the yardstick for
rocprofv3's FETCH_SIZE / WRITE_SIZE counters:

    python -m paper_2308_00890_amd.benchaid copy [--mib 1024] [--repeat 3]

and, as `stream_mix`, streaming kernels with chosen read : write ratios (the rate a kernel with that mix can reach).
"""
from __future__ import annotations

import ctypes
import os

import torch

from .binding import TangoError, _check, _ptr, _stream

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtango_benchaid.so")
_vp, _sz, _int = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
_dp = ctypes.POINTER(ctypes.c_double)

# name -> (restype, argtypes); every symbol include/tango_benchaid.h declares
SIGNATURES = {
    "tango_benchaid_mfma_i8_workspace_bytes": (_sz, []),
    "tango_benchaid_mfma_i8_launch": (_int, [_int, _int, _vp, _sz, _dp, _vp]),
    "tango_benchaid_mfma_f8f6f4_launch": (_int, [_int, _int, _int, _vp, _sz, _dp, _vp]),
    "tango_benchaid_copy": (_int, [_vp, _vp, _sz, _vp]),
    "tango_benchaid_stream_mix": (_int, [_vp, _vp, _sz, _int, _int, _vp]),
}
_lib = None


def load_library(path: str = LIB_PATH):
    global _lib
    if _lib is None:
        if not os.path.exists(path):
            raise TangoError("libtango_benchaid.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
        lib = ctypes.CDLL(path)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype = res
            fn.argtypes = args
        _lib = lib
    return _lib


def tango_benchaid_mfma_i8_workspace_bytes() -> int:
    return load_library().tango_benchaid_mfma_i8_workspace_bytes()


def tango_benchaid_mfma_i8_launch(iters, random_operands, ws) -> float:
    """Enqueues the register-only int8 matrix-core loop; returns its operation count (the caller times the launch)."""
    ops = ctypes.c_double(0.0)
    _check(load_library().tango_benchaid_mfma_i8_launch(iters, int(bool(random_operands)), _ptr(ws), ws.numel() * ws.element_size(),
                                                        ctypes.byref(ops), _stream()), "tango_benchaid_mfma_i8_launch")
    return ops.value


def tango_benchaid_mfma_f8f6f4_launch(iters, fmt, random_operands, ws) -> float:
    """The same with the scaled fp8 (fmt 0) / fp4 (fmt 1) matrix instruction."""
    ops = ctypes.c_double(0.0)
    _check(load_library().tango_benchaid_mfma_f8f6f4_launch(iters, fmt, int(bool(random_operands)), _ptr(ws),
                                                            ws.numel() * ws.element_size(), ctypes.byref(ops), _stream()),
           "tango_benchaid_mfma_f8f6f4_launch")
    return ops.value


def tango_benchaid_copy(src, dst):
    nbytes = src.numel() * src.element_size()
    if nbytes % 16 or dst.numel() * dst.element_size() != nbytes:
        raise TangoError("copy needs equal sizes that are multiples of 16 bytes")
    _check(load_library().tango_benchaid_copy(_ptr(src), _ptr(dst), nbytes // 16, _stream()), "tango_benchaid_copy")


STREAM_MIXES = ((1, 0), (4, 1), (2, 1), (1, 1), (1, 2), (1, 4), (0, 1))


def tango_benchaid_stream_mix(src, dst, n_units, reads, writes):
    if src.numel() * src.element_size() < max(reads, 1) * n_units * 16 or dst.numel() * dst.element_size() < max(writes, 1) * n_units * 16:
        raise TangoError("stream_mix: src / dst smaller than reads / writes * n_units * 16 bytes")
    _check(load_library().tango_benchaid_stream_mix(_ptr(src), _ptr(dst), n_units, reads, writes, _stream()),
           "tango_benchaid_stream_mix")


def _time(fn, repeat):
    fn()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(repeat):
        fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / repeat


def stream_mix_rates(mib=1024, repeat=10):
    """[(reads, writes, ms, GB/s)]: every mix over arrays of `mib` MiB each."""
    n_units = (mib << 20) // 16
    src = torch.ones(4 * n_units * 4, dtype=torch.float32, device="cuda:0")
    dst = torch.empty(4 * n_units * 4, dtype=torch.float32, device="cuda:0")
    out = []
    for r, w in STREAM_MIXES:
        ms = _time(lambda: tango_benchaid_stream_mix(src, dst, n_units, r, w), repeat)
        out.append((r, w, ms, (r + w) * n_units * 16 / ms / 1e6))
    return out


def _main():
    import argparse

    ap = argparse.ArgumentParser(description=__doc__)
    ap.add_argument("what", choices=["copy", "stream_mix"])
    ap.add_argument("--mib", type=int, default=1024)
    ap.add_argument("--repeat", type=int, default=3)
    args = ap.parse_args()
    if args.what == "stream_mix":
        for r, w, ms, gbs in stream_mix_rates(args.mib, max(args.repeat, 10)):
            print("k_stream_mix<%d, %d>: %d x %d MiB read + %d x %d MiB written per launch, %.3f ms, %.1f GB/s (read + write)"
                  % (r, w, r, args.mib, w, args.mib, ms, gbs))
        return
    src = torch.ones(args.mib << 18, dtype=torch.float32, device="cuda:0")
    dst = torch.empty_like(src)
    tango_benchaid_copy(src, dst)
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(args.repeat):
        tango_benchaid_copy(src, dst)
    b.record()
    torch.cuda.synchronize()
    ms = a.elapsed_time(b) / args.repeat
    nbytes = src.numel() * 4
    print("k_copy16: %d bytes read + %d bytes written per launch, %.3f ms, %.1f GB/s (read + write)"
          % (nbytes, nbytes, ms, 2 * nbytes / ms / 1e6))


if __name__ == "__main__":
    _main()
