"""Helpers of the GPU parity tests: device transfer and the comparison rules.

Integer results (int8 codes, int32 accumulators) must match the oracle bit for bit; fp32 results must agree
within |gpu - ref| <= ATOL + RTOL*|ref| (the tolerance the benchmark spec fixes for dequantized outputs).
"""
import numpy as np
import torch

RTOL = 1e-5
ATOL = 1e-6


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.to("cuda:0")


def host(t):
    return t.detach().cpu().numpy()


def scalar(v=0.0):
    return torch.full((1,), float(v), dtype=torch.float32, device="cuda:0")


def empty(shape, dtype):
    return torch.empty(shape, dtype=dtype, device="cuda:0")


def workspace(nbytes):
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device="cuda:0")


def assert_bit_exact(got, want, what=""):
    got = np.asarray(got)
    want = np.asarray(want)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    if not np.array_equal(got, want):
        bad = np.flatnonzero(got.ravel() != want.ravel())
        raise AssertionError(
            "%s: %d of %d elements differ; first at %d: got %r want %r"
            % (what, bad.size, got.size, bad[0], got.ravel()[bad[0]], want.ravel()[bad[0]])
        )


def assert_close(got, want, what="", rtol=RTOL, atol=ATOL):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    err = np.abs(got - want)
    lim = atol + rtol * np.abs(want)
    if not (err <= lim).all():
        i = int(np.argmax(err - lim))
        raise AssertionError(
            "%s: %d of %d elements out of tolerance; worst at %d: got %r want %r"
            % (what, int((err > lim).sum()), got.size, i, got.ravel()[i], want.ravel()[i])
        )
