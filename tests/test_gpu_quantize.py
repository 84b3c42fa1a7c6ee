"""GPU parity: abs-max, quantize (nearest and stochastic), dequantize against the CPU oracle, through the C ABI."""
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


def run_quantize(T, x, rounding, seed, sid, am_in=None, offset=0):
    import torch

    n = x.size
    xd_full = dev(np.concatenate([np.zeros(offset, np.float32), x.ravel()]))
    xd = xd_full[offset:]
    q_full = empty((n + 16,), torch.int8)
    q = q_full[offset : offset + n]
    s = scalar(-1.0)
    ws = workspace(T.tango_quantize_workspace_bytes(n))
    T.tango_quantize(xd, rounding, seed, sid, am_in, q, s, ws)
    torch.cuda.synchronize()
    return host(q), host(s)[0]


# sizes: empty, below one RNG block, ragged tails, several workgroups, > grid capacity
SIZES = [0, 1, 7, 8, 9, 1000, 4096, 65537, 1 << 20, (1 << 22) + 3]


@pytest.mark.parametrize("n", SIZES)
@pytest.mark.parametrize("rounding", [orc.RN, orc.SR])
def test_quantize_matches_oracle(T, n, rounding):
    x = ti.normal((n,), 1000 + n)
    q, s = run_quantize(T, x, rounding, seed=2308009301, sid=3)
    want_q, want_s = orc.quantize(x, rounding, seed=2308009301, stream=3)
    assert s == want_s
    assert_bit_exact(q, want_q, "quantize n=%d mode=%d" % (n, rounding))


@pytest.mark.parametrize("offset", [1, 2, 3])
def test_quantize_unaligned_pointers(T, offset):
    x = ti.normal((5003,), 77)
    q, s = run_quantize(T, x, orc.SR, seed=5, sid=(1 << 40) + 9, offset=offset)
    want_q, want_s = orc.quantize(x, orc.SR, seed=5, stream=(1 << 40) + 9)
    assert s == want_s
    assert_bit_exact(q, want_q, "unaligned")


def test_quantize_with_cached_absmax_and_big_seed(T):
    x = ti.normal((3, 1111), 78)
    am = np.float32(7.25)  # a cached abs-max larger than the data's own
    q, s = run_quantize(T, x, orc.SR, seed=(1 << 63) + 12345, sid=11, am_in=scalar(am))
    want_q, want_s = orc.quantize(x, orc.SR, seed=(1 << 63) + 12345, stream=11, am=am)
    assert s == want_s
    assert_bit_exact(q, want_q.ravel(), "cached absmax")


def test_quantize_degenerate_tensors(T):
    for x in (np.zeros(100, np.float32), np.full(100, -3.0, np.float32), np.arange(-127, 128, dtype=np.float32)):
        for mode in (orc.RN, orc.SR):
            q, s = run_quantize(T, x, mode, seed=1, sid=2)
            want_q, want_s = orc.quantize(x, mode, seed=1, stream=2)
            assert s == want_s
            assert_bit_exact(q, want_q, "degenerate")


def test_absmax_and_dequantize(T):
    import torch

    for n in (0, 1, 5, 4099, 1 << 21):
        x = ti.normal((n,), 5 + n) * np.float32(3.0)
        out = scalar(-5.0)
        T.tango_absmax(dev(x), out)
        torch.cuda.synchronize()
        assert host(out)[0] == orc.absmax(x)
    q = np.random.default_rng(1).integers(-127, 128, size=10007, dtype=np.int8)
    xd = empty((q.size,), torch.float32)
    T.tango_dequantize(dev(q), scalar(0.0173), xd)
    torch.cuda.synchronize()
    assert_bit_exact(host(xd), orc.dequantize(q, np.float32(0.0173)), "dequantize")


def test_bad_arguments_are_refused(T):
    import torch

    x = dev(ti.normal((64,), 1))
    q = empty((64,), torch.int8)
    s = scalar()
    with pytest.raises(T.TangoError):
        T.tango_quantize(x, 5, 0, 0, None, q, s, workspace(256))  # bad rounding
    with pytest.raises(T.TangoError):
        T.tango_quantize(x, orc.SR, 0, 0, None, q, s, None)  # needs a workspace for the reduction


@pytest.mark.parametrize("rounding", [orc.RN, orc.SR])
def test_error_x_and_bit_count_rule(T, rounding):
    import torch

    x = ti.normal((200003,), 91)
    cands = (4, 6, 8)
    err = empty((3,), torch.float64)
    bits = empty((1,), torch.int32)
    ws = workspace(T.tango_error_x_workspace_bytes())
    T.tango_error_x(dev(x), cands, 0.3, rounding, 17, 5, None, err, bits, ws)
    torch.cuda.synchronize()
    want_bits, want = orc.select_bits(x, cands, 0.3, rounding, 17, 5)
    got = host(err)
    assert np.allclose(got, want, rtol=1e-9, atol=1e-12), (got, want)
    assert int(host(bits)[0]) == want_bits
    # an exactly representable tensor has zero error at 8 bits
    T.tango_error_x(dev(np.arange(-127, 128, dtype=np.float32)), (8,), 0.3, rounding, 1, 1, None, err, bits, ws)
    torch.cuda.synchronize()
    assert host(err)[0] == 0.0 and int(host(bits)[0]) == 8


@pytest.mark.parametrize("n", [1, 3, 4, 1000, 4 * 65536 + 5, 3_000_001])
def test_quantize_xoshiro(T, n):
    import torch

    x = ti.normal((n,), 900 + n)
    q = empty((n,), torch.int8)
    q.fill_(99)
    s = scalar(-1)
    T.tango_quantize_xoshiro(dev(x), 2308, 7, None, q, s, workspace(256))
    torch.cuda.synchronize()
    want_q, want_s = orc.quantize_xoshiro(x, 2308, 7)
    assert host(s)[0] == want_s
    assert_bit_exact(host(q), want_q, "codes from the register-resident generator")


@pytest.mark.parametrize("rounding", [orc.RN, orc.SR])
@pytest.mark.parametrize("n", [0, 5, 8, 1000003])
def test_quantize_behind_relu(T, rounding, n):
    """q = quantize(x where y > 0 else 0), scale from the abs-max of the masked tensor: bit-exact against the oracle's
    quantizer applied to the masked tensor."""
    import torch

    x = ti.normal((n,), 91)
    y = np.maximum(ti.normal((n,), 92), 0)  # a ReLU output: zeros and positives
    if n > 8:
        x[np.argmax(np.abs(x))] *= 3.0  # the overall abs-max ...
        y[np.argmax(np.abs(x))] = 0.0   # ... is masked out, so the scale must come from the masked tensor
    q = torch.empty(n, dtype=torch.int8, device="cuda:0")
    s = torch.zeros(1, dtype=torch.float32, device="cuda:0")
    T.tango_quantize_relu_bwd(dev(x), dev(y), rounding, 7, 21, q, s, workspace(256))
    torch.cuda.synchronize()
    want_q, want_s = orc.quantize(np.where(y > 0, x, 0).astype(np.float32), rounding, 7, 21)
    assert_bit_exact(host(q), want_q, "q")
    assert host(s)[0] == want_s
