"""GPU parity of the quantized GEMM (forward with on-the-fly quantization, backward from cached operands) and of
the attention projections against the CPU oracle, through the C ABI."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import oracle as orc
import tango_inputs as ti
from gpu_util import assert_bit_exact, assert_close, dev, empty, host, scalar, workspace


@pytest.fixture(scope="module")
def T():
    import torch

    import paper_2308_00890_amd as tango

    assert torch.cuda.is_available()
    tango.load_library()
    return tango


# (M, K, N): toy config; K % 4 == 0, K % 2 == 0 and odd K; ragged M, N; N > 256 (two column sweeps); tiny
GEMM_SHAPES = [
    (1024, 64, 64),
    (1000, 128, 256),
    (777, 602, 256),
    (515, 100, 384),
    (130, 33, 70),
    (64, 384, 384),
    (1, 1, 1),
    (3000, 2048, 40),
    (300, 4112, 136),  # reduction longer than the panel kernel takes: quantization pass + tiled int8 kernel
    (260, 72, 2320),   # ... and the same for the dA product of the backward pass (its reduction length is N)
    (200, 128, 64),    # the largest weight matrix that one workgroup prepares (8,192 elements)
    (200, 132, 64),    # ... and a size just above, which takes the multi-launch preparation
    (20000, 64, 64),   # small weights, but an A above the size whose abs-max is handed over as partial maxima
]


@pytest.mark.parametrize("M,K,N", GEMM_SHAPES)
@pytest.mark.parametrize("rounding", [orc.RN, orc.SR])
def test_qgemm_forward(T, M, K, N, rounding):
    import torch

    A = ti.normal((M, K), 31 + M)
    B = ti.xavier_uniform(K, N, (K, N), 32 + K)
    seed = 2308009301
    A_q, B_q = empty((M, K), torch.int8), empty((K, N), torch.int8)
    s_A, s_B, am = scalar(-1), scalar(-1), scalar(-1)
    C = empty((M, N), torch.float32)
    C.fill_(float("nan"))
    ws = workspace(T.tango_qgemm_workspace_bytes(M, N, K))
    T.tango_qgemm(dev(A), dev(B), rounding, seed, 1, 2, A_q, s_A, B_q, s_B, C, am, ws)
    torch.cuda.synchronize()
    r = orc.qgemm(A, B, rounding, seed, 1, 2)
    assert host(s_A)[0] == r["s_A"] and host(s_B)[0] == r["s_B"]
    assert_bit_exact(host(A_q), r["A_q"], "A_q")
    assert_bit_exact(host(B_q), r["B_q"], "B_q")
    assert_bit_exact(host(C), r["C"], "C")  # exact int32 accumulator times one fp32 factor
    assert host(am)[0] == r["absmax_C"]


@pytest.mark.parametrize("M,K,N", GEMM_SHAPES)
def test_qgemm_backward(T, M, K, N):
    import torch

    rng = np.random.default_rng(M + K)
    A_q = rng.integers(-127, 128, size=(M, K), dtype=np.int8)
    B_q = rng.integers(-127, 128, size=(K, N), dtype=np.int8)
    sA, sB = np.float32(0.031), np.float32(0.0007)
    dC = ti.normal((M, N), 40 + N)
    seed = 77
    dC_q = empty((M, N), torch.int8)
    s_dC = scalar(-1)
    dA, dB = empty((M, K), torch.float32), empty((K, N), torch.float32)
    ws = workspace(T.tango_qgemm_bwd_workspace_bytes(M, N, K))
    T.tango_qgemm_bwd(dev(A_q), scalar(sA), dev(B_q), scalar(sB), dev(dC), orc.SR, seed, 8, None, dC_q, s_dC, dA, dB, ws)
    torch.cuda.synchronize()
    r = orc.qgemm_bwd(A_q, sA, B_q, sB, dC, orc.SR, seed, 8)
    assert host(s_dC)[0] == r["s_dC"]
    assert_bit_exact(host(dC_q), r["dC_q"], "dC_q")
    assert_bit_exact(host(dA), r["dA"], "dA")
    assert_bit_exact(host(dB), r["dB"], "dB")
    # only the weight gradient, with a cached abs-max
    dC_q2 = empty((M, N), torch.int8)
    dB2 = empty((K, N), torch.float32)
    T.tango_qgemm_bwd(dev(A_q), scalar(sA), dev(B_q), scalar(sB), dev(dC), orc.SR, seed, 8, scalar(orc.absmax(dC)), dC_q2,
                      s_dC, None, dB2, ws)
    torch.cuda.synchronize()
    assert_bit_exact(host(dC_q2), r["dC_q"], "dC_q (quantize only)")
    assert_bit_exact(host(dB2), r["dB"], "dB (alone)")


# (M, K, N) for the tiled int8 kernels: one tile, ragged M and N, K not a multiple of 128 (the kernel with register
# staging), several tiles; K a multiple of 128 (the kernel with direct global -> LDS loads): one, two, three and many
# K-steps, ragged M and N, eight tile columns (the XCD-aware tile order)
I8_SHAPES = [(256, 64, 256), (300, 80, 130), (1, 16, 1), (515, 1040, 777), (1024, 4096, 512), (257, 48, 513),
             (515, 1152, 777), (2048, 384, 2048), (130, 128, 2300), (1, 128, 1), (700, 640, 300), (300, 256, 256)]


@pytest.mark.parametrize("M,K,N", I8_SHAPES)
def test_qgemm_i8(T, M, K, N):
    import torch

    rng = np.random.default_rng(M * 7 + K)
    A_q = rng.integers(-127, 128, size=(M, K), dtype=np.int8)
    BT_q = rng.integers(-127, 128, size=(N, K), dtype=np.int8)
    if K >= 1040:  # saturated rows: the largest accumulator magnitude the shape allows
        A_q[0, :], BT_q[0, :] = 127, -127
    sA, sB = np.float32(0.0173), np.float32(0.0009)
    C = empty((M, N), torch.float32)
    C.fill_(float("nan"))
    am = scalar(-1)
    T.tango_qgemm_i8(dev(A_q), scalar(sA), dev(BT_q), scalar(sB), C, am)
    torch.cuda.synchronize()
    acc = orc.igemm(A_q, BT_q, transB=True)
    want, want_am = orc.dequant_i32(acc, sA, sB)
    assert_bit_exact(host(C), want, "C")
    assert host(am)[0] == want_am


def test_measurement_aids_of_the_harness(T):
    """libtango_benchaid.so (not part of the method): the register-only matrix-core loops report their operation
    counts and reject a short workspace; the plain copy copies."""
    import torch

    from paper_2308_00890_amd import benchaid as B

    ws = workspace(B.tango_benchaid_mfma_i8_workspace_bytes())
    assert B.tango_benchaid_mfma_i8_launch(10, 1, ws) == 2.0 * 32 * 32 * 32 * 8 * 10 * 256 * 4
    for fmt in (0, 1):
        assert B.tango_benchaid_mfma_f8f6f4_launch(10, fmt, 1, ws) == 2.0 * 32 * 32 * 64 * 8 * 10 * 256 * 4
    torch.cuda.synchronize()
    with pytest.raises(T.TangoError):
        B.tango_benchaid_mfma_i8_launch(10, 1, workspace(16))
    src = torch.arange(1 << 20, dtype=torch.int32, device="cuda:0")
    dst = torch.zeros_like(src)
    B.tango_benchaid_copy(src, dst)
    torch.cuda.synchronize()
    assert torch.equal(src, dst)
    # the stream-mix yardstick: every unit's stores carry the XOR of its loads (and its own index in the first word)
    n_units = 5000
    a = torch.randint(-2**31, 2**31 - 1, (2 * n_units * 4,), dtype=torch.int32, device="cuda:0")
    out = torch.zeros(2 * n_units * 4, dtype=torch.int32, device="cuda:0")
    B.tango_benchaid_stream_mix(a, out, n_units, 2, 1)
    torch.cuda.synchronize()
    x = a.view(2, n_units, 4)
    want = x[0] ^ x[1] ^ torch.tensor([0, 1, 2, 3], dtype=torch.int32, device="cuda:0")
    want[:, 0] ^= torch.arange(n_units, dtype=torch.int32, device="cuda:0")
    assert torch.equal(out.view(2, n_units, 4)[0], want)
    assert int(out.view(2, n_units, 4)[1].abs().sum()) == 0  # one store per unit: the second array stays untouched
    with pytest.raises(T.TangoError):
        B.tango_benchaid_stream_mix(a, out, n_units, 3, 3)  # not one of the built mixes


PROJ_SHAPES = [(1024, 2, 32), (1001, 4, 64), (333, 3, 128), (500, 1, 256), (70, 8, 16), (17, 1, 1024), (5, 2, 4)]


@pytest.mark.parametrize("n,heads,dim", PROJ_SHAPES)
def test_head_proj_forward_backward(T, n, heads, dim):
    import torch

    F = heads * dim
    X = ti.normal((n, F), 50 + n)
    a_s = ti.xavier_uniform(heads, dim, (heads, dim), 51)
    a_d = ti.xavier_uniform(heads, dim, (heads, dim), 52)
    S, D = empty((n, heads), torch.float32), empty((n, heads), torch.float32)
    amS, amD = scalar(-1), scalar(-1)
    T.tango_head_proj(dev(X), dev(a_s), dev(a_d), S, D, amS, amD)
    torch.cuda.synchronize()
    wS, wD = orc.head_proj(X, a_s), orc.head_proj(X, a_d)
    assert_close(host(S), wS, "S")
    assert_close(host(D), wD, "D")
    assert host(amS)[0] == np.abs(host(S)).max() and host(amD)[0] == np.abs(host(D)).max()

    Xq = np.random.default_rng(n).integers(-127, 128, size=(n, F), dtype=np.int8)
    sX = np.float32(0.019)
    dS, dD = ti.normal((n, heads), 53), ti.normal((n, heads), 54)
    agg = ti.normal((n, F), 55)
    dX = empty((n, F), torch.float32)
    am = scalar(-1)
    da_s, da_d = empty((heads, dim), torch.float32), empty((heads, dim), torch.float32)
    ws = workspace(T.tango_head_proj_bwd_workspace_bytes(n, heads, dim))
    T.tango_head_proj_bwd(dev(dS), dev(dD), dev(a_s), dev(a_d), dev(Xq), scalar(sX), dev(agg), dX, am, da_s, da_d, ws)
    torch.cuda.synchronize()
    w_dX, w_am, w_das, w_dad = orc.head_proj_bwd(dS, dD, a_s, a_d, Xq, sX, agg)
    assert_bit_exact(host(dX), w_dX, "dX")  # elementwise fp32 arithmetic in a fixed order
    assert host(am)[0] == w_am
    assert_close(host(da_s), w_das, "da_src")
    assert_close(host(da_d), w_dad, "da_dst")


def test_gemm_bad_arguments(T):
    import torch

    A = dev(ti.normal((8, 8), 1))
    with pytest.raises(T.TangoError):  # workspace too small
        T.tango_qgemm(A, A, orc.SR, 0, 1, 2, empty((8, 8), torch.int8), scalar(), empty((8, 8), torch.int8), scalar(),
                      empty((8, 8), torch.float32), None, workspace(256))
    with pytest.raises(T.TangoError):  # K not a multiple of 16
        T.tango_qgemm_i8(empty((8, 8), torch.int8), scalar(), empty((8, 8), torch.int8), scalar(), empty((8, 8), torch.float32),
                         None)
