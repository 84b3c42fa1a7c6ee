"""tango_qgemm_static, the entry point for callers that cannot allocate: same results as tango_qgemm, bit for bit, with
the library's fixed device scratch instead of a caller workspace.  Two calls in a row share that scratch (the second on a
smaller input, so stale contents of the first lie beyond what it clears); shapes whose scratch does not fit are refused."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import tango_inputs as ti
from gpu_util import assert_bit_exact, dev, empty, host, scalar, workspace


@pytest.fixture(scope="module")
def T():
    import torch

    import paper_2308_00890_amd as tango

    assert torch.cuda.is_available()
    tango.load_library()
    return tango


def run_both(T, M, N, K, rounding, seed):
    import torch

    A = ti.normal((M, K), seed + 1)
    B = ti.xavier_uniform(K, N, (K, N), seed + 2)
    res = []
    for static in (False, True):
        Aq, Bq = empty((M, K), torch.int8), empty((K, N), torch.int8)
        Aq.fill_(77)
        Bq.fill_(77)
        sA, sB, am = scalar(-1), scalar(-1), scalar(-1)
        C = empty((M, N), torch.float32)
        C.fill_(float("nan"))
        if static:
            T.tango_qgemm_static(dev(A), dev(B), rounding, seed, 1, 2, Aq, sA, Bq, sB, C, am)
        else:
            ws = workspace(T.tango_qgemm_workspace_bytes(M, N, K))
            ws.fill_(0xA5)
            T.tango_qgemm(dev(A), dev(B), rounding, seed, 1, 2, Aq, sA, Bq, sB, C, am, ws)
        torch.cuda.synchronize()
        res.append({k: host(v) for k, v in dict(A_q=Aq, B_q=Bq, s_A=sA, s_B=sB, C=C, absmax_C=am).items()})
    for k in res[0]:
        assert_bit_exact(res[1][k], res[0][k], "%s (M=%d N=%d K=%d)" % (k, M, N, K))


def test_static_entry_point_matches_the_workspace_one_on_two_calls_in_a_row(T):
    # configuration-3 widths first (K = 602 is no multiple of the MFMA depth: padded panel), then a smaller, ragged shape
    # whose padded B panel lies inside the region the first call filled
    run_both(T, 3001, 256, 602, T.SR, 11)
    run_both(T, 777, 100, 33, T.SR, 12)
    run_both(T, 130, 384, 100, T.RN, 13)


def test_static_entry_point_refuses_shapes_beyond_its_scratch(T):
    import torch

    M, N, K = 64, 2048, 2048  # 4 MiB of padded B
    assert T.tango_qgemm_workspace_bytes(M, N, K) > T.QGEMM_STATIC_SCRATCH_BYTES
    C = empty((M, N), torch.float32)
    C.fill_(5.0)
    with pytest.raises(T.TangoError, match="workspace"):
        T.tango_qgemm_static(dev(ti.normal((M, K), 1)), dev(ti.normal((K, N), 2)), T.SR, 1, 1, 2, empty((M, K), torch.int8),
                             scalar(), empty((K, N), torch.int8), scalar(), C, scalar())
    torch.cuda.synchronize()
    assert (host(C) == 5.0).all()  # nothing was launched
