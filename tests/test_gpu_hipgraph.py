"""The layer entry points enqueue kernels only (no allocation, no synchronisation, no memset nodes), so a caller may
record them into a HIP graph: a captured forward + backward is replayed several times, with eager work and
synchronisations between the replays, and every replay must reproduce the eager result."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import tango_inputs as ti
from gpu_util import assert_bit_exact, assert_close, dev, host

OUTPUTS_INT = ["H_q", "W_q", "Hp_q", "S_q", "D_q", "g_q"]
OUTPUTS_F32 = ["Hp", "out", "dHp", "dW", "dH", "da_src", "da_dst"]


@pytest.mark.parametrize("fused", [True, False])
def test_gat_layer_replays_from_a_hip_graph(fused):
    import torch

    import paper_2308_00890_amd as T

    T.load_library()
    li = ti.layer_inputs("toy")
    G = T.Graph.from_host(li.graph)
    L = T.GatLayer(G, dev(li.feat), dev(li.weight), dev(li.a_src), dev(li.a_dst), dev(li.grad_out), 0.2, T.SR, li.sr_seed, 0,
                   fused=fused)
    T.tango_gat_layer_fwd(L)
    T.tango_gat_layer_bwd(L)
    torch.cuda.synchronize()
    want = {k: host(L[k]).copy() for k in OUTPUTS_INT + OUTPUTS_F32}

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        T.tango_gat_layer_fwd(L)
        T.tango_gat_layer_bwd(L)
    other = dev(ti.normal((4096,), 5))
    other_q = torch.empty(4096, dtype=torch.int8, device="cuda:0")
    other_s = torch.zeros(1, device="cuda:0")
    ws = torch.empty(max(T.tango_quantize_workspace_bytes(4096), 256), dtype=torch.uint8, device="cuda:0")
    for replay in range(4):
        for k in OUTPUTS_INT + OUTPUTS_F32:  # eager work between replays: wipe every output, run another call
            L[k].zero_() if L[k].dtype == torch.int8 else L[k].fill_(float("nan"))
        T.tango_quantize(other, T.SR, 1, 1, None, other_q, other_s, ws)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k in OUTPUTS_INT:
            assert_bit_exact(host(L[k]), want[k], "%s, replay %d" % (k, replay))
        for k in OUTPUTS_F32:  # sums through atomics may differ in the last bit between runs
            assert_close(host(L[k]), want[k], "%s, replay %d" % (k, replay))
