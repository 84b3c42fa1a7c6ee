#!/usr/bin/env python3
"""Benchmark of the quantized GNN-layer hot path on one MI355X.

One "step" = one quantized GAT layer, forward + backward (every abs-max, quantization and dequantization included,
graph construction excluded), on seeded synthetic inputs already resident in HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload gat_dense|toy|gcn_arxiv|gat_products|qgemm_i8|minibatch|sage_arxiv|rgcn_arxiv] [--no-cpu-baseline]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, published
MFMA_I8_PEAK_TOPS = 5000.0  # MI355X dense int8 matrix-core rate, published


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def spmm_algorithmic_bytes(n, nnz, heads, F):
    """Per launch of the quantized SPMM: per edge 4 (index) + heads (int8 weight) + F (gathered int8 row);
    per node 4 (row pointer) + 4F (fp32 result)."""
    return nnz * (4 + heads + F) + n * (4 + 4 * F)


def rev_attention_spmm_algorithmic_bytes(n, nnz, heads, F):
    """Per launch of the reverse SPMM with recomputed attention codes (step 5'): per edge 4 (neighbour index)
    + 4 (edge id, for the random bits) + F (gathered int8 gradient row) + heads (D_q of the neighbour)
    + 4*heads (its row_lse); per node 4 (row pointer) + heads (S_q) + 4F (fp32 result)."""
    return nnz * (8 + F + 5 * heads) + n * (4 + heads + 4 * F)


def attention_bwd_src_algorithmic_bytes(n, nnz, heads, F):
    """Per launch of the source-side walk of the attention backward (steps 5' and 3' together, attention codes
    recomputed): per edge 4 (neighbour index) + 4 (edge id, for the random bits) + F (gathered int8 gradient row) and,
    per head, 1 (D_q of the neighbour) + 4 (its row_lse) + 8 (its P); per node 4 (row pointer) + heads (S_q) + F (its
    own int8 feature row) + 4F (fp32 dX_agg) + 4*heads (fp32 dS)."""
    return nnz * (8 + F + 13 * heads) + n * (4 + heads + 5 * F + 4 * heads)


# HBM-side traffic of the dominant kernel per launch (bytes), from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of
# this file, scaled by a 1 GiB copy kernel (FETCH_SIZE reads half the copied bytes, WRITE_SIZE all of them); see
# profiles/.  Keyed by workload; None where no counter run has been recorded.
MEASURED_TRAFFIC = {
    "gat_dense": 27.5e9,      # profiles/gat_dense_hbm_traffic.md, k_spmm<16, true, 2, false, true, 4>
    "gat_products": 33.85e9,  # profiles/gat_products_kernel_stats_and_traffic.md, k_spmm<16, true, 2, false, true, 8>
}


def attention_bwd_src_launch(torch, T, G, L, heads, dim, slope, seed, sid_alpha):
    """A closure that launches tango_gat_attention_bwd_src on the tensors a finished layer step left in place (the
    destination-side half is run once here to fill the P table it reads), and the name of its main kernel."""
    n = L["dS"].shape[0]
    dev = L["dS"].device
    u8 = lambda nbytes: torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=dev)
    rec = u8(T.tango_gat_attention_bwd_rec_bytes(n, heads))
    ws_d = u8(T.tango_gat_attention_bwd_dst_workspace_bytes(n, heads))
    ws_s = u8(T.tango_gat_attention_bwd_src_workspace_bytes(n, heads))
    dD = torch.empty_like(L["dD"])
    dS = torch.empty_like(L["dS"])
    T.tango_gat_attention_bwd_dst(G, heads, dim, L["S_q"], L["s_S"], L["D_q"], L["s_D"], slope, L["row_lse"], L["Hp_q"], L["s_Hp"],
                                  L["g_q"], L["s_g"], rec, dD, ws_d)
    fn = lambda: T.tango_gat_attention_bwd_src(G, heads, dim, L["S_q"], L["s_S"], L["D_q"], L["s_D"], slope, L["row_lse"],
                                               L["s_alpha"], L["absmax_alpha"], T.SR, seed, sid_alpha, L["Hp_q"], L["s_Hp"],
                                               L["g_q"], L["s_g"], rec, L["dHp"], None, dS, ws_s)
    F = heads * dim
    vec = 4 if F <= 64 else (8 if F <= 128 else 16)  # bytes of a feature row per lane, as the library picks them
    lanes_per_head = {64: 4, 128: 8}.get(dim, 0) if vec == 16 else 0  # compile-time only for the common head widths
    name = "k_spmm<%d, true, 2, false, true, %d>" % (vec, lanes_per_head)
    return fn, name + " (attention backward, source side: steps 5' and 3' in one walk over the out-edges)"


def time_events(torch, fn, iters):
    """Average milliseconds of fn() over iters launches, HIP events on the current stream."""
    st = torch.cuda.current_stream()
    a = torch.cuda.Event(enable_timing=True)
    b = torch.cuda.Event(enable_timing=True)
    a.record(st)
    for _ in range(iters):
        fn()
    b.record(st)
    b.synchronize()
    return a.elapsed_time(b) / iters


def cpu_baseline(name, scale_down, slope=0.2):
    """The CPU oracle, as it stands, on a scaled-down instance of the same workload (same mean degree and widths)."""
    import oracle as orc
    import tango_inputs as ti

    li = ti.layer_inputs(name, scale_down=scale_down)
    g = li.graph
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    t0 = time.perf_counter()
    if ti.CONFIGS[name]["kind"] == "gcn":
        w_q, s_w = orc.quantize(ti.gcn_edge_weights(g), orc.SR, li.sr_seed, orc.SID_EW)
        f = orc.gcn_layer_fwd(g, li.feat, li.weight, w_q, s_w, orc.SR, li.sr_seed)
        orc.gcn_layer_bwd(g, f, w_q, s_w, li.grad_out, orc.SR, li.sr_seed)
    else:
        f = orc.gat_layer_fwd(g, li.feat, li.weight, li.a_src, li.a_dst, slope, orc.SR, li.sr_seed)
        orc.gat_layer_bwd(g, f, li.a_src, li.a_dst, li.grad_out, slope, orc.SR, li.sr_seed)
    dt = time.perf_counter() - t0
    return {
        "value": dt * 1e3 * scale_down,
        "unit": "ms per layer fwd+bwd (extrapolated)",
        "cores": cores,
        "kind": "oracle",
        "sample": "oracle layer fwd+bwd on a 1/%d instance (%d nodes, %d edges, same widths and mean degree) took %.2f s; "
                  "value = that time x %d" % (scale_down, g.n_nodes, g.n_edges, dt, scale_down),
    }


def bench_qgemm_i8(args, torch, T, dev):
    """The int8-input quantized GEMM on a compute-bound shape that is NOT one of the paper's workloads (their GEMMs are
    HBM-bound): shows what the matrix-core main loop reaches.  One step = one tango_qgemm_i8 call, abs-max included."""
    import numpy as np

    M, N, K = (int(x) for x in args.gemm_shape.split(","))
    gen = torch.Generator(device=dev)
    gen.manual_seed(2308008900)
    A = torch.randint(-127, 128, (M, K), dtype=torch.int8, device=dev, generator=gen)
    BT = torch.randint(-127, 128, (N, K), dtype=torch.int8, device=dev, generator=gen)
    sA = torch.full((1,), 0.01, dtype=torch.float32, device=dev)
    sB = torch.full((1,), 0.02, dtype=torch.float32, device=dev)
    C = torch.empty((M, N), dtype=torch.float32, device=dev)
    am = torch.zeros(1, dtype=torch.float32, device=dev)
    step = lambda: T.tango_qgemm_i8(A, sA, BT, sB, C, am)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    kernel_ms = time_events(torch, step, max(args.steps, 5))
    ops = 2.0 * M * N * K
    tops = ops / (kernel_ms * 1e-3) / 1e12
    log("tango_qgemm_i8 %dx%dx%d: %.3f ms/step wall, %.3f ms/launch (events), %.1f TOP/s" % (M, N, K, ms_per_step, kernel_ms, tops))
    # the rate the matrix cores sustain from registers alone, constant and random operand bytes
    ws = torch.empty(T.tango_mfma_i8_rate_workspace_bytes(), dtype=torch.uint8, device=dev)
    ceiling = {}
    for label, rnd in (("constant_operands", 0), ("random_operands", 1)):
        cal_ops = [0.0]

        def cal():
            cal_ops[0] = T.tango_mfma_i8_rate_launch(20000, rnd, ws)

        cal()
        torch.cuda.synchronize()
        cal_ms = time_events(torch, cal, 5)
        ceiling[label] = cal_ops[0] / (cal_ms * 1e-3) / 1e12
        log("register-only MFMA loop, %s: %.1f TOP/s" % (label, ceiling[label]))
    out = {
        "metric": "int8 quantized GEMM throughput (int8 in, int32 accumulate, fp32 out + abs-max)",
        "value": ops / (ms_per_step * 1e-3) / 1e12,
        "unit": "TOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int8 operands, int32 accumulation, fp32 output",
        "data": "synthetic",
        "config": {"workload": "tango_qgemm_i8 M=%d N=%d K=%d, uniform random int8 operands; a compute-bound shape outside "
                               "the paper's configurations" % (M, N, K)},
        "roofline": {
            "kernel": "k_gemm_i8",
            "bound": "mfma",
            "achieved": tops,
            "peak": MFMA_I8_PEAK_TOPS,
            "unit": "TOP/s",
            "frac": tops / MFMA_I8_PEAK_TOPS,
            "traffic": None,
            "ms_per_launch": kernel_ms,
            "measured_register_only_mfma_rate": ceiling,
            "frac_of_measured_rate_random_operands": tops / ceiling["random_operands"],
        },
    }
    if not args.no_cpu_baseline:
        import oracle as orc

        m, n, k = min(M, 4096), min(N, 4096), min(K, 8192)  # about 15 s of the oracle on 8 cores
        rng = np.random.default_rng(1)
        a = rng.integers(-127, 128, size=(m, k), dtype=np.int8)
        b = rng.integers(-127, 128, size=(n, k), dtype=np.int8)
        t0 = time.perf_counter()
        acc = orc.igemm(a, b, transB=True)
        orc.dequant_i32(acc, 0.01, 0.02)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": 2.0 * m * n * k / dt / 1e12, "unit": "TOP/s", "cores": int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)),
                               "kind": "oracle", "sample": "oracle igemm + dequantize on %dx%dx%d, %.1f s" % (m, n, k, dt)}
    print(json.dumps(out), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="gat_dense", choices=["gat_dense", "toy", "gcn_arxiv", "gat_products", "qgemm_i8", "minibatch", "sage_arxiv", "rgcn_arxiv"])
    ap.add_argument("--gemm-shape", default="8192,8192,8192", help="M,N,K of the qgemm_i8 workload")
    ap.add_argument("--scale-down", type=int, default=1, help="divide nodes and edges (debugging only)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--hipgraph", action="store_true",
                    help="record one step into a HIP graph and time replays (same kernels; for the launch-bound small workloads)")
    ap.add_argument("--cpu-scale-down", type=int, default=0)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain 1 GiB device-to-device copy three times (to scale rocprofv3's FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on one GPU only (no multi-GPU path exists); use --gpus 1")
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2308_00890_amd as T
    import tango_inputs as ti

    if not torch.cuda.is_available():
        log("bench.py: no GPU visible; the HIP path has no CPU fallback")
        sys.exit(3)
    T.load_library()
    dev = torch.device("cuda:0")
    if args.calibrate_copy:
        a = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        b = torch.empty_like(a)
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
        log("copied 3 x %d bytes" % (a.numel() * 4))
        return
    name = args.workload
    if name == "qgemm_i8":
        bench_qgemm_i8(args, torch, T, dev)
        return
    minibatch = name == "minibatch"
    if minibatch:
        # 256 sampled subgraphs of configuration-1 size (1,024 nodes, 17,408 edges each) handed over as one block-diagonal
        # graph: the mini-batch regime, where per-graph launches would be dispatch-bound
        name = "toy"
    typed = name if name in ("sage_arxiv", "rgcn_arxiv") else None
    if typed:
        # GraphSAGE (mean aggregator) and a relational GCN with three relations on the configuration-2 graph and widths
        name = "gcn_arxiv"
    cfg = ti.CONFIGS[name]
    t0 = time.perf_counter()
    if minibatch:
        li = ti.layer_inputs("toy", graph=ti.minibatch_graph(256, 1024, 16384, ti.BASE_SEED + 40))
    else:
        li = ti.layer_inputs(name, scale_down=args.scale_down)
    g = li.graph
    log("inputs: %s, %d nodes, %d edges (with self-loops), built in %.1f s" % (name, g.n_nodes, g.n_edges, time.perf_counter() - t0))
    G = T.Graph.from_host(g, dev)
    to = lambda a: torch.from_numpy(a).to(dev)
    slope = 0.2
    if typed:
        tg, w_host = ti.sage_typed_graph(g) if typed == "sage_arxiv" else ti.rgcn_typed_graph(g, 3, ti.BASE_SEED + 41)
        nt, F = tg.n_types, cfg["dim"]
        G, G_src = T.Graph.from_host(tg.dst_view(), dev), T.Graph.from_host(tg.src_view(), dev)
        w = to(w_host)
        w_q = torch.empty(w.shape, dtype=torch.int8, device=dev)
        s_w = torch.zeros(1, dtype=torch.float32, device=dev)
        T.tango_quantize(w, T.SR, li.sr_seed, 9, None, w_q, s_w, torch.empty(256, dtype=torch.uint8, device=dev))
        k = li.feat.shape[1]
        W_cat = to(ti.xavier_uniform(k, F, (k, nt * F), li.sr_seed + 20))
        L = T.TypedLayer(G, G_src, nt, to(li.feat), W_cat, w_q, s_w, to(li.grad_out), T.SR, li.sr_seed, 0)
        step = lambda: (T.tango_typed_layer_fwd(L), T.tango_typed_layer_bwd(L))
        heads = 1
        spmm = lambda: T.tango_qspmm(G, T.IN, 1, F, L["w_q"], L["s_w"], L["Hp_q"], L["s_Hp"], L["out"], L["absmax_out"])
        spmm_name = "tango_qspmm, in-edge direction over (source, type) rows (k_spmm_short for rows of up to 64 edges, k_spmm for the rest, prepare/finalize)"
        alg = spmm_algorithmic_bytes(g.n_nodes, g.n_edges, heads, F)
    elif cfg["kind"] == "gcn":
        w = to(ti.gcn_edge_weights(g))  # fixed edge weights: inputs of the layer, quantized once outside the timed region
        w_q = torch.empty(w.shape, dtype=torch.int8, device=dev)
        s_w = torch.zeros(1, dtype=torch.float32, device=dev)
        T.tango_quantize(w, T.SR, li.sr_seed, 9, None, w_q, s_w, torch.empty(256, dtype=torch.uint8, device=dev))
        L = T.GcnLayer(G, to(li.feat), to(li.weight), w_q, s_w, to(li.grad_out), T.SR, li.sr_seed, 0)
        step = lambda: (T.tango_gcn_layer_fwd(L), T.tango_gcn_layer_bwd(L))
        heads, F = 1, cfg["dim"]
        spmm = lambda: T.tango_qspmm(G, T.IN, 1, F, L["w_q"], L["s_w"], L["Hp_q"], L["s_Hp"], L["out"], L["absmax_out"])
        spmm_name = "tango_qspmm, in-edge direction (k_spmm_short for rows of up to 64 edges, k_spmm for the rest, prepare/finalize)"
        alg = spmm_algorithmic_bytes(g.n_nodes, g.n_edges, heads, F)
    elif name == "gat_products":
        # configuration 4: three stacked GAT layers (K_in 100 -> 384 -> 384 -> 384), ReLU between them; one step =
        # forward through all three, then backward through all three
        F = li.heads * li.dim
        heads = li.heads
        # the ReLU sits inside the layers: a layer writes max(0, aggregate) from its SPMM epilogue and passes that
        # tensor's abs-max to the next layer's GEMM; a layer's input gradient is the layer below's grad_out, and ReLU'
        # is applied while that gradient is quantized
        layers = []
        for i in range(3):
            k = li.feat.shape[1] if i == 0 else F
            W = to(ti.xavier_uniform(k, F, (k, F), li.sr_seed + 10 + i))
            feat = to(li.feat) if i == 0 else layers[i - 1]["out"]
            grad = to(li.grad_out) if i == 2 else torch.empty((g.n_nodes, F), dtype=torch.float32, device=dev)
            layers.append(T.GatLayer(G, feat, W, to(li.a_src), to(li.a_dst), grad, slope, T.SR, li.sr_seed, i,
                                     want_dH=False, relu_out=(i < 2), relu_bits=True, src_codes=True,
                                     absmax_H=(layers[i - 1]["absmax_out"] if i > 0 else None),
                                     dH_keep_bits=(layers[i - 1]["relu_bits"] if i > 0 else None)))
        for i in (1, 2):
            # the input-gradient GEMM of layer i writes the lower layer's grad_out with that layer's ReLU' applied and
            # leaves its abs-max
            layers[i]._bind("dH", layers[i - 1]["grad_out"], torch.float32)
            layers[i - 1]._bind("absmax_grad_out", layers[i]["absmax_dH"], torch.float32)

        def step():
            for i in range(3):
                T.tango_gat_layer_fwd(layers[i])
            for i in (2, 1, 0):
                T.tango_gat_layer_bwd(layers[i])

        L = layers[2]
        spmm, spmm_name = attention_bwd_src_launch(torch, T, G, L, heads, li.dim, slope, li.sr_seed, 16 * 2 + 6)
        alg = attention_bwd_src_algorithmic_bytes(g.n_nodes, g.n_edges, heads, F)
    else:
        L = T.GatLayer(G, to(li.feat), to(li.weight), to(li.a_src), to(li.a_dst), to(li.grad_out), slope, T.SR, li.sr_seed, 0,
                       src_codes=True)
        step = lambda: (T.tango_gat_layer_fwd(L), T.tango_gat_layer_bwd(L))
        heads, F = li.heads, li.heads * li.dim
        # the kernel with the largest share of the step: the source-side walk of the attention backward (steps 5' and 3'
        # together, attention codes recomputed), launched with the arguments tango_gat_layer_bwd gives it
        spmm, spmm_name = attention_bwd_src_launch(torch, T, G, L, heads, li.dim, slope, li.sr_seed, 6)
        alg = attention_bwd_src_algorithmic_bytes(g.n_nodes, g.n_edges, heads, F)

    if args.hipgraph:
        step()  # everything allocated and warm before the capture
        torch.cuda.synchronize()
        hip_graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(hip_graph):
            step()
        step = hip_graph.replay
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    log("layer fwd+bwd: %.3f ms/step%s" % (ms_per_step, " (HIP graph replay)" if args.hipgraph else ""))

    # dominant kernel, timed with HIP events on the stream it is launched on (the step above left every input it
    # needs in place); the small helper kernels around it (zeroing, split-row dequantize, fp64 -> fp32) are included
    spmm()
    torch.cuda.synchronize()
    spmm_ms = time_events(torch, spmm, max(args.steps, 5))
    achieved = alg / (spmm_ms * 1e-3) / 1e9
    log("%s: %.3f ms/launch, %.1f algorithmic GB/s" % (spmm_name, spmm_ms, achieved))

    out = {
        "metric": ("ms per quantized GraphSAGE (mean) layer fwd+bwd" if typed == "sage_arxiv" else
                   "ms per quantized relational GCN layer (3 relations) fwd+bwd" if typed == "rgcn_arxiv" else
                   "ms per 3 stacked quantized GAT layers fwd+bwd" if name == "gat_products" else
                   "ms per quantized GAT layer fwd+bwd" if cfg["kind"] == "gat" else "ms per quantized GCN layer fwd+bwd"),
        "value": ms_per_step,
        "unit": "ms",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int8 operands, int32 accumulation, fp32 softmax/outputs",
        "data": "synthetic",
        "config": {
            "workload": ("mini-batch of 256 uniform subgraphs of configuration-1 size as one block-diagonal graph: %d nodes, "
                         "%d edges incl. self-loops, K_in %d, %d heads x %d, SR" % (g.n_nodes, g.n_edges, li.feat.shape[1], li.heads, li.dim))
            if minibatch else
            "%s on the config-2 graph: %d nodes, %d typed edges, %d edge types, K_in %d, F %d per type, SR"
            % (typed, g.n_nodes, g.n_edges, nt, li.feat.shape[1], F)
            if typed else
            "config %d (%s): %s graph, %d nodes, %d edges incl. self-loops, K_in %d, %d heads x %d, SR"
            % (cfg["config"], name, cfg["graph"], g.n_nodes, g.n_edges, li.feat.shape[1], li.heads, li.dim),
            "scale_down": args.scale_down,
            "launch": "hip graph replay" if args.hipgraph else "eager",
            "layer_caches": ("edge-ordered source codes" + (", ReLU sign bits" if name == "gat_products" else ""))
            if cfg["kind"] == "gat" and not typed else "none",
        },
        "roofline": {
            "kernel": spmm_name,
            "bound": "hbm",
            "achieved": achieved,
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS,
            "traffic": MEASURED_TRAFFIC.get(name) if args.scale_down == 1 and not typed and not minibatch else None,
            "algorithmic_bytes_per_launch": alg,
            "ms_per_launch": spmm_ms,
        },
    }
    if not args.no_cpu_baseline:
        if name == "gat_products":
            log("no CPU baseline leg for the 3-layer workload")
            print(json.dumps(out), flush=True)
            return
        if minibatch or typed:
            log("no CPU baseline leg for this workload")
            print(json.dumps(out), flush=True)
            return
        sd = args.cpu_scale_down or {"gat_dense": 8, "gcn_arxiv": 1, "toy": 1}[name]
        sd *= args.scale_down
        log("cpu baseline (oracle) on a 1/%d instance ..." % sd)
        out["cpu_baseline"] = cpu_baseline(name, sd, slope)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
