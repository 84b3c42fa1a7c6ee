#!/usr/bin/env python3
"""Benchmark of the quantized GNN-layer hot path on one MI355X.

One "step" = one quantized GAT layer, forward + backward (every abs-max, quantization and dequantization included,
graph construction excluded), on seeded synthetic inputs already resident in HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-cpu-baseline] [--no-extra]

Workloads: gat_dense (configuration 3, the default: the GAT layer the metric is quoted on), toy (1), gcn_arxiv (2),
gat_products (4: three stacked GAT layers), sweep (5: the sparse primitives alone, F = 32..512, with their fp32
twins), qgemm_i8 (a compute-bound GEMM shape outside the paper's configurations), minibatch, sage_arxiv, rgcn_arxiv.

The default line also carries (unless --no-extra): `roofline_hbm`, the dominant kernel timed on configuration 4's
graph, where its gathered table (940 MB) does not fit on chip and HBM really is the bound; and `sparse_kernels`, the
per-kernel table of the metric's second half (qSPMM in both directions and qSDDMM-dot: ms, algorithmic GB/s, % of the
HBM peak) on the configuration-3, -4 and -5 shapes.
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
ON_CHIP_BYTES = 256e6  # Infinity Cache: a gathered table below this size is served on chip after its first touch
READ_STREAM_GBS = 6200.0  # what a plain read-only streaming kernel reaches on this chip (profiles/stream_mix_yardsticks.md)

# HBM-side traffic of the dominant kernel per launch (bytes) as rocprofv3's FETCH_SIZE / WRITE_SIZE counters saw it in
# earlier runs of this file (they cannot be read from inside the process), each scaled by what the same counter reads
# for a plain copy of known size; the summaries with the commands are under profiles/.
PROFILED_TRAFFIC = {
    "gat_dense": (27.5e9, "profiles/gat_dense_hbm_traffic.md"),
    "gat_products": (33.85e9, "profiles/gat_products_kernel_stats_and_traffic.md"),
}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


# ---------------------------------------------------------------- algorithmic bytes per launch
def spmm_bytes(n, nnz, heads, F, reverse=False, elt=1):
    """Quantized SPMM: per edge 4 (index) + heads (int8 weight) + F (gathered int8 row), + 4 (edge-id map) on the
    reversed graph; per node 4 (row pointer) + 4F (fp32 result).  elt = 4 for the fp32 twin (weights and rows fp32)."""
    return nnz * (4 + elt * heads + elt * F + (4 if reverse else 0)) + n * (4 + 4 * F)


def sddmm_dot_bytes(n, nnz, heads, F, elt=1):
    """Quantized SDDMM-dot: per edge 4 (index) + F (gathered source row) + 4*heads (fp32 result); per node 4 (row pointer)
    + F (the destination's row, read once).  elt = 4 for the fp32 twin."""
    return nnz * (4 + elt * F + 4 * heads) + n * (4 + elt * F)


def attention_bwd_src_bytes(n, nnz, heads, F):
    """Source-side walk of the attention backward (steps 5' and 3' in one pass over the out-edges), counted as the
    reverse quantized SPMM it contains plus the edge-to-node sum it also delivers: per edge 4 (neighbour index) + 4 (edge
    id) + heads (the int8 attention code; recomputed here from per-node records instead of read) + F (gathered int8
    gradient row); per node 4 (row pointer) + 4F (fp32 dX_agg) + 12*heads (dS: 4 written, 8 accumulated).  The per-head
    records the kernel really fetches per edge (13*heads bytes: D_q, row_lse, P) and the source's own feature row are left
    out, so this is a lower bound of what the launch moves."""
    return nnz * (8 + heads + F) + n * (4 + 4 * F + 12 * heads)


def attention_bwd_src_compulsory_hbm_bytes(n, nnz, heads, F):
    """What must cross the HBM interface even if every gathered row hits on chip: the index and edge-id streams, each
    table once (gradient rows, feature rows, per-node records of 16 bytes per head), and the results."""
    return nnz * 8 + n * (2 * F + 16 * heads + 4 + 4 * F + 4 * heads)


# ---------------------------------------------------------------------------------- timing
def time_events(torch, fn, iters):
    """Average milliseconds of fn() over iters launches, HIP events on the stream fn launches on (torch's current one)."""
    st = torch.cuda.current_stream()
    a = torch.cuda.Event(enable_timing=True)
    b = torch.cuda.Event(enable_timing=True)
    a.record(st)
    for _ in range(iters):
        fn()
    b.record(st)
    b.synchronize()
    return a.elapsed_time(b) / iters


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


def gather_kernel_record(kernel, workload, ms, alg_bytes, table_bytes, extra=None):
    """One row of the per-kernel table: effective rate = algorithmic bytes / time.  When the gathered table fits the
    Infinity Cache the gathers are served on chip and the rate is not an HBM rate (it can exceed the HBM peak); on a
    skewed graph the rows of the hub nodes are re-gathered from the caches even when the table as a whole is not
    resident, which shows as an effective rate above what an HBM stream reaches - such rows are labelled, and no
    fraction of the HBM peak is claimed for them."""
    gbs = alg_bytes / (ms * 1e-3) / 1e9
    fits = bool(table_bytes <= ON_CHIP_BYTES)
    if fits:
        bound, frac = "on-chip gather (table cache-resident)", None
    elif gbs > READ_STREAM_GBS:
        bound, frac = "hbm + on-chip reuse of repeated rows (effective rate above a read-only HBM stream's)", None
    else:
        bound, frac = "hbm", round(gbs / HBM_PEAK_GBS, 3)
    r = {
        "kernel": kernel,
        "workload": workload,
        "ms": round(ms, 4),
        "algorithmic_GB": round(alg_bytes / 1e9, 3),
        "GBs": round(gbs, 1),
        "effective_rate_over_hbm_peak_pct": round(100.0 * gbs / HBM_PEAK_GBS, 1),
        "bound": bound,
        "frac_of_hbm_peak": frac,
        "gathered_table_MB": round(table_bytes / 1e6, 1),
        "table_fits_on_chip": fits,
    }
    if extra:
        r.update(extra)
    return r


def primitive_records(torch, T, np, G, g, heads, dim, workload, iters, twins):
    """qSPMM in both directions and qSDDMM-dot alone on graph g with random int8 operands of width heads*dim (and, if
    `twins`, the fp32 kernels of the same shape built in the same library): the rows of the per-kernel table."""
    dev = G.in_ptr.device
    F = heads * dim
    n, nnz = g.n_nodes, g.n_edges
    gen = torch.Generator(device=dev)
    gen.manual_seed(2308008900 + F)
    w = torch.randint(-127, 128, (nnz, heads), dtype=torch.int8, device=dev, generator=gen)
    X = torch.randint(-127, 128, (n, F), dtype=torch.int8, device=dev, generator=gen)
    Y = torch.randint(-127, 128, (n, F), dtype=torch.int8, device=dev, generator=gen)
    s1 = torch.full((1,), 0.01, dtype=torch.float32, device=dev)
    s2 = torch.full((1,), 0.02, dtype=torch.float32, device=dev)
    am = torch.zeros(1, dtype=torch.float32, device=dev)
    out = torch.empty((n, F), dtype=torch.float32, device=dev)
    E = torch.empty((nnz, heads), dtype=torch.float32, device=dev)
    recs = []

    def run(kernel, fn, alg, table, extra=None):
        fn()
        torch.cuda.synchronize()
        ms = time_events(torch, fn, iters)
        recs.append(gather_kernel_record(kernel, workload, ms, alg, table, extra))
        log("  %-46s %-34s %8.3f ms  %8.1f GB/s  (effective: %5.1f %% of the HBM peak; %s)" % (kernel, workload, ms, recs[-1]["GBs"], recs[-1]["effective_rate_over_hbm_peak_pct"], recs[-1]["bound"].split(" (")[0]))
        return ms

    t_in = run("tango_qspmm in-edges", lambda: T.tango_qspmm(G, T.IN, heads, dim, w, s1, X, s2, out, am), spmm_bytes(n, nnz, heads, F), n * F)
    t_out = run("tango_qspmm out-edges", lambda: T.tango_qspmm(G, T.OUT, heads, dim, w, s1, Y, s2, out, am),
                spmm_bytes(n, nnz, heads, F, reverse=True), n * F)
    w_src = torch.empty_like(w)
    T.tango_edge_to_src_order(G, heads, w, w_src)
    run("tango_qspmm out-edges, weights in source order", lambda: T.tango_qspmm(G, T.OUT_SRC_ORDER, heads, dim, w_src, s1, Y, s2, out, am),
        spmm_bytes(n, nnz, heads, F), n * F)
    del w_src
    t_dot = run("tango_qsddmm dot", lambda: T.tango_qsddmm(G, T.SDDMM_DOT, heads, dim, X, s1, Y, s2, 0.0, E),
                sddmm_dot_bytes(n, nnz, heads, F), n * F)
    del X, Y, w
    if twins:
        wf = torch.randn((nnz, heads), dtype=torch.float32, device=dev, generator=gen)
        Xf = torch.randn((n, F), dtype=torch.float32, device=dev, generator=gen)
        Yf = torch.randn((n, F), dtype=torch.float32, device=dev, generator=gen)
        t = run("tango_spmm_f32 in-edges", lambda: T.tango_spmm_f32(G, T.IN, heads, dim, wf, Xf, out), spmm_bytes(n, nnz, heads, F, elt=4), 4 * n * F)
        recs[-1]["time_ratio_fp32_over_int8"] = round(t / t_in, 2)
        t = run("tango_spmm_f32 out-edges", lambda: T.tango_spmm_f32(G, T.OUT, heads, dim, wf, Yf, out),
                spmm_bytes(n, nnz, heads, F, reverse=True, elt=4), 4 * n * F)
        recs[-1]["time_ratio_fp32_over_int8"] = round(t / t_out, 2)
        t = run("tango_sddmm_dot_f32", lambda: T.tango_sddmm_dot_f32(G, heads, dim, Xf, Yf, E), sddmm_dot_bytes(n, nnz, heads, F, elt=4), 4 * n * F)
        recs[-1]["time_ratio_fp32_over_int8"] = round(t / t_dot, 2)
        del wf, Xf, Yf
    del out, E
    torch.cuda.empty_cache()
    return recs


def sweep_records(torch, T, np, ti, dev, iters, widths=(32, 64, 128, 256, 512)):
    """Configuration 5: the sparse primitives alone on the scale-22 R-MAT graph (4,194,304 nodes, mean degree 16 with the
    self-loop), one head, feature widths 32..512, each beside its fp32 twin."""
    t0 = time.perf_counter()
    g = ti.config_graph("sweep22")
    log("inputs: sweep22, %d nodes, %d edges (with self-loops), built in %.1f s" % (g.n_nodes, g.n_edges, time.perf_counter() - t0))
    G = T.Graph.from_host(g, dev)
    recs = []
    for F in widths:
        recs += primitive_records(torch, T, np, G, g, 1, F, "config 5 (sweep22), F = %d" % F, iters, twins=True)
    del G
    torch.cuda.empty_cache()
    return recs, g


def hbm_bound_record(torch, T, np, ti, dev, iters, slope=0.2):
    """The dominant kernel (source-side walk of the attention backward) on configuration 4's graph and widths (2.4 M
    nodes, 3 heads x 128): its gathered int8 table is 940 MB, far beyond the on-chip caches, so its gathers are HBM
    traffic and algorithmic bytes / time is a fraction of the HBM roofline.  Also returns the plain-primitive rows."""
    t0 = time.perf_counter()
    li = ti.layer_inputs("gat_products")
    g = li.graph
    log("inputs: gat_products, %d nodes, %d edges (with self-loops), built in %.1f s" % (g.n_nodes, g.n_edges, time.perf_counter() - t0))
    G = T.Graph.from_host(g, dev)
    to = lambda a: torch.from_numpy(a).to(dev)
    heads, dim = li.heads, li.dim
    F = heads * dim
    L = T.GatLayer(G, to(li.feat), to(li.weight), to(li.a_src), to(li.a_dst), to(li.grad_out), slope, T.SR, li.sr_seed, 0,
                   want_dH=False, src_codes=True)
    T.tango_gat_layer_fwd(L)
    T.tango_gat_layer_bwd(L)
    fn, name = attention_bwd_src_launch(torch, T, G, L, heads, dim, slope, li.sr_seed, 6)
    fn()
    torch.cuda.synchronize()
    ms = time_events(torch, fn, iters)
    alg = attention_bwd_src_bytes(g.n_nodes, g.n_edges, heads, F)
    gbs = alg / (ms * 1e-3) / 1e9
    traffic, src = PROFILED_TRAFFIC["gat_products"]
    rec = {
        "kernel": name,
        "workload": "config 4 graph and widths (%d nodes, %d edges, %d heads x %d): the gathered int8 table is %.0f MB, so its "
                    "gathers are HBM traffic" % (g.n_nodes, g.n_edges, heads, dim, g.n_nodes * F / 1e6),
        "bound": "hbm",
        "achieved": gbs,
        "peak": HBM_PEAK_GBS,
        "unit": "GB/s",
        "frac": gbs / HBM_PEAK_GBS,
        "traffic": traffic,
        "traffic_source": "not measured by this run: rocprofv3 FETCH_SIZE/WRITE_SIZE summary in " + src,
        "algorithmic_bytes_per_launch": alg,
        "ms_per_launch": ms,
    }
    log("%s on config 4: %.3f ms/launch, %.1f algorithmic GB/s = %.2f of the HBM peak" % (name, ms, gbs, gbs / HBM_PEAK_GBS))
    del L
    torch.cuda.empty_cache()
    prim = primitive_records(torch, T, np, G, g, heads, dim, "config 4 graph, %d heads x %d" % (heads, dim), iters, twins=False)
    return rec, prim


def oracle_layer_seconds(name, scale_down, slope=0.2):
    """Wall-clock seconds of the CPU oracle, as it stands, for one layer forward + backward of a named configuration
    (or a scaled-down instance of it: same widths and mean degree), and the instance's size."""
    import oracle as orc
    import tango_inputs as ti

    li = ti.layer_inputs(name, scale_down=scale_down)
    g = li.graph
    t0 = time.perf_counter()
    if ti.CONFIGS[name]["kind"] == "gcn":
        w_q, s_w = orc.quantize(ti.gcn_edge_weights(g), orc.SR, li.sr_seed, orc.SID_EW)
        f = orc.gcn_layer_fwd(g, li.feat, li.weight, w_q, s_w, orc.SR, li.sr_seed)
        orc.gcn_layer_bwd(g, f, w_q, s_w, li.grad_out, orc.SR, li.sr_seed)
    else:
        f = orc.gat_layer_fwd(g, li.feat, li.weight, li.a_src, li.a_dst, slope, orc.SR, li.sr_seed)
        orc.gat_layer_bwd(g, f, li.a_src, li.a_dst, li.grad_out, slope, orc.SR, li.sr_seed)
    return time.perf_counter() - t0, g


def cpu_baseline(name, scale_down, layers=1):
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    dt, g = oracle_layer_seconds(name, scale_down)
    if scale_down == 1 and layers == 1:
        return {"value": dt * 1e3, "unit": "ms per layer fwd+bwd", "cores": cores, "kind": "oracle",
                "sample": "the whole workload: oracle layer fwd+bwd at full size (%d nodes, %d edges), one run, %.1f s"
                          % (g.n_nodes, g.n_edges, dt)}
    return {"value": dt * 1e3 * scale_down * layers,
            "unit": "ms per %s fwd+bwd (extrapolated from the sample)" % ("layer" if layers == 1 else "%d layers" % layers),
            "cores": cores, "kind": "oracle",
            "sample": "oracle layer fwd+bwd on a 1/%d instance (%d nodes, %d edges, same widths and mean degree; first-layer "
                      "input width) took %.2f s; value = that time x %d%s"
                      % (scale_down, g.n_nodes, g.n_edges, dt, scale_down, (" x %d layers" % layers) if layers > 1 else "")}


def bench_qgemm_i8(args, torch, T, dev):
    """The int8-input quantized GEMM on a compute-bound shape that is NOT one of the paper's workloads (their GEMMs are
    HBM-bound): shows what the matrix-core main loop reaches.  One step = one tango_qgemm_i8 call, abs-max included."""
    import numpy as np

    from paper_2308_00890_amd import benchaid as B

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
    # the matrix cores' clock takes a fraction of a second of sustained load to settle (from a resting GPU the first few
    # milliseconds of launches run about 12 % slower): warm up for at least 300 launches, whatever --warmup says
    clock_warmup = max(args.warmup, 300)
    for _ in range(clock_warmup):
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
    # the rate the matrix cores sustain from registers alone (int8, and the fp8 / fp4 forms of the scaled instruction)
    ws = torch.empty(B.tango_benchaid_mfma_i8_workspace_bytes(), dtype=torch.uint8, device=dev)
    ceiling = {}
    launches = {"int8": lambda rnd: B.tango_benchaid_mfma_i8_launch(20000, rnd, ws),
                "fp8": lambda rnd: B.tango_benchaid_mfma_f8f6f4_launch(20000, 0, rnd, ws),
                "fp4": lambda rnd: B.tango_benchaid_mfma_f8f6f4_launch(20000, 1, rnd, ws)}
    for fmt, launch in launches.items():
        for label, rnd in (("constant_operands", 0), ("random_operands", 1)):
            cal_ops = [0.0]

            def cal():
                cal_ops[0] = launch(rnd)

            cal()
            torch.cuda.synchronize()
            cal_ms = time_events(torch, cal, 5)
            ceiling["%s_%s" % (fmt, label)] = cal_ops[0] / (cal_ms * 1e-3) / 1e12
            log("register-only MFMA loop, %s, %s: %.1f TOP/s" % (fmt, label, ceiling["%s_%s" % (fmt, label)]))
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
                               "the paper's configurations" % (M, N, K),
                   "untimed_launches_before_the_timed_ones": clock_warmup},
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
            "frac_of_measured_rate_random_operands": tops / ceiling["int8_random_operands"],
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


def bench_sweep(args, torch, T, dev):
    """Configuration 5.  One step = the quantized launches of the sweep (qSPMM over in-edges, over out-edges with the
    weights in either order, and qSDDMM-dot, at the five widths); the per-kernel table is the result."""
    import numpy as np

    import tango_inputs as ti

    recs, g = sweep_records(torch, T, np, ti, dev, max(args.steps, 5))
    q = [r for r in recs if "f32" not in r["kernel"]]
    ms_per_step = sum(r["ms"] for r in q)
    worst = max(q, key=lambda r: r["ms"])
    # the dominant launch of the sweep is its longest one; the lowest HBM fraction among the launches whose table is
    # HBM-resident (where the 60 % target is judged: F >= 128, 537 MB and up) is reported beside it
    big = [r for r in q if not r["table_fits_on_chip"]]
    low = min(big, key=lambda r: r["effective_rate_over_hbm_peak_pct"])
    out = {
        "metric": "ms for the quantized sparse primitives of the sweep (qSPMM in-edges, out-edges with weights in either order, qSDDMM-dot; F = 32..512); "
                  "per kernel HBM GB/s and % of peak",
        "value": ms_per_step,
        "unit": "ms",
        "n_gpus": 1,
        "steps": max(args.steps, 5),
        "warmup": 1,
        "ms_per_step": ms_per_step,
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int8 operands, int32 accumulation, fp32 outputs",
        "data": "synthetic",
        "config": {"workload": "config 5 (sweep22): R-MAT scale 22, %d nodes, %d edges incl. self-loops (mean degree 16), one "
                               "head, F = 32, 64, 128, 256, 512; every launch timed alone with HIP events" % (g.n_nodes, g.n_edges)},
        "roofline": {
            "kernel": worst["kernel"] + ", " + worst["workload"] + " (the longest launch of the sweep)",
            "bound": worst["bound"],
            "achieved": worst["GBs"],
            "peak": HBM_PEAK_GBS if worst["frac_of_hbm_peak"] is not None else None,
            "unit": "GB/s",
            "frac": worst["frac_of_hbm_peak"],
            "traffic": None,
            "algorithmic_bytes_per_launch": worst["algorithmic_GB"] * 1e9,
            "ms_per_launch": worst["ms"],
        },
        "lowest_hbm_fraction": {"kernel": low["kernel"] + ", " + low["workload"], "GBs": low["GBs"],
                                "frac_of_hbm_peak": low["GBs"] / HBM_PEAK_GBS, "ms_per_launch": low["ms"]},
        "sparse_kernels": recs,
        "longest_launch": worst["kernel"] + ", " + worst["workload"],
    }
    if not args.no_cpu_baseline:
        import oracle as orc

        # bounded sample: the oracle's SPMM and SDDMM-dot at F = 128 on the in-edges of the first 1/16 of the nodes
        nsub = g.n_nodes // 16
        e1 = int(g.in_ptr[nsub])
        sub = ti.graph_from_keys(g.n_nodes, (np.repeat(np.arange(nsub, dtype=np.uint64), np.diff(g.in_ptr[: nsub + 1])) << np.uint64(32))
                                 | g.in_src[:e1].astype(np.uint64))
        rng = np.random.default_rng(3)
        F = 128
        w = rng.integers(-127, 128, size=(e1, 1), dtype=np.int8)
        X = rng.integers(-127, 128, size=(g.n_nodes, F), dtype=np.int8)
        t0 = time.perf_counter()
        orc.spmm_in(sub, w, np.float32(0.01), X, np.float32(0.02))
        orc.sddmm_dot(sub, X, np.float32(0.01), X, np.float32(0.02), 1)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": dt * 1e3 * g.n_edges / e1, "unit": "ms for qSPMM in-edges + qSDDMM-dot at F = 128 (extrapolated by edge count)",
                               "cores": int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)), "kind": "oracle",
                               "sample": "oracle spmm_in + sddmm_dot at F = 128 on the %d in-edges of the first %d nodes: %.2f s" % (e1, nsub, dt)}
    print(json.dumps(out), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="gat_dense",
                    choices=["gat_dense", "toy", "gcn_arxiv", "gat_products", "sweep", "qgemm_i8", "minibatch", "sage_arxiv", "rgcn_arxiv"])
    ap.add_argument("--gemm-shape", default="8192,8192,8192", help="M,N,K of the qgemm_i8 workload")
    ap.add_argument("--scale-down", type=int, default=1, help="divide nodes and edges (debugging only)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true",
                    help="gat_dense only: leave out the configuration-4 record of the dominant kernel and the per-kernel table")
    ap.add_argument("--hipgraph", action="store_true",
                    help="record one step into a HIP graph and time replays (same kernels; for the launch-bound small workloads)")
    ap.add_argument("--cpu-scale-down", type=int, default=0)
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
    name = args.workload
    if name == "qgemm_i8":
        bench_qgemm_i8(args, torch, T, dev)
        return
    if name == "sweep":
        bench_sweep(args, torch, T, dev)
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
    attention_kernel = False
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
        w_src = torch.empty_like(w_q)
        T.tango_edge_to_src_order(G_src, 1, w_q, w_src)
        L = T.TypedLayer(G, G_src, nt, to(li.feat), W_cat, w_q, s_w, to(li.grad_out), T.SR, li.sr_seed, 0, w_q_src_order=w_src)
        step = lambda: (T.tango_typed_layer_fwd(L), T.tango_typed_layer_bwd(L))
        heads = 1
        spmm = lambda: T.tango_qspmm(G, T.IN, 1, F, L["w_q"], L["s_w"], L["Hp_q"], L["s_Hp"], L["out"], L["absmax_out"])
        spmm_name = "tango_qspmm, in-edge direction over (source, type) rows (k_spmm_short for rows of up to 64 edges, k_spmm for the rest, prepare/finalize)"
        alg = spmm_bytes(g.n_nodes, g.n_edges, heads, F)
        table_bytes = g.n_nodes * nt * F
    elif cfg["kind"] == "gcn":
        w = to(ti.gcn_edge_weights(g))  # fixed edge weights: inputs of the layer, quantized once outside the timed region
        w_q = torch.empty(w.shape, dtype=torch.int8, device=dev)
        s_w = torch.zeros(1, dtype=torch.float32, device=dev)
        T.tango_quantize(w, T.SR, li.sr_seed, 9, None, w_q, s_w, torch.empty(256, dtype=torch.uint8, device=dev))
        w_src = torch.empty_like(w_q)  # the same codes in source-major order for the backward pass: also made once
        T.tango_edge_to_src_order(G, 1, w_q, w_src)
        L = T.GcnLayer(G, to(li.feat), to(li.weight), w_q, s_w, to(li.grad_out), T.SR, li.sr_seed, 0, w_q_src_order=w_src)
        step = lambda: (T.tango_gcn_layer_fwd(L), T.tango_gcn_layer_bwd(L))
        heads, F = 1, cfg["dim"]
        spmm = lambda: T.tango_qspmm(G, T.IN, 1, F, L["w_q"], L["s_w"], L["Hp_q"], L["s_Hp"], L["out"], L["absmax_out"])
        spmm_name = "tango_qspmm, in-edge direction (k_spmm_short for rows of up to 64 edges, k_spmm for the rest, prepare/finalize)"
        alg = spmm_bytes(g.n_nodes, g.n_edges, heads, F)
        table_bytes = g.n_nodes * F
    elif name == "gat_products":
        # configuration 4: three stacked GAT layers (K_in 100 -> 384 -> 384 -> 384), ReLU between them (inside the layers);
        # one step = forward through all three, then backward through all three
        F = li.heads * li.dim
        heads = li.heads
        Ws, a_srcs, a_dsts = ti.stack_weights(li, 3)
        stack = T.GatStack(G, to(li.feat), [to(w) for w in Ws], [to(a) for a in a_srcs], [to(a) for a in a_dsts],
                           to(li.grad_out), slope, T.SR, li.sr_seed)
        step = stack.step
        L = stack[2]
        spmm, spmm_name = attention_bwd_src_launch(torch, T, G, L, heads, li.dim, slope, li.sr_seed, 16 * 2 + 6)
        alg = attention_bwd_src_bytes(g.n_nodes, g.n_edges, heads, F)
        table_bytes = g.n_nodes * F
        attention_kernel = True
    else:
        L = T.GatLayer(G, to(li.feat), to(li.weight), to(li.a_src), to(li.a_dst), to(li.grad_out), slope, T.SR, li.sr_seed, 0,
                       src_codes=True)
        step = lambda: (T.tango_gat_layer_fwd(L), T.tango_gat_layer_bwd(L))
        heads, F = li.heads, li.heads * li.dim
        # the kernel with the largest share of the step: the source-side walk of the attention backward (steps 5' and 3'
        # together, attention codes recomputed), launched with the arguments tango_gat_layer_bwd gives it
        spmm, spmm_name = attention_bwd_src_launch(torch, T, G, L, heads, li.dim, slope, li.sr_seed, 6)
        alg = attention_bwd_src_bytes(g.n_nodes, g.n_edges, heads, F)
        table_bytes = g.n_nodes * F
        attention_kernel = True

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
    full = args.scale_down == 1 and not typed and not minibatch
    traffic, traffic_src = PROFILED_TRAFFIC.get(name, (None, None)) if full else (None, None)
    on_chip = table_bytes <= ON_CHIP_BYTES
    roofline = {
        "kernel": spmm_name,
        "achieved": achieved,
        "unit": "GB/s",
        "traffic": traffic,
        "traffic_source": ("not measured by this run: rocprofv3 FETCH_SIZE/WRITE_SIZE summary in " + traffic_src) if traffic_src else None,
        "algorithmic_bytes_per_launch": alg,
        "ms_per_launch": spmm_ms,
        "gathered_table_MB": table_bytes / 1e6,
    }
    if on_chip:
        # The gathered table fits the 256 MB Infinity Cache: the gathers are served on chip, HBM does not bind and
        # `achieved` (gathered bytes counted as if they were memory traffic) is an effective rate that may exceed the HBM
        # peak.  No published peak exists for the on-chip gather path, so no fraction is printed for it; what HBM must
        # deliver (the streams and each table once) is reported beside it.
        roofline.update({
            "bound": "on-chip gather (L2 / Infinity Cache to the CUs): the gathered table is cache-resident, HBM does not bind",
            "peak": None,
            "frac": None,
            "effective_rate_over_hbm_peak": achieved / HBM_PEAK_GBS,
        })
        if attention_kernel:
            comp = attention_bwd_src_compulsory_hbm_bytes(g.n_nodes, g.n_edges, heads, F)
            roofline["compulsory_hbm_bytes_per_launch"] = comp
            roofline["compulsory_hbm_GBs"] = comp / (spmm_ms * 1e-3) / 1e9
            roofline["compulsory_hbm_frac_of_peak"] = comp / (spmm_ms * 1e-3) / 1e9 / HBM_PEAK_GBS
    else:
        roofline.update({"bound": "hbm", "peak": HBM_PEAK_GBS, "frac": achieved / HBM_PEAK_GBS})

    out = {
        "metric": ("ms per quantized GraphSAGE (mean) layer fwd+bwd" if typed == "sage_arxiv" else
                   "ms per quantized relational GCN layer (3 relations) fwd+bwd" if typed == "rgcn_arxiv" else
                   "ms per 3 stacked quantized GAT layers fwd+bwd" if name == "gat_products" else
                   "ms per quantized GAT layer fwd+bwd; qSPMM/qSDDMM HBM GB/s and % of peak" if cfg["kind"] == "gat" else
                   "ms per quantized GCN layer fwd+bwd"),
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
        "roofline": roofline,
    }
    if name == "gat_dense" and full and not args.no_extra:
        iters = max(args.steps, 5)
        log("per-kernel table (every launch alone, HIP events, %d launches each):" % iters)
        table = primitive_records(torch, T, np, G, g, heads, li.dim, "config 3 graph, %d heads x %d" % (heads, li.dim), iters, twins=False)
        spmm = step = None  # (the closures hold the layer's tensors)
        del L, G
        torch.cuda.empty_cache()
        out["roofline_hbm"], prim4 = hbm_bound_record(torch, T, np, ti, dev, iters, slope)
        table += prim4
        sweep, _ = sweep_records(torch, T, np, ti, dev, iters)
        out["sparse_kernels"] = table + sweep
    if not args.no_cpu_baseline:
        if minibatch or typed:
            log("no CPU baseline leg for this workload")
        elif name == "gat_products":
            sd = (args.cpu_scale_down or 8) * args.scale_down
            log("cpu baseline (oracle): one layer on a 1/%d instance, extrapolated to three full layers ..." % sd)
            out["cpu_baseline"] = cpu_baseline(name, sd, layers=3)
        else:
            sd = (args.cpu_scale_down or 1) * args.scale_down
            log("cpu baseline (oracle) on %s ..." % ("the full workload" if sd == 1 else "a 1/%d instance" % sd))
            out["cpu_baseline"] = cpu_baseline(name, sd)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
