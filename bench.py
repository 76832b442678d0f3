#!/usr/bin/env python3
"""Benchmark of the fused Bi-GCN forward on one MI355X.

A "step" is one pass of the whole hot path (binarise+pack of X, then per layer bit-GEMM and
fused aggregation) over one seeded synthetic graph, with every input already resident in
HBM.  The default workload is the largest of the five (the OGBN-Products-shaped one), on which
the aggregation's bandwidth target is stated.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c1..c5 | s4 | s5]

s4 / s5 run the Bi-GraphSAGE forward (mean aggregator, two weight matrices per layer) through
the same kernels; they are extra workloads, not the headline configuration.
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

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published
INFINITY_CACHE_BYTES = 256 << 20   # MI355X last-level (memory-side) cache, published
VALU_BINARY_MAC_PEAK = 256 * 4 * 16 * 2.4e9 * 32 / 2   # 2 VALU instructions per 32 binary MACs

# HBM bytes per launch of the dominant kernel, measured with rocprofv3 --pmc (FETCH_SIZE and
# WRITE_SIZE, scaled by a copy kernel of known size); see profiles/.  None = not measured.
MEASURED_TRAFFIC_BYTES = {"c5": 3.23e10}    # profiles/spmm_fused_c5.md (layer 1, the slowest launch)


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def standardisation(t, eps=1e-5):
    """Frozen per-column (shift, mul) of a device matrix, from the library's own statistics kernel
    (the parameters are inputs of the forward pass, like running statistics)."""
    from paper_2210_13149_amd import binding as B
    return B.bigcn_column_stats(t, eps)


def build_model(work, B):
    """Upload the workload, pack the weights and calibrate the standardisation of every layer
    that has one with the library's own forward (untimed set-up)."""
    import numpy as np
    import torch
    cfg = work.config
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    drp, dci, dx = dev(work.row_ptr), dev(work.col_idx), dev(work.x)
    if cfg.model == "sage":
        return build_sage_model(work, B, drp, dci, dx)
    weights = [dev(w) for w in work.weights]
    plan = B.Plan(drp, dci, validate=True)
    dinv, _ = B.bigcn_gcn_norm(drp, dci)
    layers = []
    for l, w in enumerate(weights):
        use_bn = l == 0 or cfg.bn_layers == "all"
        shift = mul = None
        if use_bn:
            if l == 0:
                shift, mul = standardisation(dx)
            else:
                h = B.bigcn_forward(plan, drp, dci, dinv, dx, layers)
                shift, mul = standardisation(h)
                del h
        layers.append(B.Layer.from_weight(w, shift, mul))
    need = B.bigcn_forward_workspace_bytes(work.n, layers)
    workspace = torch.empty((need,), dtype=torch.uint8, device="cuda")
    logits = torch.empty((work.n, layers[-1].d_out), dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    return dict(plan=plan, row_ptr=drp, col_idx=dci, dinv=dinv, x=dx, layers=layers,
                workspace=workspace, logits=logits, forward=B.bigcn_forward)


def build_sage_model(work, B, drp, dci, dx):
    """The same set-up for a Bi-GraphSAGE workload (neighbour-list graph, weight pairs)."""
    import numpy as np
    import torch
    cfg = work.config
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    plan = B.Plan(drp, dci, validate=B.VALIDATE_NEIGHBOURS)
    inv_deg = B.bigcn_mean_norm(drp)
    layers = []
    for l, (w_self, w_nbr) in enumerate(work.weights):
        shift = mul = None
        if l == 0 or cfg.bn_layers == "all":
            if l == 0:
                shift, mul = standardisation(dx)
            else:
                h = B.bigcn_sage_forward(plan, drp, dci, inv_deg, dx, layers)
                shift, mul = standardisation(h)
                del h
        layers.append(B.SageLayer.from_weights(dev(w_self), dev(w_nbr), shift, mul))
    need = B.bigcn_sage_forward_workspace_bytes(work.n, layers)
    workspace = torch.empty((need,), dtype=torch.uint8, device="cuda")
    out = torch.empty((work.n, layers[-1].d_out), dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    return dict(plan=plan, row_ptr=drp, col_idx=dci, dinv=inv_deg, x=dx, layers=layers,
                workspace=workspace, logits=out, forward=B.bigcn_sage_forward)


def aggregation_bytes(cfg, nnz, layer, B):
    """Algorithmic bytes of one launch of the fused aggregation of `layer`: per stored entry a
    4-byte column index, one gathered row of integer products and (unless the row carries it) a
    4-byte source scale; per node 8 bytes of row pointer, 4 bytes of row order, 4 bytes of
    per-node factor and the output (packed signs + scale, or fp32 logits); with an own-row term
    (Bi-GraphSAGE) also the node's own product row and scale.  Also the compulsory minimum (every
    array read or written exactly once)."""
    d_in, d_out = cfg.dims[layer], cfg.dims[layer + 1]
    row_bytes, embedded = B.bigcn_forward_row_bytes(d_in, d_out)
    scale_bytes = 0 if embedded else 4
    n = cfg.n_nodes
    last = layer == cfg.n_layers - 1
    out_bytes = 4 * d_out if last else 8 * ((d_out + 63) // 64) + 4
    per_node = 8 + 4 + 4 + out_bytes
    if cfg.model == "sage":
        per_node += row_bytes + scale_bytes
    gather = nnz * (4 + scale_bytes + row_bytes) + n * per_node
    minimum = nnz * 4 + n * (scale_bytes + row_bytes) + n * per_node
    return gather, minimum, row_bytes


MFMA_INT8_MAC_PEAK = 2.5e15     # MI355X dense int8: 5.0 POP/s, two operations per multiply-accumulate
MFMA_FP4_MAC_PEAK = 5.05e15     # MI355X dense fp4: 10.1 PFLOP/s


def gemm_sweep(B, m=262144, n=256, k=4096, reps=10):
    """Compute-bound bit-GEMM outside the workloads (their GEMMs are bound by writing the product
    rows): the three evaluation paths of bigcn_binary_gemm on random bits, int32 accumulators
    only."""
    import torch
    words = (k + 63) // 64
    gen = torch.Generator(device="cuda").manual_seed(1)
    a = torch.randint(-2**62, 2**62, (m, words), dtype=torch.int64, device="cuda", generator=gen)
    b = torch.randint(-2**62, 2**62, (n, words), dtype=torch.int64, device="cuda", generator=gen)
    out = []
    ref = None
    for name, variant in (("valu_xor_popcount", B.GEMM_VALU), ("mfma_int8", B.GEMM_MFMA), ("mfma_fp4", B.GEMM_FP4)):
        acc, _ = B.bigcn_binary_gemm(a, None, b, None, k, want_out=False, variant=variant)
        torch.cuda.synchronize()
        if ref is None:
            ref = acc
        identical = bool(torch.equal(ref, acc))
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            B.bigcn_binary_gemm(a, None, b, None, k, want_out=False, variant=variant)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        rate = m * n * k / (ms * 1e-3)
        out.append({"path": name, "m": m, "n": n, "k_bits": k, "ms": ms, "binary_op_per_s": rate,
                    "frac_valu_peak": rate / VALU_BINARY_MAC_PEAK,
                    "frac_mfma_int8_peak": rate / MFMA_INT8_MAC_PEAK,
                    "frac_mfma_fp4_peak": rate / MFMA_FP4_MAC_PEAK, "identical_to_first": identical})
    return out


def steps_around(B, m, reps=5):
    """The steps on either side of the path, timed on their own (not part of a step): column
    statistics of X, the prediction from the logits and the binning entropy estimate (run on X: two
    passes over the matrix); GB/s of the bytes each must read / write."""
    import torch
    x, logits = m["x"], m["logits"]
    out = {}
    for name, call, nbytes in (
            ("column_stats", lambda: B.bigcn_column_stats(x), x.numel() * 4),
            ("predict_labels", lambda: B.bigcn_predict(logits), logits.numel() * 4 + logits.shape[0] * 4),
            ("predict_softmax", lambda: B.bigcn_predict(logits, want_probs=True),
             logits.numel() * 8 + logits.shape[0] * 4),
            ("entropy_1000_bins_of_x", lambda: B.bigcn_entropy(x, 1000), 2 * x.numel() * 4)):
        call()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            call()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        out[name] = {"ms": ms, "GBps": nbytes / (ms * 1e-3) / 1e9}
    return out


def packed_input_leg(B, m, n_nodes, reps=10):
    """The forward from an input that is stored in binarised form (packed signs + row scales, the
    loaded data of Sec. 5.2): the standardisation of the first layer is applied when the input
    is packed, once, outside the timed region."""
    import torch
    first = m["layers"][0]
    bits, beta = B.bigcn_pack(m["x"], first.bn_shift, first.bn_mul)
    layers = [B.Layer(first.w_bits, first.alpha, first.d_in, first.d_out)] + list(m["layers"][1:])
    call = lambda: B.bigcn_forward_packed(m["plan"], m["row_ptr"], m["col_idx"], m["dinv"], bits, beta,
                                          layers, workspace=m["workspace"], logits=m["logits"])
    call()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        call()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    return {"ms": ms, "nodes_per_s": n_nodes / (ms * 1e-3),
            "input_bytes": bits.numel() * 8 + beta.numel() * 4, "fp32_input_bytes": m["x"].numel() * 4}


def backward_leg(B, m, cfg, reps=3):
    """Back propagation through each layer of the workload (Sec. 4.3, Algorithm 1), timed on its
    own with seeded stand-ins for the layer inputs and the upstream gradient (not part of a
    step).  FLOP rate counts the two dense products (2 * 2 n d_in d_out)."""
    import torch
    n = m["x"].shape[0]
    gen = torch.Generator(device="cuda").manual_seed(7)
    _, vals = B.bigcn_gcn_norm(m["row_ptr"], m["col_idx"], want_vals=True)
    out = []
    for l in range(cfg.n_layers):
        d_in, d_out = cfg.dims[l], cfg.dims[l + 1]
        x = m["x"] if l == 0 else torch.randn((n, d_in), dtype=torch.float32, device="cuda", generator=gen)
        bits, beta = B.bigcn_pack(x)
        w = torch.empty((d_in, d_out), dtype=torch.float32, device="cuda").uniform_(-1.5, 1.5, generator=gen)
        g = torch.randn((n, d_out), dtype=torch.float32, device="cuda", generator=gen) * 0.1
        need = int(B.lib().bigcn_layer_backward_workspace_bytes(n, d_in, d_out))
        ws = torch.empty((need,), dtype=torch.uint8, device="cuda")
        call = lambda: B.bigcn_layer_backward(m["plan"], m["row_ptr"], m["col_idx"], vals, g, bits, beta, w,
                                              want_input_grad=l > 0, workspace=ws)
        call()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            call()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        products = 1 if l == 0 else 2
        out.append({"layer": l, "d_in": d_in, "d_out": d_out, "ms": ms,
                    "dense_TFLOPs": products * 2.0 * n * d_in * d_out / (ms * 1e-3) / 1e12})
        del x, bits, beta, w, g, ws
    return out


def gat_leg(B, m, cfg, reps=3):
    """One Bi-GAT layer (Sec. 4.4.1) on the workload's graph and features, timed alone: first-layer
    shape of the paper's OGBN-Products GAT (two heads of 128 columns) scaled to the workload's
    input width."""
    import torch
    d_in, d_out, heads = cfg.dims[0], 256, 2
    gen = torch.Generator(device="cuda").manual_seed(11)
    w = torch.empty((d_in, d_out), dtype=torch.float32, device="cuda").uniform_(-1, 1, generator=gen)
    layer = B.Layer.from_weight(w)
    a_src = torch.randn((heads, d_out // heads), dtype=torch.float32, device="cuda", generator=gen) * 0.1
    a_dst = torch.randn((heads, d_out // heads), dtype=torch.float32, device="cuda", generator=gen) * 0.1
    call = lambda: B.bigcn_gat_layer(m["plan"], m["row_ptr"], m["col_idx"], m["x"], layer, a_src, a_dst, heads=heads)
    call()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        call()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    nnz = int(m["col_idx"].numel())
    # per neighbour: its index, its compact product row (one byte per product up to 255 input
    # bits, fp16 to 2048, fp32 beyond) and its record {beta, t[heads]}
    elem = 1 if d_in <= 255 else (2 if d_in <= 2048 else 4)
    per_neighbour = 4 + elem * d_out + 4 * (1 + heads)
    return {"d_in": d_in, "d_out": d_out, "heads": heads, "ms": ms, "bytes_per_neighbour": per_neighbour,
            "row_gather_GBps": nnz * per_neighbour / (ms * 1e-3) / 1e9}


def cpu_baseline(work, target_nodes):
    """The plain oracle, as it stands, timed on the host cores: on the benchmark's own workload,
    or on a smaller graph of the same recipe (same mean degree, dims, feature law); nodes/s."""
    import oracle
    from workloads import make_workload, scaled_config
    cfg = work.config
    small = work if target_nodes >= work.n else make_workload(scaled_config(cfg.name, target_nodes))
    calibrate = [True] + [cfg.bn_layers == "all"] * (cfg.n_layers - 1)
    run = oracle.sage_forward if cfg.model == "sage" else oracle.forward
    t0 = time.perf_counter()
    run(small.row_ptr, small.col_idx, small.x, small.weights, calibrate=calibrate)
    dt = time.perf_counter() - t0
    return {"value": small.n / dt, "unit": "nodes/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"whole {cfg.n_layers}-layer oracle forward (with its calibration passes) on "
                      + ("the benchmark's own graph" if small is work else
                         f"a {small.n}-node, {small.config.n_edges}-edge graph of the same recipe")
                      + f" ({dt:.1f} s)"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c5")
    ap.add_argument("--cpu-baseline-nodes", type=int, default=-1,
                    help="nodes in the oracle's timed sample (-1 = the whole workload, about 10 s "
                         "of CPU work for c5 on 16 cores, except s5: 400000 nodes; 0 = skip the "
                         "cpu_baseline leg)")
    ap.add_argument("--copy-probe-mib", type=int, default=0,
                    help="also run one device-to-device copy kernel of this many MiB (a known "
                         "traffic figure to scale rocprofv3 FETCH_SIZE / WRITE_SIZE readings by)")
    ap.add_argument("--graph", action="store_true",
                    help="capture one forward in a HIP graph and time replays (launch-bound small "
                         "workloads; per-kernel figures then come from a separate profiled pass)")
    ap.add_argument("--no-backward", action="store_true",
                    help="skip the back-propagation leg (one bigcn_layer_backward per layer, timed alone)")
    ap.add_argument("--no-gemm-sweep", action="store_true",
                    help="skip the compute-bound bit-GEMM leg (three evaluation paths, M=262144, n=256, K=4096)")
    ap.add_argument("--gemm-sweep-only", action="store_true",
                    help="run only the compute-bound bit-GEMM leg and print it (for counter collection)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
                 "(no collectives are part of it).")

    import torch
    from paper_2210_13149_amd import binding as B, cost_model
    from workloads import get_config, make_workload

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    B.lib()
    if args.gemm_sweep_only:
        print(json.dumps({"bit_gemm_sweep": gemm_sweep(B)}), flush=True)
        return
    cfg = get_config(args.workload)
    t0 = time.perf_counter()
    work = make_workload(cfg)
    log(f"[bench] generated {cfg.name}: {work.n} nodes, nnz {work.nnz} in {time.perf_counter() - t0:.1f} s")
    t0 = time.perf_counter()
    m = build_model(work, B)
    log(f"[bench] set-up (upload, plan, weights, calibration) {time.perf_counter() - t0:.1f} s")
    if args.copy_probe_mib > 0:
        src = torch.ones((args.copy_probe_mib << 18,), dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)                      # one elementwise copy kernel: reads and writes MiB each
        torch.cuda.synchronize()
        log(f"[bench] copy probe: {args.copy_probe_mib} MiB read + {args.copy_probe_mib} MiB written")
        del src, dst
    n_layers = cfg.n_layers
    steps, warmup = max(1, args.steps), max(0, args.warmup)
    profile = B.Profile(n_layers, steps)

    def step(prof=None):
        m["forward"](m["plan"], m["row_ptr"], m["col_idx"], m["dinv"], m["x"], m["layers"],
                     m["workspace"], m["logits"], prof)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    if args.graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
        torch.cuda.current_stream().wait_stream(side)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        graph.replay()
        torch.cuda.synchronize()
        start.record()
        for _ in range(steps):
            graph.replay()
        stop.record()
        torch.cuda.synchronize()
        for _ in range(steps):
            step(profile)                     # per-kernel figures: eager, event-bracketed
        torch.cuda.synchronize()
        per_step = None
    else:
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
        start.record()
        marks[0].record()
        for i in range(steps):
            step(profile)
            marks[i + 1].record()
        stop.record()
        torch.cuda.synchronize()
        per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(steps))
    ms_per_step = start.elapsed_time(stop) / steps
    launch_ms, calls = profile.read()
    assert calls == steps

    nodes_per_s = work.n / (ms_per_step * 1e-3)
    # per-kernel figures from the events recorded inside the timed region
    gemm = []
    spmm = []
    for l in range(n_layers):
        t_gemm = launch_ms[1 + 2 * l] * 1e-3
        t_spmm = launch_ms[2 + 2 * l] * 1e-3
        macs = work.n * cfg.dims[l] * cfg.dims[l + 1] * (2 if cfg.model == "sage" else 1)
        gather, minimum, row_bytes = aggregation_bytes(cfg, work.nnz, l, B)
        # the products are written as rows of row_bytes per node (and per product for Bi-GraphSAGE):
        # on the large workloads this step is bound by those writes, not by the multiplies
        rows_written = work.n * row_bytes * (2 if cfg.model == "sage" else 1)
        gemm.append({"layer": l, "ms": t_gemm * 1e3, "binary_op_per_s": macs / t_gemm,
                     "frac_valu_peak": macs / t_gemm / VALU_BINARY_MAC_PEAK,
                     "frac_mfma_fp4_peak": macs / t_gemm / MFMA_FP4_MAC_PEAK,
                     "rows_written_GBps": rows_written / t_gemm / 1e9,
                     "frac_hbm_peak": rows_written / t_gemm / 1e9 / HBM_PEAK_GBPS})
        # a gathered row moves whole 128-byte lines: rows of 64 bytes cost one line each
        line_bytes = work.nnz * (-(-row_bytes // 128) * 128)
        spmm.append({"layer": l, "ms": t_spmm * 1e3, "row_bytes": row_bytes,
                     "gather_GBps": gather / t_spmm / 1e9, "frac_hbm_peak": gather / t_spmm / 1e9 / HBM_PEAK_GBPS,
                     "row_lines_GBps": line_bytes / t_spmm / 1e9,
                     "compulsory_GBps": minimum / t_spmm / 1e9,
                     # a row array that fits the 256 MB Infinity Cache is gathered from there: the
                     # algorithmic bytes over the HBM peak can then exceed 1 and is no HBM figure
                     "rows_fit_infinity_cache": work.n * row_bytes <= INFINITY_CACHE_BYTES})
    # dominant kernel: the slowest launch of a step (an aggregation on every workload here)
    dom = max(range(n_layers), key=lambda l: spmm[l]["ms"])
    dom_ms = spmm[dom]["ms"]
    dom_bytes = aggregation_bytes(cfg, work.nnz, dom, B)[0]
    achieved = dom_bytes / (dom_ms * 1e-3) / 1e9
    traffic = MEASURED_TRAFFIC_BYTES.get(cfg.name)
    roofline = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": achieved / HBM_PEAK_GBPS, "traffic": traffic,
                "kernel": f"spmm_kernel (fused aggregation), layer {dom}",
                "avg_launch_ms": dom_ms, "algorithmic_bytes_per_launch": dom_bytes,
                "rows_fit_infinity_cache": spmm[dom]["rows_fit_infinity_cache"]}

    result = {
        "metric": "Bi-GCN forward nodes/s; bit-GEMM binary-op/s; SpMM HBM GB/s (% roofline)",
        "model": "Bi-GCN" if cfg.model == "gcn" else "Bi-GraphSAGE (mean aggregator)",
        "value": nodes_per_s, "unit": "nodes/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": ms_per_step, "ms_per_step_median": None if per_step is None else per_step[len(per_step) // 2],
        "ms_per_step_min": None if per_step is None else per_step[0],
        "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "u64 xor/popcount + f32", "data": "synthetic",
        "launch": "hip graph replay" if args.graph else "eager",
        "config": {"workload": f"{cfg.name}: {cfg.stands_in_for}-shaped Chung-Lu graph, {work.n} nodes, "
                               f"{cfg.n_edges} undirected edges "
                               + ("(+ self-loops), Bi-GCN, dims " if cfg.model == "gcn" else
                                  "(neighbour lists), Bi-GraphSAGE mean aggregator, dims ")
                               + "-".join(str(d) for d in cfg.dims),
                   "layers": n_layers, "nnz": work.nnz, "standardisation": cfg.bn_layers},
        "pack_ms": launch_ms[0],
        "pack_GBps": (work.n * (4 * cfg.dims[0] + 8 * ((cfg.dims[0] + 63) // 64) + 4)) / (launch_ms[0] * 1e-3) / 1e9,
        "bit_gemm": gemm, "spmm": spmm,
        "bit_gemm_binary_op_per_s": max(g["binary_op_per_s"] for g in gemm),
        "spmm_GBps": achieved,
        "roofline": roofline,
        "paper_theory": {k: v for k, v in (cost_model.sage_summary if cfg.model == "sage" else
                                           cost_model.summary)(cfg.n_nodes, cfg.n_edges, cfg.dims).items()
                         if k.endswith("ratio")},
    }
    result["steps_around"] = steps_around(B, m)
    if cfg.model == "gcn":
        result["packed_input_forward"] = packed_input_leg(B, m, work.n)
    if not args.no_backward and cfg.model == "gcn":
        result["backward"] = backward_leg(B, m, cfg)
        result["gat_layer"] = gat_leg(B, m, cfg)
    if not args.no_gemm_sweep:
        result["bit_gemm_sweep"] = gemm_sweep(B)
        best = max(result["bit_gemm_sweep"], key=lambda r: r["binary_op_per_s"])
        result["bit_gemm_binary_op_per_s"] = max(result["bit_gemm_binary_op_per_s"], best["binary_op_per_s"])
    if args.cpu_baseline_nodes != 0:
        t0 = time.perf_counter()
        del m
        torch.cuda.empty_cache()
        whole = 400000 if cfg.name == "s5" else cfg.n_nodes
        sample = whole if args.cpu_baseline_nodes < 0 else min(args.cpu_baseline_nodes, cfg.n_nodes)
        result["cpu_baseline"] = cpu_baseline(work, sample)
        log(f"[bench] cpu_baseline leg {time.perf_counter() - t0:.1f} s")
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
