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
SMALL_GRAPH_ROWS = 32768        # up to here the forward uses the one-row-per-wavefront kernels

# Bytes that crossed the L2-to-fabric boundary per launch of the dominant kernel, measured with
# rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE, each scaled by a copy of known size): read from the
# tracked summary that names the kernel and the commit it was measured at.  Absent = null.
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "dominant_kernel_traffic.txt")


def measured_traffic(workload):
    """{"bytes": ..., "kernel": ..., "commit": ...} for `workload` from TRAFFIC_FILE, or None.
    Lines: `workload | kernel | commit | bytes per launch`; `#` starts a comment."""
    try:
        lines = open(TRAFFIC_FILE).read().splitlines()
    except OSError:
        return None
    for line in lines:
        parts = [f.strip() for f in line.split("#")[0].split("|")]
        if len(parts) == 4 and parts[0] == workload:
            return {"bytes": float(parts[3]), "kernel": parts[1], "measured_at_commit": parts[2]}
    return None


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
MFMA_FP32_FLOP_PEAK = 157.3e12  # MI355X dense fp32 matrix


def _time_calls(call, reps):
    """Mean milliseconds of `call` over `reps` back-to-back launches (events on torch's stream)."""
    import torch
    call()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        call()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def multiply_only_probe(B, iterations=4000):
    """The rate of a launch of nothing but FP4 matrix-core multiplies on pseudo-random +-1 codes
    (library entry bigcn_probe_fp4_multiply_rate): what this device sustains when loads, code
    expansion and stores cost nothing."""
    import torch
    sink = torch.empty((256 * 1024,), dtype=torch.float32, device="cuda")
    macs = B.bigcn_probe_fp4_multiply_rate(iterations, sink)
    ms = _time_calls(lambda: B.bigcn_probe_fp4_multiply_rate(iterations, sink), 3)
    # the same with the expansion of packed bits to FP4 codes put back, alternating with the
    # multiplies of the step before: what a kernel with bit-packed inputs could reach if only
    # loads and stores were free
    macs_x = B.bigcn_probe_fp4_expand_multiply_rate(iterations, sink)
    ms_x = _time_calls(lambda: B.bigcn_probe_fp4_expand_multiply_rate(iterations, sink), 3)
    return {"ms": ms, "binary_op_per_s": macs / (ms * 1e-3), "frac_mfma_fp4_peak": macs / (ms * 1e-3) / MFMA_FP4_MAC_PEAK,
            "with_expansion": {"ms": ms_x, "binary_op_per_s": macs_x / (ms_x * 1e-3),
                               "frac_mfma_fp4_peak": macs_x / (ms_x * 1e-3) / MFMA_FP4_MAC_PEAK}}


def gemm_sweep(B, m=262144, n=256, ks=(1024, 4096, 8192), reps=10):
    """Bit-GEMM outside the workloads (their GEMMs are bound by writing the product rows): random
    bits, int32 accumulators only.  The three evaluation paths of bigcn_binary_gemm at K = 4096 and
    the FP4 path over K (the int32 output is 4 bytes per K multiply-accumulates, so the shape is
    the more compute-bound the larger K: at K = 4096 the 268 MB of output and 134 MB of input are
    0.05 ms at 8 TB/s against 0.054 ms of multiplies at the FP4 peak).  Each FP4 result carries its
    fraction of the published peak and of the multiply-only rate measured in the same run."""
    import torch
    gen = torch.Generator(device="cuda").manual_seed(1)
    ceiling = multiply_only_probe(B)
    out = {"shape": {"m": m, "n": n}, "multiply_only": ceiling, "paths": []}
    ref = {}
    for k in ks:
        words = (k + 63) // 64
        a = torch.randint(-2**62, 2**62, (m, words), dtype=torch.int64, device="cuda", generator=gen)
        b = torch.randint(-2**62, 2**62, (n, words), dtype=torch.int64, device="cuda", generator=gen)
        variants = (("valu_xor_popcount", B.GEMM_VALU), ("mfma_int8", B.GEMM_MFMA), ("mfma_fp4", B.GEMM_FP4)) \
            if k == 4096 else (("mfma_fp4", B.GEMM_FP4),)
        for name, variant in variants:
            acc, _ = B.bigcn_binary_gemm(a, None, b, None, k, want_out=False, variant=variant)
            torch.cuda.synchronize()
            if k not in ref:
                ref[k] = acc
            identical = bool(torch.equal(ref[k], acc))
            ms = _time_calls(lambda: B.bigcn_binary_gemm(a, None, b, None, k, want_out=False, variant=variant), reps)
            rate = m * n * k / (ms * 1e-3)
            bytes_moved = m * words * 8 + n * words * 8 + m * n * 4
            out["paths"].append({"path": name, "m": m, "n": n, "k_bits": k, "ms": ms, "binary_op_per_s": rate,
                                 "frac_valu_peak": rate / VALU_BINARY_MAC_PEAK,
                                 "frac_mfma_int8_peak": rate / MFMA_INT8_MAC_PEAK,
                                 "frac_mfma_fp4_peak": rate / MFMA_FP4_MAC_PEAK,
                                 "frac_of_multiply_only_rate": rate / ceiling["binary_op_per_s"],
                                 "frac_of_expand_and_multiply_rate": rate / ceiling["with_expansion"]["binary_op_per_s"],
                                 "compulsory_bytes": bytes_moved,
                                 "ms_of_compulsory_bytes_at_hbm_peak": bytes_moved / (HBM_PEAK_GBPS * 1e9) * 1e3,
                                 "identical_to_first": identical})
        del a, b
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
        flops = products * 2.0 * n * d_in * d_out
        nnz = int(m["col_idx"].numel())
        if l == 0:
            # no input gradient and d_in <= d_out: the aggregation gathers packed sign rows (index,
            # coefficient, scale and the row's words per stored entry) and writes n x d_in fp32
            words = (d_in + 63) // 64
            gather = nnz * (4 + 4 + 4 + 8 * words) + n * 4 * d_in + n * 4 * d_out
        else:
            # g_zeta = A~^T g_out: per stored entry an index, a coefficient and one fp32 gradient row;
            # then g_zeta is read by both dense products and g_in is written
            gather = nnz * (4 + 4 + 4 * d_out) + n * 4 * d_out * 3 + n * 4 * d_in
        t_hbm, t_mfma = gather / (HBM_PEAK_GBPS * 1e9), flops / MFMA_FP32_FLOP_PEAK
        bound = "hbm" if t_hbm >= t_mfma else "mfma"
        out.append({"layer": l, "d_in": d_in, "d_out": d_out, "ms": ms,
                    "dense_TFLOPs": flops / (ms * 1e-3) / 1e12,
                    "frac_mfma_fp32_peak": flops / (ms * 1e-3) / MFMA_FP32_FLOP_PEAK,
                    "algorithmic_bytes": gather, "algorithmic_GBps": gather / (ms * 1e-3) / 1e9,
                    "bound": bound, "frac": (t_hbm if bound == "hbm" else t_mfma) / (ms * 1e-3)})
        del x, bits, beta, w, g, ws
    return out


def gat_leg(B, m, cfg, reps=3, hidden=False):
    """One Bi-GAT layer (Sec. 4.4.1) on the workload's graph, timed alone: first-layer shape of the
    paper's OGBN-Products GAT (two heads of 128 columns) on the workload's features, or
    (hidden=True) a hidden layer of the same width on seeded stand-ins for its 256 input columns."""
    import torch
    d_in, d_out, heads = (256 if hidden else cfg.dims[0]), 256, 2
    gen = torch.Generator(device="cuda").manual_seed(11)
    x = m["x"]
    if hidden:
        x = torch.randn((x.shape[0], d_in), dtype=torch.float32, device="cuda", generator=gen)
    w = torch.empty((d_in, d_out), dtype=torch.float32, device="cuda").uniform_(-1, 1, generator=gen)
    layer = B.Layer.from_weight(w)
    a_src = torch.randn((heads, d_out // heads), dtype=torch.float32, device="cuda", generator=gen) * 0.1
    a_dst = torch.randn((heads, d_out // heads), dtype=torch.float32, device="cuda", generator=gen) * 0.1
    call = lambda: B.bigcn_gat_layer(m["plan"], m["row_ptr"], m["col_idx"], x, layer, a_src, a_dst, heads=heads)
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
    # per neighbour: its index, its compact product row (one byte per product up to 256 input
    # bits, fp16 to 2048, fp32 beyond; 256 bits: values over the first 255, the last bit on the
    # sign of beta) and its record {beta, t[heads]}, which rides in the row's spare top bits when
    # the products fit 7 bits (256 columns, at most two heads and 256 input bits; beyond 127 bits
    # the library tests the rows, and seeded random signs never leave 7 bits)
    elem = 1 if d_in <= 256 else (2 if d_in <= 2048 else 4)
    embedded = d_in <= 256 and d_out == 256 and heads <= 2
    per_neighbour = 4 + elem * d_out + (0 if embedded else 4 * (1 + heads))
    lines = 128 * (-(-(elem * d_out) // 128) + (0 if embedded else 1))   # the row's cache lines (+ one for the record)
    return {"d_in": d_in, "d_out": d_out, "heads": heads, "ms": ms, "bytes_per_neighbour": per_neighbour,
            "record_inside_row": embedded,
            "row_gather_GBps": nnz * per_neighbour / (ms * 1e-3) / 1e9,
            "bound": "hbm", "frac": nnz * per_neighbour / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
            "cache_line_bytes_per_neighbour": lines,
            "cache_line_GBps": nnz * lines / (ms * 1e-3) / 1e9}


def stream_probe(mib=2048, B=None):
    """Streaming rates of this machine for scale, on `mib` MiB of fp32, in GB/s of the bytes each must
    move: torch's own elementwise kernels for copy (read + write), sum (read) and fill (write), and
    the library's read-only launch (bigcn_probe_stream_read: contiguous pieces, eight 16-byte loads
    per thread in flight), which is the rate a step bound by reading its input is compared with."""
    import torch
    n = mib << 18
    src = torch.ones((n,), dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    nbytes = n * 4
    out = {"mib": mib}
    for name, call, moved in (("copy", lambda: dst.copy_(src), 2 * nbytes), ("read_sum", lambda: src.sum(), nbytes),
                              ("fill", lambda: dst.fill_(1.0), nbytes)):
        ms = _time_calls(call, 5)
        out[name + "_GBps"] = moved / (ms * 1e-3) / 1e9
    if B is not None:
        sink = torch.empty((8192 * 1024,), dtype=torch.float32, device="cuda")
        ms = _time_calls(lambda: B.bigcn_probe_stream_read(src, sink), 5)
        out["read_GBps"] = nbytes / (ms * 1e-3) / 1e9
    return out


def gather_probe(B, m, row_bytes_list, reps=5):
    """The plain gather of this graph: the public fp32 aggregation bigcn_spmm (unit coefficients)
    on rows of the given widths, i.e. the same cache lines per neighbour that the fused
    aggregation gathers, without its conversions and epilogue.  The reference a gather of
    cache-resident rows is compared with (no published peak exists for it)."""
    import torch
    n = m["x"].shape[0]
    out = {}
    for row_bytes in sorted(set(row_bytes_list)):
        d = max(1, row_bytes // 4)
        z = torch.ones((n, d), dtype=torch.float32, device="cuda")
        o = torch.empty_like(z)
        ms = _time_calls(lambda: B.bigcn_spmm(m["plan"], m["row_ptr"], m["col_idx"], None, z, o), reps)
        out[str(row_bytes)] = ms
        del z, o
    return out


def infinity_cache_model(row_ptr_host, row_bytes, cache_bytes=INFINITY_CACHE_BYTES):
    """A MODEL, not a measurement (no counter of this box sees behind the L2-to-fabric boundary):
    share of the gathered rows that a least-recently-used cache of `cache_bytes` would serve when
    node k's row is requested deg(k) times per launch (once per stored entry of column k; the
    pattern is symmetric), by the characteristic-time approximation: a row is resident with
    probability 1 - exp(-deg_k T), T set so that the expected resident bytes equal the cache."""
    import numpy as np
    deg = np.diff(row_ptr_host).astype(np.float64)
    lines = -(-row_bytes // 128) * 128
    capacity_rows = cache_bytes / lines
    if capacity_rows >= deg.size:
        return {"hit_rate": 1.0, "kind": "model: rows fit the cache"}
    lo, hi = 0.0, 1.0
    while (1.0 - np.exp(-deg * hi)).sum() < capacity_rows:
        hi *= 2.0
    for _ in range(60):
        mid = 0.5 * (lo + hi)
        if (1.0 - np.exp(-deg * mid)).sum() < capacity_rows:
            lo = mid
        else:
            hi = mid
    resident = 1.0 - np.exp(-deg * hi)
    hit = float((deg * resident).sum() / deg.sum())
    return {"hit_rate": hit, "kind": "model: LRU characteristic-time approximation, requests proportional to degree"}


def slot_bounds(cfg, work_n, nnz, B, launch_ms):
    """For every launch of a forward the bound it is compared with and the fraction reached:
    slot 0 = binarise + pack, then per layer the bit-GEMM and the aggregation.  Bounds: HBM for the
    pack (X once), the larger of HBM (packed input + product rows) and the arithmetic peak of the
    path that runs (FP4 matrix cores or XOR + bit count, as bigcn_forward_gemm_path says) for the
    bit-GEMM, and the gather's algorithmic
    bytes over HBM for the aggregation.  On graphs of at most 32768 nodes the binarisation is part
    of the first bit-GEMM launch (slot 0 is empty)."""
    n = work_n
    dims = cfg.dims
    small = n <= SMALL_GRAPH_ROWS
    words0 = (dims[0] + 63) // 64
    slots = []
    pack_bytes = n * (4 * dims[0] + 8 * words0 + 4)
    if not small or cfg.model == "sage":
        t = launch_ms[0] * 1e-3
        slots.append({"slot": "pack", "ms": launch_ms[0], "bound": "hbm", "algorithmic_bytes": pack_bytes,
                      "achieved": pack_bytes / t / 1e9, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                      "frac": pack_bytes / t / 1e9 / HBM_PEAK_GBPS})
    for l in range(cfg.n_layers):
        d_in, d_out = dims[l], dims[l + 1]
        products = 2 if cfg.model == "sage" else 1
        row_bytes, _ = B.bigcn_forward_row_bytes(d_in, d_out)
        t = launch_ms[1 + 2 * l] * 1e-3
        macs = n * d_in * d_out * products
        fp4 = B.bigcn_forward_gemm_path(n, d_in, d_out) == B.GEMM_FP4
        in_bytes = n * 8 * ((d_in + 63) // 64) if not (small and l == 0 and cfg.model == "gcn") else n * 4 * d_in
        hbm_bytes = in_bytes + n * row_bytes * products
        peak_ops = MFMA_FP4_MAC_PEAK if fp4 else VALU_BINARY_MAC_PEAK
        t_hbm, t_ops = hbm_bytes / (HBM_PEAK_GBPS * 1e9), macs / peak_ops
        if t_hbm >= t_ops:
            slots.append({"slot": f"bit_gemm[{l}]", "ms": t * 1e3, "bound": "hbm", "algorithmic_bytes": hbm_bytes,
                          "achieved": hbm_bytes / t / 1e9, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                          "frac": hbm_bytes / t / 1e9 / HBM_PEAK_GBPS, "path": "fp4-mfma" if fp4 else "xor-popcount"})
        else:
            slots.append({"slot": f"bit_gemm[{l}]", "ms": t * 1e3, "bound": "mfma" if fp4 else "alu", "binary_macs": macs,
                          "achieved": macs / t / 1e12, "peak": peak_ops / 1e12, "unit": "T binary MAC/s",
                          "frac": macs / t / peak_ops, "path": "fp4-mfma" if fp4 else "xor-popcount"})
        gather, minimum, row_bytes = aggregation_bytes(cfg, nnz, l, B)
        t = launch_ms[2 + 2 * l] * 1e-3
        slots.append({"slot": f"aggregation[{l}]", "ms": t * 1e3, "bound": "hbm", "algorithmic_bytes": gather,
                      "achieved": gather / t / 1e9, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                      "frac": gather / t / 1e9 / HBM_PEAK_GBPS, "row_bytes": row_bytes,
                      "compulsory_bytes": minimum, "compulsory_GBps": minimum / t / 1e9,
                      "rows_fit_infinity_cache": n * row_bytes <= INFINITY_CACHE_BYTES})
    return slots


def time_forward(m, n_layers, steps, warmup, graph, B):
    """ms per forward (mean, median, min where available) and mean ms per launch slot.  Eager:
    every step is event-bracketed per launch inside the timed region.  Graph: one forward is
    captured in a HIP graph and `steps` replays are timed; the per-launch figures then come from a
    separate eager, event-bracketed pass of min(steps, 200) forwards."""
    import torch

    def step(prof=None):
        m["forward"](m["plan"], m["row_ptr"], m["col_idx"], m["dinv"], m["x"], m["layers"],
                     m["workspace"], m["logits"], prof)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    if graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
        torch.cuda.current_stream().wait_stream(side)
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            step()
        g.replay()
        torch.cuda.synchronize()
        start.record()
        for _ in range(steps):
            g.replay()
        stop.record()
        torch.cuda.synchronize()
        ms = start.elapsed_time(stop) / steps
        eager_steps = min(steps, 200)
        profile = B.Profile(n_layers, eager_steps)
        for _ in range(eager_steps):
            step(profile)
        torch.cuda.synchronize()
        launch_ms, _ = profile.read()
        return {"ms": ms, "median": None, "min": None, "launch_ms": launch_ms, "launch": "hip graph replay"}
    profile = B.Profile(n_layers, steps)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    start.record()
    marks[0].record()
    for i in range(steps):
        step(profile)
        marks[i + 1].record()
    stop.record()
    torch.cuda.synchronize()
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(steps))
    launch_ms, calls = profile.read()
    assert calls == steps
    return {"ms": start.elapsed_time(stop) / steps, "median": per_step[len(per_step) // 2], "min": per_step[0],
            "launch_ms": launch_ms, "launch": "eager"}


def apply_cache_bound(slots, gather_ms):
    """An aggregation whose product rows fit the 256 MB Infinity Cache is gathered from there, so
    its algorithmic bytes over the HBM peak say nothing (they can exceed 1).  Such a launch is
    compared with the plain gather of the same cache lines on the same graph, measured in the same
    run (`gather_ms`, see gather_probe): the HBM figure is kept beside it as `algorithmic_GBps`."""
    for s in slots:
        if not s.get("rows_fit_infinity_cache"):
            continue
        t_plain = gather_ms[str(max(128, s["row_bytes"]))]
        s.update({"bound": "cache-resident gather (rows fit the 256 MB Infinity Cache; no published peak)",
                  "algorithmic_GBps": s["achieved"], "algorithmic_frac_of_hbm_peak": s["frac"],
                  "peak": s["algorithmic_bytes"] / (t_plain * 1e-3) / 1e9,
                  "peak_is": "the plain fp32 gather (bigcn_spmm, unit coefficients) of the same cache lines "
                             "on the same graph, measured in this run",
                  "frac": t_plain / s["ms"], "plain_gather_ms": t_plain})


def dominant_roofline(slots):
    """The `roofline` object of a workload: its slowest launch against its bound."""
    dom = max(slots, key=lambda s: s["ms"])
    r = {"bound": dom["bound"], "achieved": dom["achieved"], "peak": dom["peak"], "unit": dom["unit"],
         "frac": dom["frac"], "kernel": dom["slot"], "avg_launch_ms": dom["ms"]}
    for k in ("peak_is", "plain_gather_ms", "algorithmic_frac_of_hbm_peak"):
        if k in dom:
            r[k] = dom[k]
    return r


def config_leg(name, B, steps, warmup, graph):
    """One of the other workloads, timed in the same run: ms per forward, nodes/s, every launch
    against its bound and the workload's own `roofline` (its slowest launch)."""
    import torch
    from workloads import get_config, make_workload
    cfg = get_config(name)
    t0 = time.perf_counter()
    work = make_workload(cfg)
    m = build_model(work, B)
    log(f"[bench] {name}: generated and set up in {time.perf_counter() - t0:.1f} s")
    timing = time_forward(m, cfg.n_layers, steps, warmup, graph, B)
    slots = slot_bounds(cfg, work.n, work.nnz, B, timing["launch_ms"])
    gather_ms = None
    if any(s.get("rows_fit_infinity_cache") for s in slots):
        gather_ms = gather_probe(B, m, [max(128, s["row_bytes"]) for s in slots if s.get("rows_fit_infinity_cache")])
        apply_cache_bound(slots, gather_ms)
    leg = {"workload": f"{cfg.name}: {cfg.stands_in_for}-shaped, {work.n} nodes, {cfg.n_edges} edges, dims "
                       + "-".join(str(d) for d in cfg.dims),
           "ms_per_forward": timing["ms"], "ms_median": timing["median"], "ms_min": timing["min"],
           "nodes_per_s": work.n / (timing["ms"] * 1e-3), "launch": timing["launch"], "steps": steps,
           "launches": slots, "sum_of_launches_ms": sum(timing["launch_ms"]),
           "roofline": dominant_roofline(slots)}
    if gather_ms is not None:
        leg["plain_gather_ms_by_row_bytes"] = gather_ms
    del m
    torch.cuda.empty_cache()
    return leg


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
                    help="skip the back-propagation and Bi-GAT legs (timed alone, not part of a step)")
    ap.add_argument("--no-gemm-sweep", action="store_true",
                    help="skip the bit-GEMM leg outside the workloads (three evaluation paths at K = 4096, "
                         "the FP4 path over K, M=262144, n=256, and the multiply-only rate)")
    ap.add_argument("--gemm-sweep-only", action="store_true",
                    help="run only the bit-GEMM leg and print it (for counter collection)")
    ap.add_argument("--no-configs", action="store_true",
                    help="skip the legs of the other four workloads (c1-c3 as HIP-graph replays of 1000 "
                         "forwards, c4 eager) that a default run of c5 adds to its line")
    ap.add_argument("--probe", choices=["stream", "gather", "mfma"],
                    help="run only one probe and print it: streaming rates of the box, the plain gather "
                         "by row width on the workload's graph, or the multiply-only matrix-core rate")
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
    if args.probe == "stream":
        print(json.dumps({"stream_probe": stream_probe(B=B)}), flush=True)
        return
    if args.probe == "mfma":
        print(json.dumps({"multiply_only": multiply_only_probe(B)}), flush=True)
        return
    cfg = get_config(args.workload)
    t0 = time.perf_counter()
    work = make_workload(cfg)
    log(f"[bench] generated {cfg.name}: {work.n} nodes, nnz {work.nnz} in {time.perf_counter() - t0:.1f} s")
    t0 = time.perf_counter()
    m = build_model(work, B)
    log(f"[bench] set-up (upload, plan, weights, calibration) {time.perf_counter() - t0:.1f} s")
    if args.probe == "gather":
        print(json.dumps({"workload": cfg.name, "plain_gather_ms_by_row_bytes": gather_probe(B, m, [32, 64, 128, 256])}),
              flush=True)
        return
    if args.copy_probe_mib > 0:
        src = torch.ones((args.copy_probe_mib << 18,), dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)                      # one elementwise copy kernel: reads and writes MiB each
        torch.cuda.synchronize()
        log(f"[bench] copy probe: {args.copy_probe_mib} MiB read + {args.copy_probe_mib} MiB written")
        del src, dst
    n_layers = cfg.n_layers
    steps, warmup = max(1, args.steps), max(0, args.warmup)
    timing = time_forward(m, n_layers, steps, warmup, args.graph, B)
    ms_per_step = timing["ms"]
    launch_ms = timing["launch_ms"]

    nodes_per_s = work.n / (ms_per_step * 1e-3)
    slots = slot_bounds(cfg, work.n, work.nnz, B, launch_ms)
    gemm = [s for s in slots if s["slot"].startswith("bit_gemm")]
    spmm = [s for s in slots if s["slot"].startswith("aggregation")]
    for l, g in enumerate(gemm):
        macs = work.n * cfg.dims[l] * cfg.dims[l + 1] * (2 if cfg.model == "sage" else 1)
        g["binary_op_per_s"] = macs / (g["ms"] * 1e-3)
    gather_widths = [max(128, s["row_bytes"]) for s in spmm]
    gather_ms = gather_probe(B, m, gather_widths)
    apply_cache_bound(slots, gather_ms)
    roofline = dominant_roofline(slots)
    dom = max(slots, key=lambda s: s["ms"])
    if dom["slot"].startswith("aggregation"):
        # What this figure is and is not.  `achieved` is algorithmic gather bytes (no reuse assumed)
        # over the launch time, as a fraction of the published HBM peak.  The only memory counters
        # rocprofv3 offers on this machine (FETCH_SIZE / WRITE_SIZE = TCC_EA0_RDREQ* / WRREQ*) sit on the
        # L2-to-fabric boundary; none sees the memory controllers or the Infinity Cache, so the share
        # of these bytes that the 256 MB memory-side cache served instead of HBM cannot be measured.
        model = infinity_cache_model(work.row_ptr, dom["row_bytes"])
        hbm_est = dom["algorithmic_bytes"] - model["hit_rate"] * work.nnz * dom["row_bytes"]
        roofline.update({
            "measured_at": "algorithmic bytes; the counter-measured traffic (`traffic`) is bytes across the "
                           "L2-to-fabric boundary = HBM + Infinity Cache; no counter on this box sees HBM alone",
            "algorithmic_bytes_per_launch": dom["algorithmic_bytes"],
            "rows_fit_infinity_cache": dom["rows_fit_infinity_cache"],
            "hbm_side": {"compulsory_bytes": dom["compulsory_bytes"], "compulsory_GBps": dom["compulsory_GBps"],
                         "compulsory_frac_of_hbm_peak": dom["compulsory_GBps"] / HBM_PEAK_GBPS,
                         "infinity_cache_model": model,
                         "modelled_hbm_bytes": hbm_est,
                         "modelled_hbm_GBps": hbm_est / (dom["ms"] * 1e-3) / 1e9,
                         "modelled_frac_of_hbm_peak": hbm_est / (dom["ms"] * 1e-3) / 1e9 / HBM_PEAK_GBPS}})
    traffic = measured_traffic(cfg.name)
    roofline["traffic"] = None if traffic is None else traffic["bytes"]
    if traffic is not None:
        roofline["traffic_source"] = {k: v for k, v in traffic.items() if k != "bytes"}
        roofline["traffic_source"]["file"] = os.path.relpath(TRAFFIC_FILE, ROOT)
    roofline["plain_gather_ms_by_row_bytes"] = gather_ms
    if dom["slot"].startswith("aggregation") and gather_ms and str(max(128, dom["row_bytes"])) in gather_ms:
        # the same launch against the plain fp32 gather of the same cache lines (no conversions, no
        # epilogue), measured in this run: what the memory system gives this access pattern
        plain = gather_ms[str(max(128, dom["row_bytes"]))]
        roofline["frac_of_plain_gather"] = plain / dom["ms"]
        roofline["l2_miss_rate_limit_note"] = ("gathers on this box are bound by the rate at which L2 misses are served "
                                               "(7-7.6 TB/s from the Infinity Cache or HBM alike; profiles/spmm_fused_c5.md)")
    roofline["stream_probe"] = stream_probe(B=B)

    fp4_ran = any(g.get("path") == "fp4-mfma" for g in gemm)
    result = {
        "metric": "Bi-GCN forward nodes/s; bit-GEMM binary-op/s; SpMM HBM GB/s (% roofline)",
        "model": "Bi-GCN" if cfg.model == "gcn" else "Bi-GraphSAGE (mean aggregator)",
        "value": nodes_per_s, "unit": "nodes/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": ms_per_step, "ms_per_step_median": timing["median"], "ms_per_step_min": timing["min"],
        "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None,
        "dtype": ("fp4-mfma +-1 products (exact integers in f32 accumulators) + f32 aggregation" if fp4_ran
                  else "u64 xor/popcount products (int32, exact) + f32 aggregation"),
        "data": "synthetic", "launch": timing["launch"],
        "config": {"workload": f"{cfg.name}: {cfg.stands_in_for}-shaped Chung-Lu graph, {work.n} nodes, "
                               f"{cfg.n_edges} undirected edges "
                               + ("(+ self-loops), Bi-GCN, dims " if cfg.model == "gcn" else
                                  "(neighbour lists), Bi-GraphSAGE mean aggregator, dims ")
                               + "-".join(str(d) for d in cfg.dims),
                   "layers": n_layers, "nnz": work.nnz, "standardisation": cfg.bn_layers},
        "launches": slots,
        "bit_gemm": gemm, "spmm": spmm,
        "bit_gemm_binary_op_per_s": max(g["binary_op_per_s"] for g in gemm),
        "spmm_GBps": roofline["achieved"],
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
        result["gat_hidden_layer"] = gat_leg(B, m, cfg, hidden=True)
    del m
    torch.cuda.empty_cache()
    if not args.no_gemm_sweep:
        sweep = gemm_sweep(B)
        result["bit_gemm_sweep"] = sweep
        best = max(sweep["paths"], key=lambda r: r["binary_op_per_s"])
        result["bit_gemm_binary_op_per_s"] = max(result["bit_gemm_binary_op_per_s"], best["binary_op_per_s"])
        # the bit-GEMM target is stated on the path the automatic choice takes for such shapes
        # (FP4 matrix cores) against the published FP4 peak: visible beside the headline roofline
        roofline["bit_gemm"] = {"bound": "mfma", "chosen_path": "mfma_fp4", "peak": MFMA_FP4_MAC_PEAK / 1e12,
                                "unit": "T binary MAC/s",
                                "by_k_bits": {str(r["k_bits"]): {"achieved": r["binary_op_per_s"] / 1e12,
                                                                 "frac": r["frac_mfma_fp4_peak"],
                                                                 "frac_of_multiply_only_rate": r["frac_of_multiply_only_rate"],
                                                                 "frac_of_expand_and_multiply_rate": r["frac_of_expand_and_multiply_rate"]}
                                              for r in sweep["paths"] if r["path"] == "mfma_fp4"},
                                "multiply_only_frac_of_peak": sweep["multiply_only"]["frac_mfma_fp4_peak"],
                                "expand_and_multiply_frac_of_peak": sweep["multiply_only"]["with_expansion"]["frac_mfma_fp4_peak"],
                                "ceiling_is": "a launch of nothing but the expansion of packed bits to FP4 codes and the "
                                              "multiplies, the codes of a step built between the multiplies of the step "
                                              "before (bigcn_probe_fp4_expand_multiply_rate): what a kernel fed with "
                                              "bit-packed operands could reach if loads and stores were free",
                                "target_0p5_met": best["frac_mfma_fp4_peak"] >= 0.5}
    if not args.no_configs and args.workload == "c5":
        legs = {}
        for name in ("c1", "c2", "c3"):
            legs[name] = config_leg(name, B, steps=1000, warmup=20, graph=True)
        legs["c4"] = config_leg("c4", B, steps=steps, warmup=warmup, graph=False)
        result["configs"] = legs
        roofline["per_config"] = {name: {"ms_per_forward": leg["ms_per_forward"], "nodes_per_s": leg["nodes_per_s"],
                                         "launch": leg["launch"],
                                         **{k: leg["roofline"][k] for k in ("bound", "kernel", "achieved", "peak", "unit", "frac")}}
                                  for name, leg in legs.items()}
    if args.cpu_baseline_nodes != 0:
        t0 = time.perf_counter()
        whole = 400000 if cfg.name == "s5" else cfg.n_nodes
        sample = whole if args.cpu_baseline_nodes < 0 else min(args.cpu_baseline_nodes, cfg.n_nodes)
        result["cpu_baseline"] = cpu_baseline(work, sample)
        log(f"[bench] cpu_baseline leg {time.perf_counter() - t0:.1f} s")
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
