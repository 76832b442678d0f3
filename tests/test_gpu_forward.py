"""End-to-end parity of the fused forward against the CPU oracle, through the C ABI.

The first three workloads run at full size; the two large ones run on a scaled-down graph of
the same recipe here and at full size in test_gpu_full_size.py.  The comparison is layer by
layer (helpers.compare_forward_layerwise): every layer's output is checked on all rows whose
inputs were bit-identical on both sides.
"""
import numpy as np
import pytest

import oracle
from helpers import assert_close, close, compare_forward_layerwise, compare_forward_teacher_forced, to_device
from workloads import get_config, make_workload, scaled_config

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import torch
    from paper_2210_13149_amd import binding
    assert torch.cuda.is_available()
    binding.lib()
    return binding


def calibration_spec(work):
    """Which layers standardise their input (first layer only, or every layer, as the workload
    prescribes); the parameters themselves are computed by the oracle during the comparison."""
    cfg = work.config
    return ["calibrate"] + ["calibrate" if cfg.bn_layers == "all" else None] * (cfg.n_layers - 1)


def calibrated_bn(work):
    """Frozen standardisation parameters per layer, computed by the oracle from its own
    activations."""
    calibrate = [p == "calibrate" for p in calibration_spec(work)]
    _, recs = oracle.forward(work.row_ptr, work.col_idx, work.x, work.weights, calibrate=calibrate)
    return [(r["shift"], r["mul"]) if r["shift"] is not None else None for r in recs]


def gpu_prefix_runner(B, work):
    """run(l, params): fused forward over the first l layers with params[:l] as standardisation."""
    import torch
    drp, dci, dx = to_device(work.row_ptr, work.col_idx, work.x)
    dweights = [to_device(w) for w in work.weights]
    plan = B.Plan(drp, dci)
    dinv, _ = B.bigcn_gcn_norm(drp, dci)
    layers = []

    def run(l, params):
        while len(layers) < l:
            p = params[len(layers)]
            shift, mul = (None, None) if p is None else tuple(to_device(*p))
            layers.append(B.Layer.from_weight(dweights[len(layers)], shift, mul))
        out = B.bigcn_forward(plan, drp, dci, dinv, dx, layers[:l])
        torch.cuda.synchronize()
        return out.cpu().numpy()

    return run


@pytest.mark.parametrize("name,n_scaled", [("c1", None), ("c2", None), ("c3", None),
                                           ("c4", 6000), ("c5", 30000)])
def test_forward_matches_oracle(B, name, n_scaled):
    cfg = get_config(name) if n_scaled is None else scaled_config(name, n_scaled)
    work = make_workload(cfg)
    teacher = compare_forward_teacher_forced(work, calibration_spec(work), gpu_prefix_runner(B, work))
    assert all(t['rows_compared'] == work.n for t in teacher)
    stats = compare_forward_layerwise(work, calibration_spec(work), gpu_prefix_runner(B, work))
    print(name, stats)
    # a legal sign flip removes its two-hop neighbourhood from the comparison of later layers;
    # most rows must still take part in the comparison of the logits
    assert stats[-1]["rows_compared"] >= 0.9 * work.n


def test_forward_without_standardisation_and_repeatability(B):
    import torch
    work = make_workload(scaled_config("c5", 5000))
    bn = [None] * work.config.n_layers
    run = gpu_prefix_runner(B, work)
    teacher = compare_forward_teacher_forced(work, bn, gpu_prefix_runner(B, work))
    assert all(t["rows_compared"] == work.n for t in teacher)
    stats = compare_forward_layerwise(work, bn, run)
    # mean degree 50 on 5000 nodes: one legal sign flip reaches a quarter of the graph in two hops
    assert stats[-1]["rows_compared"] >= 0.5 * work.n
    a, b = run(work.config.n_layers, bn), run(work.config.n_layers, bn)
    assert np.array_equal(a, b)


def test_bigcn_model_wrapper_reuses_buffers(B):
    import torch
    work = make_workload("c1")
    bn = calibrated_bn(work)
    drp, dci, dx = to_device(work.row_ptr, work.col_idx, work.x)
    model = B.BiGCN(drp, dci, [to_device(w) for w in work.weights],
                    [None if p is None else tuple(to_device(*p)) for p in bn])
    first = model.forward(dx).clone()
    second = model.forward(dx)
    assert torch.equal(first, second) and second.data_ptr() == model.logits.data_ptr()
    # the wrapper is the plain entry point on buffers it keeps: same bits as bigcn_forward, whose
    # result the layer-by-layer comparisons of this file hold to the oracle
    direct = B.bigcn_forward(model.plan, drp, dci, model.dinv_sqrt, dx, model.layers)
    assert torch.equal(first, direct)
    ref, _ = oracle.forward(work.row_ptr, work.col_idx, work.x, work.weights, bn=bn)
    assert close(first.cpu().numpy(), ref).all(axis=1).mean() >= 0.99


def test_forward_layer_chain_equals_separate_kernels(B):
    """pack -> binary_gemm -> spmm through the public entry points gives the same first-layer
    activations as the fused driver (both against the oracle)."""
    import torch
    work = make_workload("c3")
    bn = calibrated_bn(work)
    shift, mul = bn[0]
    drp, dci, dx, dw, dshift, dmul = to_device(work.row_ptr, work.col_idx, work.x, work.weights[0],
                                               shift, mul)
    plan = B.Plan(drp, dci)
    bits, beta = B.bigcn_pack(dx, dshift, dmul)
    wbits, alpha = B.pack_weight(dw)
    _, zeta = B.bigcn_binary_gemm(bits, beta, wbits, alpha, work.x.shape[1], want_acc=False)
    _, vals = B.bigcn_gcn_norm(drp, dci, want_vals=True)
    h1 = B.bigcn_spmm(plan, drp, dci, vals, zeta).cpu().numpy()
    a_tilde = oracle.gcn_norm(work.row_ptr, work.col_idx)
    rec = oracle.layer(work.row_ptr, work.col_idx, a_tilde, work.x, work.weights[0], shift, mul)
    assert_close(h1, rec["out"], "H1 through separate kernels")


@pytest.mark.parametrize("d_in", [64, 100, 127, 128, 129, 200, 254, 255, 256, 257, 602, 1023, 1024, 1025, 2048, 2049])
def test_forward_extreme_products(B, d_in):
    """Nodes whose sign pattern equals, or is the exact opposite of, a weight column give the
    extreme products +K and -K: the ends of the range of every compact product-row format
    (seven bits per product up to K = 128 with the scale in the spare top bits; up to K = 256 the
    same form for rows that fit it and one byte per product in the alternate array for rows that
    do not, which these inputs produce in numbers; up to K = 1024 again that form, with fp16
    alternates; the last input bit carried separately at K = 128 and K = 256; plain fp16 rows up
    to K = 2048; fp32 beyond)."""
    _extreme_products(B, d_in, 256)


@pytest.mark.parametrize("d_in,d_hidden", [(100, 128), (128, 128), (200, 100), (256, 128), (64, 96),
                                           (300, 128), (1024, 90), (513, 20), (700, 3)])
def test_forward_extreme_products_rows_of_sixteen_lanes(B, d_in, d_hidden):
    """The same with 80 to 128 hidden columns: product rows of 16 lanes, which carry two bits of
    the scale per lane; layers of 257..1024 input bits use such rows for any narrower output too."""
    _extreme_products(B, d_in, d_hidden)


@pytest.mark.parametrize("d_in,d_hidden,n", [(100, 40, 400), (128, 47, 400), (200, 56, 400), (256, 60, 400),
                                             (255, 61, 400), (64, 41, 400), (256, 47, 33000),
                                             (100, 60, 33000)])
def test_forward_extreme_products_rows_of_eight_lanes(B, d_in, d_hidden, n):
    """The same with 40 to 60 hidden columns and at most 256 input bits: 64-byte rows of 8 lanes
    whose scale is spread over the last value of the last four lanes (61 columns: widened to 16
    lanes with the scale in the tail, as before)."""
    _extreme_products(B, d_in, d_hidden, n=n, n_edges=3000 if n < 1000 else 150000)


@pytest.mark.parametrize("d_in,d_hidden", [(100, 256), (128, 100), (200, 256), (256, 256), (256, 128),
                                           (602, 128), (1024, 300), (2049, 64), (200, 70), (64, 75),
                                           (255, 200), (65, 256), (192, 160), (512, 512), (600, 400),
                                           (1024, 256), (700, 200), (257, 90), (100, 512)])
def test_forward_extreme_products_many_rows(B, d_in, d_hidden):
    """The same on 33000 nodes: beyond 32768 rows the bit-GEMM runs its kernels for large row
    counts (the matrix-core row kernel for rows of 128, 256 or 512 one-byte values up to 1024 input
    bits, with the scale in the top bits, in the row's tail (70 and 75 columns) or separate, and
    one-byte or fp16 alternates; the vector-ALU kernels where the weights of a layer do not fit
    its LDS budget (1024 bits x 300 columns) and for fp16 and fp32 rows), which must take the same
    per-row decisions."""
    _extreme_products(B, d_in, d_hidden, n=33000, n_edges=150000)


@pytest.mark.parametrize("d_in,d_hidden", [(200, 256), (512, 128)])
def test_forward_every_row_outside_seven_bits_many_rows(B, d_in, d_hidden):
    """Every node equals (or opposes) a weight column: all 33000 product rows of the first layer
    leave the 7-bit form and take the alternate array (one-byte and fp16), in the bit-GEMM and in
    the aggregation."""
    _extreme_products(B, d_in, d_hidden, n=33000, n_edges=150000, planted=33000)


def _hidden_escape_workload(d_hidden, d_next, n, n_edges, with_columns, seed):
    """dims 64 -> d_hidden -> d_next -> 5 whose second weight matrix has (with_columns) or has not
    40 columns equal to the hidden sign pattern of a node (alternately its opposite): products of
    +-d_hidden in the second layer."""
    from workloads import chung_lu_csr
    from workloads.build import Workload
    from workloads.configs import WorkloadConfig
    rng = np.random.default_rng(seed)
    dims = (64, d_hidden, d_next, 5)
    rp, ci = chung_lu_csr(n, n_edges, 2.5, 2.0, seed=seed)
    ws = [rng.uniform(-1, 1, size=(dims[i], dims[i + 1])).astype(np.float32) for i in range(3)]
    x = rng.standard_normal((n, 64)).astype(np.float32)
    if with_columns:
        h1 = oracle.layer(rp, ci, oracle.gcn_norm(rp, ci), x, ws[0], None, None)["out"]
        # the nodes whose hidden values stay farthest from zero: no sign of theirs is in doubt
        nodes = np.argsort(-np.abs(h1[:2000]).min(axis=1))[:40]
        for j in range(40):
            pattern = np.where(h1[nodes[j]] >= 0, 1.0, -1.0) * (1 if j % 2 == 0 else -1)
            ws[1][:, j] = (pattern * np.abs(ws[1][:, j]).clip(min=0.05)).astype(np.float32)
    cfg = WorkloadConfig("hidden-extreme", "none", n, n_edges, 2.0, dims, "normal", 1.0, "first", 0)
    return Workload(cfg, rp, ci, x, ws)


@pytest.mark.parametrize("d_hidden,d_next,n", [(200, 256, 3000), (512, 128, 3000), (200, 256, 33000),
                                               (512, 512, 33000)])
def test_rows_outside_seven_bits_in_a_hidden_layer(B, d_hidden, d_next, n):
    """Product rows of the second layer that leave the 7-bit form (one-byte and fp16 alternates).
    From the second layer on the bit-GEMM reports such rows through a flag and the aggregation
    only tests its rows when the flag is set: the same buffers run a model with such rows, then
    one without, then the first again, and every result must equal the first of its kind bit for
    bit and match the oracle."""
    import torch
    with_rows = _hidden_escape_workload(d_hidden, d_next, n, 5 * n, True, seed=d_hidden + n)
    without = _hidden_escape_workload(d_hidden, d_next, n, 5 * n, False, seed=d_hidden + n)
    assert np.array_equal(with_rows.x, without.x) and np.array_equal(with_rows.col_idx, without.col_idx)
    _, recs = oracle.forward(with_rows.row_ptr, with_rows.col_idx, with_rows.x, with_rows.weights,
                             bn=[None] * 3, keep_trace=True)
    assert recs[1]["acc"].max() == d_hidden and recs[1]["acc"].min() == -d_hidden
    _, recs = oracle.forward(without.row_ptr, without.col_idx, without.x, without.weights, bn=[None] * 3,
                             keep_trace=True)
    assert np.abs(recs[1]["acc"]).max() < 128                 # every product of the plain model fits 7 bits
    del recs
    for work in (with_rows, without):
        teacher = compare_forward_teacher_forced(work, [None] * 3, gpu_prefix_runner(B, work), own_sum_bound=True)
        assert all(t['rows_compared'] == work.n for t in teacher)
        stats = compare_forward_layerwise(work, [None] * 3, gpu_prefix_runner(B, work), cancellation_aware=True)
        assert stats[1]["rows_compared"] >= 0.9 * n
    # one set of buffers, alternating models
    drp, dci, dx = to_device(with_rows.row_ptr, with_rows.col_idx, with_rows.x)
    plan = B.Plan(drp, dci)
    dinv, _ = B.bigcn_gcn_norm(drp, dci)
    layers = {name: [B.Layer.from_weight(to_device(w)) for w in work.weights]
              for name, work in (("with", with_rows), ("without", without))}
    need = max(B.bigcn_forward_workspace_bytes(n, layers["with"]), B.bigcn_forward_workspace_bytes(n, layers["without"]))
    workspace = torch.empty(need + 256, dtype=torch.uint8, device="cuda")
    first = {}
    for name in ("with", "without", "with", "without", "without", "with"):
        out = B.bigcn_forward(plan, drp, dci, dinv, dx, layers[name], workspace=workspace)
        torch.cuda.synchronize()
        if name in first:
            assert torch.equal(out, first[name]), name
        else:
            first[name] = out.clone()
    plan.destroy()


def _extreme_products(B, d_in, d_hidden, n=400, n_edges=3000, planted=120):
    from workloads import chung_lu_csr
    from workloads.build import Workload
    from workloads.configs import WorkloadConfig
    rng = np.random.default_rng(d_in + 7 * d_hidden)
    d_out = 5
    rp, ci = chung_lu_csr(n, n_edges, 2.5, 2.0, seed=d_in)
    w0 = rng.uniform(-1, 1, size=(d_in, d_hidden)).astype(np.float32)
    w1 = rng.uniform(-1, 1, size=(d_hidden, d_out)).astype(np.float32)
    x = rng.standard_normal((n, d_in)).astype(np.float32)
    for k in range(0, planted):
        j = (7 * k) % d_hidden
        x[k] = w0[:, j] if k % 2 == 0 else -w0[:, j]      # products +K / -K in column j
    if planted + 2 <= n:
        x[planted] = np.abs(x[planted])                     # all +1
        x[planted + 1] = -np.abs(x[planted + 1]) - 1e-3     # all -1
    cfg = WorkloadConfig("extreme", "none", n, n_edges, 2.0, (d_in, d_hidden, d_out), "normal", 1.0,
                         "first", 0)
    work = Workload(cfg, rp, ci, x, [w0, w1])
    bn = [None, None]
    _, recs = oracle.forward(rp, ci, x, [w0, w1], bn=bn, keep_trace=True)
    assert recs[0]["acc"].max() == d_in and recs[0]["acc"].min() == -d_in
    teacher = compare_forward_teacher_forced(work, bn, gpu_prefix_runner(B, work), own_sum_bound=True)
    assert all(t['rows_compared'] == work.n for t in teacher)
    stats = compare_forward_layerwise(work, bn, gpu_prefix_runner(B, work), cancellation_aware=True)
    assert stats[-1]["rows_compared"] >= 0.5 * n


def _hand_graph(kind):
    from workloads import csr_from_undirected_edges
    if kind == "single":                      # one node: only its self-loop
        return csr_from_undirected_edges(1, np.zeros(0, dtype=np.int64), np.zeros(0, dtype=np.int64))
    if kind == "isolated":                    # no edges at all: A~ is the identity
        return csr_from_undirected_edges(70, np.zeros(0, dtype=np.int64), np.zeros(0, dtype=np.int64))
    if kind == "star":                        # one hub of 1500 neighbours: a row shared by a workgroup
        return csr_from_undirected_edges(1501, np.zeros(1500, dtype=np.int64), np.arange(1, 1501, dtype=np.int64))
    if kind == "path":
        return csr_from_undirected_edges(130, np.arange(129, dtype=np.int64), np.arange(1, 130, dtype=np.int64))
    raise ValueError(kind)


@pytest.mark.parametrize("kind", ["single", "isolated", "star", "path"])
@pytest.mark.parametrize("dims", [(7, 3), (100, 512, 512, 10), (70, 64, 1), (256, 128, 47), (100, 56, 60),
                                  (200, 40, 41)])
def test_forward_on_degenerate_graphs_and_extreme_widths(B, kind, dims):
    """Hand-built graphs (one node, no edges, a star whose hub row is shared by a workgroup, a path)
    with the narrowest and the widest layers the fused forward takes (1 and 512 columns)."""
    from workloads.build import Workload
    from workloads.configs import WorkloadConfig
    from workloads.features import make_weights
    rp, ci = _hand_graph(kind)
    n = rp.size - 1
    rng = np.random.default_rng(len(kind) + sum(dims))
    x = rng.standard_normal((n, dims[0])).astype(np.float32)
    weights = make_weights(dims, rng)
    cfg = WorkloadConfig(kind, "none", n, (ci.size - n) // 2, 2.0, tuple(dims), "normal", 1.0, "first", 0)
    work = Workload(cfg, rp, ci, x, weights)
    bn = [None] * (len(dims) - 1)
    teacher = compare_forward_teacher_forced(work, bn, gpu_prefix_runner(B, work), own_sum_bound=True)
    assert all(t['rows_compared'] == work.n for t in teacher)
    stats = compare_forward_layerwise(work, bn, gpu_prefix_runner(B, work), cancellation_aware=True)
    assert stats[0]["rows_compared"] == n
    if kind == "isolated":
        # A~ = I: the logits of the last layer are the node's own rescaled products
        out = gpu_prefix_runner(B, work)(1, bn)
        sign, beta = oracle.binarize_rows(x)
        bt, alpha = oracle.binarize_weight(weights[0])
        assert_close(out, oracle.rescale(oracle.sign_matmul(sign, bt), beta, alpha), "identity aggregation")


@pytest.mark.parametrize("name", ["c1", "c3"])
def test_forward_captured_in_a_hip_graph_replays_identically(B, name):
    """The fused forward allocates nothing, clears no memory and only launches kernels on the
    caller's stream, so it can be captured once and replayed: every replay, with eager work and
    synchronisation between replays and with new feature values in the same buffers, must equal
    the eager result bit for bit."""
    import torch
    work = make_workload(name)
    bn = calibrated_bn(work)
    drp, dci, dx = to_device(work.row_ptr, work.col_idx, work.x)
    model = B.BiGCN(drp, dci, [to_device(w) for w in work.weights],
                    [None if p is None else tuple(to_device(*p)) for p in bn])
    eager = model.forward(dx).clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        model.forward(dx)                         # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        model.forward(dx)
    for rep in range(4):
        model.logits.fill_(float("nan"))          # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(model.logits, eager), f"replay {rep} differs from the eager forward"
    # new inputs in the captured buffers
    dx.mul_(-0.5).add_(0.01)
    want = None
    graph.replay()
    torch.cuda.synchronize()
    got = model.logits.clone()
    want = model.forward(dx).clone()
    assert torch.equal(got, want)
