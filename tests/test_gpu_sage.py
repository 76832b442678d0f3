"""Parity of the Bi-GraphSAGE path (mean aggregator, Sec. 4.4.2) against the CPU oracle, through
the C ABI: the degree coefficients, plan validation for neighbour lists, and the fused forward
layer by layer (helpers.compare_forward_layerwise) on scaled-down versions of the two workloads
and on small graphs that cover every product-row format, empty rows and the folded last bit."""
import numpy as np
import pytest

import oracle
from helpers import compare_forward_layerwise, compare_forward_teacher_forced, to_device
from workloads import chung_lu_csr, make_workload, scaled_config
from workloads.build import Workload
from workloads.configs import WorkloadConfig
from workloads.features import make_weights

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import torch
    from paper_2210_13149_amd import binding
    assert torch.cuda.is_available()
    binding.lib()
    return binding


def sage_prefix_runner(B, work):
    """run(l, params): fused Bi-GraphSAGE forward over the first l layers."""
    import torch
    drp, dci, dx = to_device(work.row_ptr, work.col_idx, work.x)
    dweights = [(to_device(ws), to_device(wn)) for ws, wn in work.weights]
    plan = B.Plan(drp, dci, validate=B.VALIDATE_NEIGHBOURS)
    inv_deg = B.bigcn_mean_norm(drp)
    layers = []

    def run(l, params):
        while len(layers) < l:
            p = params[len(layers)]
            shift, mul = (None, None) if p is None else tuple(to_device(*p))
            ws, wn = dweights[len(layers)]
            layers.append(B.SageLayer.from_weights(ws, wn, shift, mul))
        out = B.bigcn_sage_forward(plan, drp, dci, inv_deg, dx, layers[:l])
        torch.cuda.synchronize()
        return out.cpu().numpy()

    return run


def small_sage_workload(n, n_edges, dims, seed, i0=2.0, gamma=2.5):
    rng = np.random.Generator(np.random.PCG64([seed, 7]))
    rp, ci = chung_lu_csr(n, n_edges, gamma, i0, seed=seed, self_loops=False)
    x = rng.standard_normal((n, dims[0])).astype(np.float32)
    weights = list(zip(make_weights(dims, rng), make_weights(dims, rng)))
    cfg = WorkloadConfig(f"sage-{seed}", "none", n, n_edges, i0, tuple(dims), "normal", 1.0, "all", seed,
                         model="sage")
    return Workload(cfg, rp, ci, x, weights)


def test_mean_norm_matches_oracle_and_handles_empty_rows(B):
    rp, ci = chung_lu_csr(5000, 4000, 2.5, 2.0, seed=11, self_loops=False)
    deg = np.diff(rp)
    assert (deg == 0).any() and deg.max() > 64
    got = B.bigcn_mean_norm(to_device(rp)).cpu().numpy()
    want = np.where(deg > 0, 1.0 / np.maximum(deg, 1), 0.0)
    # one correctly rounded fp32 division
    assert np.array_equal(got, want.astype(np.float32))
    coeff = oracle.mean_norm(rp, ci)
    assert np.allclose(np.repeat(got, deg), coeff, rtol=6e-8, atol=0)


def test_plan_validation_modes(B):
    rp, ci = chung_lu_csr(300, 900, 2.5, 2.0, seed=5, self_loops=False)
    drp, dci = to_device(rp, ci)
    B.Plan(drp, dci, validate=B.VALIDATE_NEIGHBOURS).destroy()
    with pytest.raises(B.BigcnError) as err:
        B.Plan(drp, dci, validate=B.VALIDATE_GCN)            # no self-loops
    assert err.value.status == B.BIGCN_EGRAPH
    bad = ci.copy()
    bad[3] = 300                                             # out of range
    with pytest.raises(B.BigcnError) as err:
        B.Plan(drp, to_device(bad), validate=B.VALIDATE_NEIGHBOURS)
    assert err.value.status == B.BIGCN_EGRAPH
    row = int(np.argmax(np.diff(rp) >= 2))
    swapped = ci.copy()
    p = rp[row]
    swapped[p], swapped[p + 1] = swapped[p + 1], swapped[p]  # order broken
    with pytest.raises(B.BigcnError) as err:
        B.Plan(drp, to_device(swapped), validate=B.VALIDATE_NEIGHBOURS)
    assert err.value.status == B.BIGCN_EGRAPH
    with pytest.raises(B.BigcnError) as err:
        B.Plan(drp, dci, validate=7)
    assert err.value.status == B.BIGCN_EINVAL


@pytest.mark.parametrize("name,n_scaled", [("s4", 6000), ("s5", 20000)])
def test_sage_forward_matches_oracle(B, name, n_scaled):
    work = make_workload(scaled_config(name, n_scaled))
    assert work.config.model == "sage" and not (work.col_idx == np.repeat(
        np.arange(work.n), np.diff(work.row_ptr))).any()
    bn = ["calibrate"] * work.config.n_layers
    stats = compare_forward_layerwise(work, bn, sage_prefix_runner(B, work))
    print(name, stats)
    assert stats[0]["rows_compared"] == work.n
    assert stats[-1]["rows_compared"] >= 0.9 * work.n


# d_in / d_out pairs chosen to reach: one-byte rows with and without the embedded scale (in the
# row's tail, or in the spare top bits when d_in <= 128), the folded last bit (d_in = 128, 256), fp16 rows, fp32 rows, rows as wide as a wavefront (d_out = 512), and
# graphs with empty rows and rows long enough for the workgroup-per-row path.
@pytest.mark.parametrize("dims,n,n_edges,i0", [
    ((64, 40, 7), 3000, 2500, 2.0),
    ((100, 256, 47), 3000, 40000, 1.2),
    ((255, 256, 256, 5), 2000, 9000, 2.0),
    ((257, 300, 12), 2000, 9000, 2.0),
    ((130, 512, 512, 9), 1500, 30000, 1.1),
    ((2100, 33, 64, 3), 1200, 5000, 2.0),
    ((128, 300, 128, 256, 4), 1500, 30000, 1.1),
    ((100, 47, 41), 3000, 40000, 1.2),
    ((256, 60, 40, 56), 2000, 9000, 2.0),
])
def test_sage_forward_formats_and_edge_cases(B, dims, n, n_edges, i0):
    # the dense cases get a heavier tail: rows on both sides of the workgroup-per-row threshold (1024)
    work = small_sage_workload(n, n_edges, dims, seed=sum(dims), i0=i0, gamma=2.1 if i0 < 1.5 else 2.5)
    deg = np.diff(work.row_ptr)
    if n_edges < n:
        assert (deg == 0).any()
    if i0 < 1.5:
        assert deg.max() >= 1024 and ((deg >= 256) & (deg < 1024)).sum() >= 5
    for bn in (["calibrate"] * (len(dims) - 1), [None] * (len(dims) - 1)):
        stats = compare_forward_layerwise(work, bn, sage_prefix_runner(B, work))
        assert stats[0]["rows_compared"] == n
        assert stats[-1]["rows_compared"] >= 0.5 * n


@pytest.mark.parametrize("d_in", [129, 200, 256, 300, 1024])
def test_sage_rows_that_do_not_fit_seven_bits(B, d_in):
    """Nodes whose signs equal (or oppose) a column of W_theta or of W_n give products of +-K:
    their product rows, own and neighbour, take the escape path of layers with 129..1024 input
    bits (one-byte alternates up to 256 bits, fp16 alternates beyond)."""
    _sage_rows_that_do_not_fit(B, d_in, 256, 600, 4000)


@pytest.mark.parametrize("d_in,d_hidden", [(100, 128), (128, 256), (200, 256), (256, 256), (200, 72),
                                           (512, 512), (300, 100), (100, 512)])
def test_sage_rows_that_do_not_fit_seven_bits_many_rows(B, d_in, d_hidden):
    """The same on 33000 nodes, where both products of a layer are written by the matrix-core
    kernel (rows of 128, 256 and 512 stored values; scale in the top bits, in the row's tail, or
    separate; one-byte and fp16 alternates)."""
    _sage_rows_that_do_not_fit(B, d_in, d_hidden, 33000, 150000)


def _sage_rows_that_do_not_fit(B, d_in, d_hidden, n, n_edges):
    d_out = 6
    work = small_sage_workload(n, n_edges, (d_in, d_hidden, d_out), seed=900 + d_in)
    w_self, w_nbr = work.weights[0]
    for k in range(0, 200):
        src = w_self if k % 4 < 2 else w_nbr
        col = src[:, (11 * k) % d_hidden]
        work.x[k] = col if k % 2 == 0 else -col
    sign, _ = oracle.binarize_rows(work.x)
    bt, _ = oracle.binarize_weight(w_nbr)
    acc = oracle.sign_matmul(sign, bt)
    assert acc.max() == d_in and acc.min() == -d_in
    for bn in ([None, None], ["calibrate", "calibrate"]):
        teacher = compare_forward_teacher_forced(work, bn, sage_prefix_runner(B, work), own_sum_bound=True)
        assert all(t['rows_compared'] == work.n for t in teacher)
        stats = compare_forward_layerwise(work, bn, sage_prefix_runner(B, work), cancellation_aware=True)
        assert stats[0]["rows_compared"] == n and stats[-1]["rows_compared"] >= 0.5 * n
        if n > 10000:
            break                                             # one pass of the oracle is enough at this size


@pytest.mark.parametrize("d_hidden,n", [(200, 3000), (512, 33000)])
def test_sage_rows_outside_seven_bits_in_a_hidden_layer(B, d_hidden, n):
    """Columns of the second layer's two weight matrices equal the hidden sign pattern of a node:
    own and neighbour product rows of the second layer leave the 7-bit form, which from the second
    layer on is reported by the bit-GEMMs through a flag that the aggregation consults."""
    work = small_sage_workload(n, 5 * n, (64, d_hidden, 256, 5), seed=300 + d_hidden)
    coeff = oracle.mean_norm(work.row_ptr, work.col_idx)
    w_self0, w_nbr0 = work.weights[0]
    h1 = oracle.sage_layer(work.row_ptr, work.col_idx, coeff, work.x, w_self0, w_nbr0, None, None)["out"]
    nodes = np.argsort(-np.abs(h1[:2000]).min(axis=1))[:40]
    w_self1, w_nbr1 = (w.copy() for w in work.weights[1])
    for j in range(40):
        pattern = np.where(h1[nodes[j]] >= 0, 1.0, -1.0) * (1 if j % 2 == 0 else -1)
        target = w_self1 if j % 4 < 2 else w_nbr1
        target[:, j] = (pattern * np.abs(target[:, j]).clip(min=0.05)).astype(np.float32)
    work.weights[1] = (w_self1, w_nbr1)
    sign, _ = oracle.binarize_rows(h1)
    for w in (w_self1, w_nbr1):
        bt, _ = oracle.binarize_weight(w)
        acc = oracle.sign_matmul(sign, bt)
        assert acc.max() == d_hidden and acc.min() == -d_hidden
    teacher = compare_forward_teacher_forced(work, [None] * 3, sage_prefix_runner(B, work), own_sum_bound=True)
    assert all(t['rows_compared'] == work.n for t in teacher)
    stats = compare_forward_layerwise(work, [None] * 3, sage_prefix_runner(B, work), cancellation_aware=True)
    assert stats[1]["rows_compared"] >= 0.9 * n


def test_sage_isolated_node_output_is_its_own_term_and_runs_are_identical(B):
    import torch
    work = small_sage_workload(2000, 1200, (96, 128, 10), seed=77)
    deg = np.diff(work.row_ptr)
    lonely = np.flatnonzero(deg == 0)
    assert lonely.size > 0
    run = sage_prefix_runner(B, work)
    bn = [None, None]
    h1 = run(1, bn)
    sign, beta = oracle.binarize_rows(work.x)
    bt, alpha = oracle.binarize_weight(work.weights[0][0])
    own = oracle.rescale(oracle.sign_matmul(sign[lonely], bt), beta[lonely], alpha)
    assert np.allclose(h1[lonely], own, rtol=1e-5, atol=1e-6)
    a, b = run(2, bn), run(2, bn)
    assert np.array_equal(a, b)


def test_sage_model_wrapper_and_error_paths(B):
    import torch
    work = small_sage_workload(800, 3000, (70, 64, 6), seed=3)
    drp, dci, dx = to_device(work.row_ptr, work.col_idx, work.x)
    ref, used = oracle.sage_forward(work.row_ptr, work.col_idx, work.x, work.weights,
                                    calibrate=[True, True])
    model = B.BiGraphSAGE(drp, dci, [(to_device(a), to_device(b)) for a, b in work.weights],
                          [tuple(to_device(*p)) for p in used])
    first = model.forward(dx).clone()
    second = model.forward(dx)
    assert torch.equal(first, second) and second.data_ptr() == model.out.data_ptr()
    direct = B.bigcn_sage_forward(model.plan, drp, dci, model.inv_deg, dx, model.layers)
    assert torch.equal(first, direct)          # the wrapper is the plain entry point on kept buffers
    ok = np.abs(first.cpu().numpy() - ref) <= 1e-5 * np.abs(ref) + 1e-6
    assert ok.all(axis=1).mean() >= 0.99
    # workspace too small / wrong layer chain are reported, not executed
    with pytest.raises(B.BigcnError) as err:
        B.bigcn_sage_forward(model.plan, drp, dci, model.inv_deg, dx, model.layers,
                             workspace=torch.empty(256, dtype=torch.uint8, device="cuda"))
    assert err.value.status == B.BIGCN_EWORKSPACE
    with pytest.raises(B.BigcnError) as err:
        B.bigcn_sage_forward(model.plan, drp, dci, model.inv_deg, dx, model.layers[::-1])
    assert err.value.status == B.BIGCN_EINVAL
    need = B.bigcn_sage_forward_workspace_bytes(work.n, model.layers)
    gcn_like = B.bigcn_forward_workspace_bytes(
        work.n, [B.Layer(l.w_nbr_bits, l.alpha_nbr, l.d_in, l.d_out) for l in model.layers])
    assert need > gcn_like        # second product array
