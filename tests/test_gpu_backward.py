"""Parity of the back propagation through one binarised layer (Sec. 4.3, Algorithm 1) against the
CPU oracle, through the C ABI.

Both sides start from the same fp32 inputs (features, weights, upstream gradient); nothing flows
from the GPU into the oracle.  Tolerances, per output element, with u = 2^-24:
  * the standard bar |gpu - ref| <= 1e-5 |ref| + 1e-6, or
  * the worst-case rounding bound of the fp32 evaluation, (m + 64) u * sum |terms|, where m is the
    length of the longest fp32 accumulation chain of that output (an element whose terms cancel
    cannot be resolved to 1e-5 of itself by any fp32 evaluation order).
The clipped straight-through rule decides on |g| < 1 in fp32 on the GPU and in fp64 in the oracle:
elements whose |g| lies within the rounding bound of 1 may come out either way and are checked to
be one of the two valid values.
"""
import numpy as np
import pytest

import oracle
from helpers import close, to_device
from workloads import chung_lu_csr, make_workload, scaled_config

pytestmark = pytest.mark.gpu
U = 2.0 ** -24


@pytest.fixture(scope="module")
def B():
    import torch
    from paper_2210_13149_amd import binding
    assert torch.cuda.is_available()
    binding.lib()
    return binding


def chain_length_weight(B, n, d_in, d_out):
    """Nodes per fp32 accumulation chain of g_wt (one chunk of the split over the nodes)."""
    blocks = ((d_out + 63) // 64) * ((d_in + 255) // 256)
    chunks = max(1, min((1024 + blocks - 1) // blocks, (n + 63) // 64))
    rpc = ((n + chunks - 1) // chunks + 63) // 64 * 64
    return rpc


def run_both(B, rp, ci, x, w, g_out, bn=None, want_input_grad=True):
    """One layer backward on both sides; returns (gpu dict, oracle dict, bounds dict)."""
    import torch
    n, d_in = x.shape
    d_out = w.shape[1]
    shift, mul = bn if bn is not None else (None, None)
    # oracle side
    a = oracle.gcn_norm(rp, ci)
    sign, beta = oracle.binarize_rows(x, shift, mul)
    ref = oracle.layer_backward(rp, ci, a, g_out, sign, beta, w, mul=mul)
    # GPU side, from the same fp32 inputs
    drp, dci, dx, dw, dg = to_device(rp, ci, x, w, g_out.astype(np.float32))
    dshift, dmul = (None, None) if bn is None else to_device(shift, mul)
    plan = B.Plan(drp, dci)
    _, vals = B.bigcn_gcn_norm(drp, dci, want_vals=True)
    f_bits, dbeta = B.bigcn_pack(dx, dshift, dmul)
    g_w, g_in = B.bigcn_layer_backward(plan, drp, dci, vals, dg, f_bits, dbeta, dw, bn_mul=dmul,
                                       want_input_grad=want_input_grad)
    torch.cuda.synchronize()
    gpu = {"g_w": g_w.cpu().numpy(), "g_in": None if g_in is None else g_in.cpu().numpy()}
    # rounding bounds from the oracle's own intermediates
    gz_abs = np.abs(ref["g_zeta"])
    deg = np.diff(rp).astype(np.float64)[:, None]
    gz_err = (deg + 4.0) * U * oracle.aggregate(rp, ci, a, np.abs(g_out))         # error of g_zeta itself
    abs_wt = np.abs(ref["h_tilde"]).T @ gz_abs
    abs_ht = gz_abs @ np.abs(ref["w_tilde"]).T
    m_wt = chain_length_weight(B, n, d_in, d_out)
    bound_wt = (m_wt + 64) * U * abs_wt + np.abs(ref["h_tilde"]).T @ gz_err
    bound_ht = (d_out + 64) * U * abs_ht + gz_err @ np.abs(ref["w_tilde"]).T
    if not want_input_grad and d_in <= d_out:
        # first-layer evaluation order g_wt = (A~ H~)^T g_out: every entry of U = A~ H~ is a sum of
        # deg_i terms of magnitude a_ik beta_k, then a chain of m_wt products over the nodes
        u_mag = oracle.aggregate(rp, ci, a, np.abs(beta)[:, None])[:, 0]
        per_node = (deg[:, 0] + 4.0 + m_wt + 64) * U * u_mag
        bound_wt = np.broadcast_to((per_node[None, :] @ np.abs(g_out))[0][None, :], bound_wt.shape).copy()
    return gpu, ref, {"g_wt": bound_wt, "g_ht": bound_ht}


def check_weight_gradient(gpu_gw, ref, bound_wt, w):
    """g_w = B (colsum / d_in) + alpha g_wt ste: propagate the bound of g_wt through both terms."""
    d_in = w.shape[0]
    alpha = np.abs(w.astype(np.float64)).mean(axis=0)
    ste = np.abs(w.astype(np.float64)) < 1.0
    bound = bound_wt.sum(axis=0)[None, :] / d_in + alpha[None, :] * bound_wt * ste
    diff = np.abs(gpu_gw - ref["g_w"])
    ok = close(gpu_gw, ref["g_w"]) | (diff <= bound + 1e-30)
    assert ok.all(), f"g_w: {int((~ok).sum())} of {ok.size} out of tolerance, worst {diff[~ok].max():.3e}"
    # the worst-case bound is loose; typical errors must be far inside it
    scale = np.abs(ref["g_w"]).mean() + 1e-30
    assert np.median(diff) <= 1e-5 * scale + 1e-7


def check_input_gradient(gpu_gin, ref, bound_ht, mul):
    g_ht = ref["g_ht"]
    m = np.ones(g_ht.shape[1]) if mul is None else mul.astype(np.float64)
    kept = g_ht * m[None, :]
    near_one = np.abs(np.abs(g_ht) - 1.0) <= bound_ht + 1e-7
    diff_kept = np.abs(gpu_gin - kept)
    ok_kept = (diff_kept <= 1e-5 * np.abs(kept) + 1e-6) | (diff_kept <= bound_ht * np.abs(m)[None, :] + 1e-30)
    is_zero = gpu_gin == 0.0
    expect_zero = np.abs(g_ht) >= 1.0
    ok = np.where(near_one, ok_kept | is_zero, np.where(expect_zero, is_zero, ok_kept))
    assert ok.all(), f"g_in: {int((~ok).sum())} of {ok.size} out of tolerance"
    return int(near_one.sum()), int(expect_zero.sum())


@pytest.mark.parametrize("n,n_edges,d_in,d_out,g_scale,with_bn", [
    (500, 2000, 70, 9, 0.5, False),
    (3000, 30000, 256, 47, 1.0, True),
    (2000, 9000, 100, 256, 0.05, True),
    (1500, 8000, 300, 130, 0.1, False),
    (4000, 20000, 64, 64, 0.3, True),
    (130, 400, 513, 257, 0.05, False),
    (1, 0, 5, 3, 1.0, False),
    (60000, 400000, 100, 256, 0.1, True),      # many node chunks; first-layer order without g_in
    (3000, 40000, 300, 300, 0.05, False),      # five packed words: two passes of the sign aggregation
])
def test_layer_backward_matches_oracle(B, n, n_edges, d_in, d_out, g_scale, with_bn):
    rng = np.random.default_rng(n + 7 * d_in + 13 * d_out)
    rp, ci = chung_lu_csr(n, n_edges, 2.5, 1.5, seed=n + d_in) if n > 1 else (
        np.array([0, 1], dtype=np.int64), np.array([0], dtype=np.int32))
    x = (rng.standard_normal((n, d_in)) * 1.5 + 0.3).astype(np.float32)
    w = rng.uniform(-1.6, 1.6, size=(d_in, d_out)).astype(np.float32)        # both sides of |w| = 1
    g_out = (rng.standard_normal((n, d_out)) * g_scale).astype(np.float32).astype(np.float64)
    bn = oracle.column_standardisation(x) if with_bn else None
    gpu, ref, bounds = run_both(B, rp, ci, x, w, g_out, bn)
    check_weight_gradient(gpu["g_w"], ref, bounds["g_wt"], w)
    near, clipped = check_input_gradient(gpu["g_in"], ref, bounds["g_ht"], None if bn is None else bn[1])
    if n >= 500 and g_scale >= 0.3:
        assert clipped > 0 and clipped < ref["g_ht"].size      # both branches of the indicator taken
    # without the input gradient: the same weight gradient, bit for bit when d_in > d_out; for
    # d_in <= d_out it is evaluated as (A~ H~)^T g_out (the first-layer order) and checked against
    # the oracle with that order's rounding bound
    gpu2, ref2, bounds2 = run_both(B, rp, ci, x, w, g_out, bn, want_input_grad=False)
    assert gpu2["g_in"] is None
    if d_in > d_out:
        assert np.array_equal(gpu2["g_w"], gpu["g_w"])
    else:
        check_weight_gradient(gpu2["g_w"], ref2, bounds2["g_wt"], w)


def test_two_layer_chain_from_a_cross_entropy_gradient(B):
    """Back propagation through both layers of the PubMed-shaped model.  The upstream gradient of
    each layer is the oracle's (cross-entropy of its own logits against seeded random labels, then
    its own g_in), rounded to fp32 and handed to both sides."""
    work = make_workload("c3")
    rng = np.random.default_rng(3)
    n = work.n
    logits, recs = oracle.forward(work.row_ptr, work.col_idx, work.x, work.weights,
                                  calibrate=[True, False], keep_trace=True)
    labels = rng.integers(0, logits.shape[1], size=n)
    labeled = rng.random(n) < 0.3
    _, probs = oracle.predict(logits)
    g = probs.copy()
    g[np.arange(n), labels] -= 1.0
    g[~labeled] = 0.0
    g /= labeled.sum()
    # layer 2 (64 -> 3): input is the oracle's hidden activation, no standardisation
    h1 = recs[1]["input"].astype(np.float32)
    g2 = g.astype(np.float32).astype(np.float64)
    gpu, ref, bounds = run_both(B, work.row_ptr, work.col_idx, h1, work.weights[1], g2)
    check_weight_gradient(gpu["g_w"], ref, bounds["g_wt"], work.weights[1])
    check_input_gradient(gpu["g_in"], ref, bounds["g_ht"], None)
    # layer 1 (500 -> 64): standardised input features; no input gradient needed
    g1 = ref["g_in"].astype(np.float32).astype(np.float64)
    bn = (recs[0]["shift"], recs[0]["mul"])
    gpu, ref, bounds = run_both(B, work.row_ptr, work.col_idx, work.x, work.weights[0], g1, bn,
                                want_input_grad=False)
    check_weight_gradient(gpu["g_w"], ref, bounds["g_wt"], work.weights[0])
    assert np.abs(ref["g_w"]).max() > 0


def test_backward_is_repeatable_and_rejects_bad_arguments(B):
    import torch
    rng = np.random.default_rng(11)
    n, d_in, d_out = 900, 96, 40
    rp, ci = chung_lu_csr(n, 5000, 2.5, 2.0, seed=4)
    x = rng.standard_normal((n, d_in)).astype(np.float32)
    w = rng.uniform(-1.5, 1.5, size=(d_in, d_out)).astype(np.float32)
    g = rng.standard_normal((n, d_out)).astype(np.float32)
    drp, dci, dx, dw, dg = to_device(rp, ci, x, w, g)
    plan = B.Plan(drp, dci)
    _, vals = B.bigcn_gcn_norm(drp, dci, want_vals=True)
    bits, beta = B.bigcn_pack(dx)
    a = B.bigcn_layer_backward(plan, drp, dci, vals, dg, bits, beta, dw)
    b = B.bigcn_layer_backward(plan, drp, dci, vals, dg, bits, beta, dw)
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])
    with pytest.raises(B.BigcnError) as err:
        B.bigcn_layer_backward(plan, drp, dci, vals, dg, bits, beta, dw,
                               workspace=torch.empty(256, dtype=torch.uint8, device="cuda"))
    assert err.value.status == B.BIGCN_EWORKSPACE
    assert B.lib().bigcn_layer_backward_workspace_bytes(0, 4, 4) == 0
    with pytest.raises(ValueError):
        B.bigcn_layer_backward(plan, drp, dci, vals, dg[:, :8], bits, beta, dw)


@pytest.mark.timeout(600)
def test_backward_of_the_last_layer_at_full_size(B):
    """Layer 2 of the largest workload (256 -> 47) at its full size, from a seeded upstream
    gradient; the layer input is a seeded stand-in with the statistics of a hidden activation."""
    cfg = scaled_config("c5", 2449029)
    work = make_workload(cfg)
    rng = np.random.default_rng(55)
    n, d_in, d_out = work.n, 256, 47
    x = rng.standard_normal((n, d_in), dtype=np.float32)
    w = work.weights[2]
    g_out = (rng.standard_normal((n, d_out), dtype=np.float32) * 0.2).astype(np.float64)
    gpu, ref, bounds = run_both(B, work.row_ptr, work.col_idx, x, w, g_out)
    check_weight_gradient(gpu["g_w"], ref, bounds["g_wt"], w)
    check_input_gradient(gpu["g_in"], ref, bounds["g_ht"], None)
