"""Parity of the steps on either side of the layer path, through the C ABI: column statistics
(the standardisation parameters), the forward from a pre-binarised input, and the prediction
(softmax / largest class)."""
import numpy as np
import pytest

import oracle
from helpers import assert_close, to_device
from workloads import make_workload, scaled_config

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import torch
    from paper_2210_13149_amd import binding
    assert torch.cuda.is_available()
    binding.lib()
    return binding


# ---- column statistics ---------------------------------------------------------------------
@pytest.mark.parametrize("rows,cols", [(1, 5), (7, 1), (31, 64), (33, 65), (1000, 100), (4097, 47),
                                       (20000, 602), (300, 3703), (123457, 256)])
def test_column_stats_match_oracle(B, rows, cols):
    rng = np.random.default_rng(rows * 131 + cols)
    x = (rng.standard_normal((rows, cols)) * rng.uniform(0.01, 30.0, size=(1, cols))
         + rng.uniform(-50.0, 50.0, size=(1, cols))).astype(np.float32)
    if cols > 3:
        x[:, 3] = 7.25                      # constant column: variance exactly zero
    shift, mul = B.bigcn_column_stats(to_device(x))
    want_shift, want_mul = oracle.column_standardisation(x)
    # fp64 accumulation, one rounding to fp32 (the oracle rounds its fp64 result the same way)
    assert np.allclose(shift.cpu().numpy(), want_shift, rtol=2e-7, atol=1e-30)
    assert np.allclose(mul.cpu().numpy(), want_mul, rtol=2e-7, atol=0)
    if cols > 3:
        assert shift.cpu().numpy()[3] == np.float32(7.25)
        assert mul.cpu().numpy()[3] == np.float32(1.0 / np.sqrt(1e-5))


def test_column_stats_large_mean_small_spread_and_strided_input(B):
    """Mean 1e4 against a spread of 1e-2: sums of raw squares would lose the variance; the pivoted
    sums keep it.  Input is a column slice of a wider matrix (row stride > cols)."""
    import torch
    rng = np.random.default_rng(5)
    wide = (1e4 + 1e-2 * rng.standard_normal((50000, 80))).astype(np.float32)
    view = to_device(wide)[:, 8:72]
    shift, mul = B.bigcn_column_stats(view)
    want_shift, want_mul = oracle.column_standardisation(wide[:, 8:72])
    assert np.allclose(shift.cpu().numpy(), want_shift, rtol=2e-7, atol=0)
    assert np.allclose(mul.cpu().numpy(), want_mul, rtol=1e-6, atol=0)
    again = B.bigcn_column_stats(view)
    assert torch.equal(again[0], shift) and torch.equal(again[1], mul)


def test_column_stats_full_size_input_features(B):
    """The statistics of the largest workload's feature matrix (2 449 029 x 100)."""
    work = make_workload("c5").x
    shift, mul = B.bigcn_column_stats(to_device(work))
    want_shift, want_mul = oracle.column_standardisation(work)
    assert np.allclose(shift.cpu().numpy(), want_shift, rtol=2e-7, atol=1e-9)
    assert np.allclose(mul.cpu().numpy(), want_mul, rtol=2e-7, atol=0)


def test_column_stats_errors(B):
    import torch
    x = torch.zeros((4, 4), dtype=torch.float32, device="cuda")
    out = torch.zeros((4,), dtype=torch.float32, device="cuda")
    ws = torch.zeros((64,), dtype=torch.float64, device="cuda")
    L, p = B.lib(), lambda t: t.data_ptr()
    assert L.bigcn_column_stats(p(x), 0, 4, 4, 1e-5, p(out), p(out), p(ws), 512, None) == B.BIGCN_EINVAL
    assert L.bigcn_column_stats(p(x), 4, 4, 3, 1e-5, p(out), p(out), p(ws), 512, None) == B.BIGCN_EINVAL
    assert L.bigcn_column_stats(p(x), 4, 4, 4, -1.0, p(out), p(out), p(ws), 512, None) == B.BIGCN_EINVAL
    assert L.bigcn_column_stats(p(x), 4, 4, 4, 1e-5, p(out), p(out), p(ws), 8, None) == B.BIGCN_EWORKSPACE
    assert L.bigcn_column_stats(None, 4, 4, 4, 1e-5, p(out), p(out), p(ws), 512, None) == B.BIGCN_ENULL
    assert L.bigcn_column_stats_workspace_bytes(0, 4) == 0
    assert L.bigcn_column_stats_workspace_bytes(4, 4) == 1 * 2 * 4 * 8


# ---- forward from a pre-binarised input ---------------------------------------------------------
@pytest.mark.parametrize("name,n_scaled", [("c1", None), ("c3", None), ("c5", 30000)])
def test_forward_packed_is_bit_identical_to_forward(B, name, n_scaled):
    import torch
    work = make_workload(name if n_scaled is None else scaled_config(name, n_scaled))
    drp, dci, dx = to_device(work.row_ptr, work.col_idx, work.x)
    plan = B.Plan(drp, dci)
    dinv, _ = B.bigcn_gcn_norm(drp, dci)
    shift, mul = B.bigcn_column_stats(dx)
    weights = [to_device(w) for w in work.weights]
    fused = [B.Layer.from_weight(weights[0], shift, mul)] + [B.Layer.from_weight(w) for w in weights[1:]]
    want = B.bigcn_forward(plan, drp, dci, dinv, dx, fused).clone()
    x_bits, x_beta = B.bigcn_pack(dx, shift, mul)
    packed_layers = [B.Layer.from_weight(w) for w in weights]
    got = B.bigcn_forward_packed(plan, drp, dci, dinv, x_bits, x_beta, packed_layers)
    torch.cuda.synchronize()
    assert torch.equal(got, want)
    # and against the oracle, with the same fp32 parameters
    ref, _ = oracle.forward(work.row_ptr, work.col_idx, work.x, work.weights,
                            bn=[(shift.cpu().numpy(), mul.cpu().numpy())] + [None] * (len(weights) - 1))
    ok = np.abs(got.cpu().numpy() - ref) <= 1e-5 * np.abs(ref) + 1e-6
    assert ok.mean() > 0.99


def test_forward_packed_with_folded_last_bit_and_padded_rows(B):
    """d_in = 256 (the last input bit rides on the stored scale's sign) and an input whose packed
    rows are wider than needed."""
    import torch
    from workloads import chung_lu_csr
    rng = np.random.default_rng(256)
    n = 700
    rp, ci = chung_lu_csr(n, 4000, 2.5, 2.0, seed=256)
    x = rng.standard_normal((n, 256)).astype(np.float32)
    ws = [rng.uniform(-1, 1, size=(256, 256)).astype(np.float32),
          rng.uniform(-1, 1, size=(256, 9)).astype(np.float32)]
    drp, dci, dx = to_device(rp, ci, x)
    plan = B.Plan(drp, dci)
    dinv, _ = B.bigcn_gcn_norm(drp, dci)
    layers = [B.Layer.from_weight(to_device(w)) for w in ws]
    want = B.bigcn_forward(plan, drp, dci, dinv, dx, layers).clone()
    bits, beta = B.bigcn_pack(dx)
    padded = torch.full((n, 7), -1, dtype=torch.int64, device="cuda")
    padded[:, :4] = bits
    got = B.bigcn_forward_packed(plan, drp, dci, dinv, padded[:, :4], beta, layers)
    assert got.data_ptr() != want.data_ptr() and torch.equal(got, want)
    ref, _ = oracle.forward(rp, ci, x, ws)
    ok = np.abs(got.cpu().numpy() - ref) <= 1e-5 * np.abs(ref) + 1e-6
    assert ok.mean() > 0.99
    with pytest.raises(B.BigcnError) as err:
        B.bigcn_forward_packed(plan, drp, dci, dinv, bits, beta,
                               [B.Layer.from_weight(to_device(ws[0]), dinv[:256].contiguous(), None), layers[1]])
    assert err.value.status == B.BIGCN_EINVAL


# ---- prediction ---------------------------------------------------------------------------------
@pytest.mark.parametrize("n,d", [(1, 1), (5, 2), (1000, 3), (777, 7), (4096, 41), (30000, 47), (500, 64),
                                 (300, 65), (200, 300), (64, 512)])
def test_predict_matches_oracle(B, n, d):
    rng = np.random.default_rng(n * 7 + d)
    h = (rng.standard_normal((n, d)) * 6).astype(np.float32)
    if d >= 3 and n >= 4:
        h[0, :] = 1.5                                   # all equal -> class 0
        h[1, d - 1] = h[1].max() + 1
        h[1, d // 2] = h[1, d - 1]                      # tie: the lower index wins
        h[2] = 80.0 * np.sign(h[2])                     # saturating softmax
        h[3] = -1e4
        h[3, d - 1] = 1e4                               # huge range, no overflow
    labels, probs = B.bigcn_predict(to_device(h), want_probs=True)
    want_labels, want_probs = oracle.predict(h)
    assert np.array_equal(labels.cpu().numpy(), want_labels)
    assert_close(probs.cpu().numpy(), want_probs, "softmax")
    only_labels, none = B.bigcn_predict(to_device(h))
    assert none is None and np.array_equal(only_labels.cpu().numpy(), want_labels)


def test_predict_on_forward_output_with_padded_rows(B):
    import torch
    work = make_workload("c3")
    drp, dci, dx = to_device(work.row_ptr, work.col_idx, work.x)
    model = B.BiGCN(drp, dci, [to_device(w) for w in work.weights],
                    [B.bigcn_column_stats(dx), None])
    logits = model.forward(dx)
    wide = torch.full((work.n, 8), 1e30, dtype=torch.float32, device="cuda")
    wide[:, :3] = logits
    labels, probs = B.bigcn_predict(wide[:, :3], want_probs=True)
    want_labels, want_probs = oracle.predict(logits.cpu().numpy())
    assert np.array_equal(labels.cpu().numpy(), want_labels)
    assert_close(probs.cpu().numpy(), want_probs, "softmax of logits")
    assert B.lib().bigcn_predict(wide.data_ptr(), 4, 3, 2, labels.data_ptr(), None, 0, None) == B.BIGCN_EINVAL
    assert B.lib().bigcn_predict(wide.data_ptr(), 4, 3, 8, None, None, 0, None) == B.BIGCN_ENULL


# ---- entropy of a hidden layer by binning -------------------------------------------------------
@pytest.mark.parametrize("rows,cols,bins", [(1, 3, 4), (100, 1, 1), (5000, 9, 200), (40000, 64, 1000),
                                            (12345, 130, 37), (3000, 512, 1024)])
def test_entropy_matches_oracle(B, rows, cols, bins):
    rng = np.random.default_rng(rows + 3 * cols + bins)
    h = (rng.standard_normal((rows, cols)) * rng.uniform(0.1, 5.0, size=(1, cols))
         + rng.uniform(-3, 3, size=(1, cols))).astype(np.float32)
    if cols > 2:
        h[:, 1] = -0.75                                           # constant neuron: one bin, entropy 0
        h[:, 2] = np.where(np.arange(rows) % 2 == 0, 1.0, 2.0)    # two values: one bit (even rows)
    per, total, counts = B.bigcn_entropy(to_device(h), bins, want_counts=True)
    want_per, want_total, want_counts = oracle.binned_entropy(h, bins)
    assert np.array_equal(counts.cpu().numpy().astype(np.int64), want_counts)      # integer work: exact
    assert np.allclose(per.cpu().numpy(), want_per, rtol=1e-12, atol=1e-14)
    assert float(total) == pytest.approx(want_total, rel=1e-12, abs=1e-14)
    per2, total2, none = B.bigcn_entropy(to_device(h), bins)
    assert none is None and float(total2) == float(total)


def test_entropy_of_a_hidden_layer_at_full_width(B):
    """The estimate on a hidden activation of the largest workload's shape (one million rows of
    256 neurons, M = 1000 as in the paper's table), on a strided view."""
    import torch
    gen = torch.Generator(device="cuda").manual_seed(9)
    wide = torch.randn((1_000_000, 260), dtype=torch.float32, device="cuda", generator=gen)
    view = wide[:, 2:258]
    per, total, counts = B.bigcn_entropy(view, 1000, want_counts=True)
    want_per, want_total, want_counts = oracle.binned_entropy(view.cpu().numpy(), 1000)
    assert np.array_equal(counts.cpu().numpy().astype(np.int64), want_counts)
    assert float(total) == pytest.approx(want_total, rel=1e-12)
    assert 256 * 7.0 < float(total) < 256 * np.log2(1000)


def test_entropy_errors(B):
    import torch
    h = torch.zeros((8, 4), dtype=torch.float32, device="cuda")
    out = torch.zeros((4,), dtype=torch.float64, device="cuda")
    ws = torch.zeros((1 << 16,), dtype=torch.uint8, device="cuda")
    L, p = B.lib(), lambda t: t.data_ptr()
    assert L.bigcn_entropy(p(h), 8, 4, 4, 0, p(out), p(out), None, p(ws), ws.numel(), None) == B.BIGCN_EINVAL
    assert L.bigcn_entropy(p(h), 8, 4, 4, 2000, p(out), p(out), None, p(ws), ws.numel(), None) == B.BIGCN_ESHAPE
    assert L.bigcn_entropy(p(h), 8, 4, 4, 16, p(out), None, None, p(ws), ws.numel(), None) == B.BIGCN_ENULL
    assert L.bigcn_entropy(p(h), 8, 4, 4, 16, p(out), p(out), None, p(ws), 16, None) == B.BIGCN_EWORKSPACE
    assert L.bigcn_entropy_workspace_bytes(4, 0) == 0 and L.bigcn_entropy_workspace_bytes(4, 16) > 0
