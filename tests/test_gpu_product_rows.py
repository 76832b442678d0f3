"""The integers of the fused path, bit for bit: after a one-layer bigcn_forward the test reads the
workspace back, decodes the compact product rows from their documented format
(helpers.decode_product_rows: byte manipulation only) and compares every c'_ij = sum_{k < K'} F_ik B_kj
with the oracle's literal +-1 dot product.  One case per row format and per kernel that writes
product rows: the vector-ALU kernel with the binarisation folded in (fp32 input, at most 32768
nodes), the one-row-per-wavefront kernel (packed input, at most 32768 nodes), and beyond 32768
nodes the matrix-core row kernel or the vector-ALU row kernels, whichever the layer's shape
selects.  Inputs equal to a weight column (and its opposite) give products of +-K, so the escape
rows of the 7-bit formats are among the rows compared."""
import numpy as np
import pytest

import oracle
from helpers import decode_product_rows, to_device
from workloads import chung_lu_csr

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import torch
    from paper_2210_13149_amd import binding
    assert torch.cuda.is_available()
    binding.lib()
    return binding


# (d_in, d_out): fp16 rows; fp32 rows; one byte with the scale in the tail; in the last bytes of an
# 8-lane row; in the top bits of 32 / 64 / 16 lanes; K = 128 and K = 256 with the last bit folded
# out; 7-bit rows with one-byte escape; with fp16 escape (16 lanes and wider); separate scale; 8-bit
# 64-byte rows of more than 256 input bits with fp16 escape (up to 60 columns)
FORMATS = [(1433, 64), (3703, 64), (64, 7), (2, 5), (128, 41), (256, 47), (100, 256), (100, 512), (100, 100),
           (128, 128), (256, 256), (200, 256), (602, 128), (500, 64), (1024, 300), (300, 40), (1100, 300),
           (255, 61), (64, 75), (31, 33), (512, 47), (1024, 60), (257, 3)]


def _one_layer(B, n, d_in, d_out, seed, packed_input):
    """Run one layer on the GPU; returns (decoded c', K', escaped rows, oracle signs F, B^T)."""
    import torch
    rng = np.random.default_rng(seed)
    rp, ci = chung_lu_csr(n, 3 * n, 2.5, 2.0, seed=seed)
    w = rng.uniform(-1, 1, size=(d_in, d_out)).astype(np.float32)
    x = rng.standard_normal((n, d_in)).astype(np.float32)
    for k in range(min(24, n)):                      # products of +K and -K: rows that leave the 7-bit form
        x[k] = w[:, k % d_out] * (1 if k % 2 == 0 else -1)
    drp, dci, dx, dw = to_device(rp, ci, x, w)
    plan = B.Plan(drp, dci)
    dinv, _ = B.bigcn_gcn_norm(drp, dci)
    layers = [B.Layer.from_weight(dw)]
    need = B.bigcn_forward_workspace_bytes(n, layers)
    ws = torch.zeros((need,), dtype=torch.uint8, device="cuda")
    if packed_input:
        bits, beta = B.bigcn_pack(dx)
        B.bigcn_forward_packed(plan, drp, dci, dinv, bits, beta, layers, workspace=ws)
    else:
        B.bigcn_forward(plan, drp, dci, dinv, dx, layers, workspace=ws)
    torch.cuda.synchronize()
    layout = B.bigcn_forward_row_layout(d_in, d_out)
    offsets = B.bigcn_forward_workspace_map(n, layers)
    assert offsets["total"] == need
    values, k_eff, escaped = decode_product_rows(ws.cpu().numpy(), offsets, layout, n, d_out)
    f, _ = oracle.binarize_rows(x)
    bt, _ = oracle.binarize_weight(w)
    return values, k_eff, escaped, f, bt, layout


def _check(values, k_eff, f, bt, label):
    want = oracle.sign_matmul(np.ascontiguousarray(f[:, :k_eff]), np.ascontiguousarray(bt[:, :k_eff])).astype(np.int64)
    assert values.shape == want.shape
    if not np.array_equal(values, want):
        bad = np.argwhere(values != want)
        i = tuple(bad[0])
        raise AssertionError(f"{label}: {bad.shape[0]} of {want.size} integer products differ from the oracle; "
                             f"first at {i}: decoded {values[i]} oracle {want[i]}")


@pytest.mark.parametrize("d_in,d_out", FORMATS)
@pytest.mark.parametrize("producer", ["folded_pack_small", "packed_small", "large"])
def test_fused_path_integers_match_the_oracle_bit_for_bit(B, d_in, d_out, producer):
    n = {"folded_pack_small": 1500, "packed_small": 1500, "large": 33100}[producer]
    values, k_eff, escaped, f, bt, layout = _one_layer(B, n, d_in, d_out, seed=d_in * 1000 + d_out,
                                                        packed_input=producer == "packed_small")
    _check(values, k_eff, f, bt, f"{producer} {d_in}->{d_out} {layout}")
    if layout["escape"]:
        # the planted rows hold a product of +-d_in: beyond 7 bits whenever d_in / 2 > 63
        assert escaped[:24].all() == (d_in // 2 > 63), "planted rows and the alternate array disagree"
    else:
        assert not escaped.any()


def test_every_row_in_the_alternate_array(B):
    """All rows planted: every product row of a 200 -> 256 layer leaves the 7-bit form."""
    import torch
    n, d_in, d_out = 33000, 200, 256
    rng = np.random.default_rng(5)
    rp, ci = chung_lu_csr(n, 2 * n, 2.5, 2.0, seed=5)
    w = rng.uniform(-1, 1, size=(d_in, d_out)).astype(np.float32)
    x = np.stack([w[:, k % d_out] * (1 if k % 2 == 0 else -1) for k in range(n)]).astype(np.float32)
    drp, dci, dx, dw = to_device(rp, ci, x, w)
    plan = B.Plan(drp, dci)
    dinv, _ = B.bigcn_gcn_norm(drp, dci)
    layers = [B.Layer.from_weight(dw)]
    ws = torch.zeros((B.bigcn_forward_workspace_bytes(n, layers),), dtype=torch.uint8, device="cuda")
    B.bigcn_forward(plan, drp, dci, dinv, dx, layers, workspace=ws)
    torch.cuda.synchronize()
    layout = B.bigcn_forward_row_layout(d_in, d_out)
    values, k_eff, escaped = decode_product_rows(ws.cpu().numpy(), B.bigcn_forward_workspace_map(n, layers), layout, n, d_out)
    assert escaped.all()
    f, _ = oracle.binarize_rows(x)
    bt, _ = oracle.binarize_weight(w)
    _check(values, k_eff, f, bt, "all rows escaped")

