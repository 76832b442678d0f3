"""The closed forms of Sec. 5 against every storage / work figure the paper prints."""
import os

import pytest

from paper_2210_13149_amd import cost_model as cm

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rows():
    rows = []
    with open(os.path.join(GOLDEN, "paper_cost_figures.txt")) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            name, n, e, dims, *vals = line.split()
            rows.append((name, int(n), int(e), tuple(int(d) for d in dims.split("-")),
                         [float(v) for v in vals]))
    return rows


def _table1():
    out = {}
    with open(os.path.join(GOLDEN, "paper_table1_cora.txt")) as fh:
        for line in fh:
            if line.strip() and not line.startswith("#"):
                k, v = line.split()
                out[k] = float(v)
    return out


def _printed(value, text_digits):
    """Round `value` the way a figure with `text_digits` decimals was printed."""
    return round(value, text_digits)


@pytest.mark.parametrize("row", _rows(), ids=lambda r: r[0])
def test_printed_sizes_and_cycle_ops(row):
    name, n, e, dims, (ms, msb, ds, dsb, co, cob) = row
    s = cm.summary(n, e, dims)
    assert abs(s["model_size_bytes"] / 1024 - ms) <= 0.005 + 1e-9
    assert abs(s["model_size_bytes_binary"] / 1024 - msb) <= 0.0051
    # data sizes are printed with 1 or 2 decimals
    tol_ds = 0.051 if ds == round(ds, 1) else 0.0051
    assert abs(s["data_size_bytes"] / 2**20 - ds) <= tol_ds
    assert abs(s["data_size_bytes_binary"] / 2**20 - dsb) <= 0.0051
    # cycle operations are printed with three significant digits
    assert abs(s["cycle_ops"] / co - 1) < 5.1e-3
    assert abs(s["cycle_ops_binary"] / cob - 1) < 5.1e-3


def _sage_rows():
    rows = []
    with open(os.path.join(GOLDEN, "paper_cost_figures_sage.txt")) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            name, n, e, dims, *vals = line.split()
            rows.append((name, int(n), int(e), tuple(int(d) for d in dims.split("-")),
                         [float(v) for v in vals]))
    return rows


@pytest.mark.parametrize("row", _sage_rows(), ids=lambda r: r[0])
def test_printed_sage_sizes_and_cycle_ops(row):
    name, n, e, dims, (ms, msb, co, cob) = row
    s = cm.sage_summary(n, e, dims)
    assert abs(s["model_size_bytes"] / 1024 - ms) <= 0.005 + 1e-9
    assert abs(s["model_size_bytes_binary"] / 1024 - msb) <= 0.0051
    assert abs(s["cycle_ops"] / co - 1) < 5.1e-3
    assert abs(s["cycle_ops_binary"] / cob - 1) < 5.1e-3


def test_table1_exact_counts():
    t = _table1()
    dims = (1433, 64, 7)
    assert cm.cycle_ops(2708, 5429, dims) == t["calculations_gcn"]
    assert round(cm.cycle_ops_binary(2708, 5429, dims)) == t["calculations_bigcn"]
    s = cm.summary(2708, 5429, dims)
    assert round(s["model_size_ratio"], 1) == t["ratio_model_size"]
    assert round(s["cycle_ops_ratio"], 1) == t["ratio_calculations"]
    # the printed data-size ratio is the quotient of the rounded sizes 14.8 / 0.47
    assert round(14.8 / 0.47, 1) == t["ratio_data_size"]
    assert abs(s["data_size_ratio"] - t["ratio_data_size"]) < 0.3


def test_per_layer_speedups():
    t = _table1()
    assert round(cm.speedup_feature_extraction(1433)) == t["speedup_layer1"]
    assert round(cm.speedup_feature_extraction(64)) == t["speedup_layer2"]
    s = cm.summary(2708, 5429, (1433, 64, 7))
    assert int(s["cycle_ops_ratio"]) == t["speedup_total"]


def test_closed_form_ratios_agree_with_counts():
    # PC and DC are the per-layer / per-matrix ratios of the byte counts
    for d_in, d_out in [(1433, 64), (64, 7), (100, 256)]:
        dims = (d_in, d_out)
        assert cm.model_size_bytes(dims) / cm.model_size_bytes_binary(dims) == pytest.approx(
            cm.parameter_compression(d_in))
    assert cm.data_size_bytes(1000, 602) / cm.data_size_bytes_binary(1000, 602) == pytest.approx(
        cm.data_compression(602))
    # S_full with |E| = N*deg/2 reproduces the ratio of the operation counts of one layer
    n, deg, d_in, d_out = 5000, 6.0, 300, 32
    e = int(n * deg / 2)
    ratio = cm.cycle_ops(n, e, (d_in, d_out)) / cm.cycle_ops_binary(n, e, (d_in, d_out))
    assert ratio == pytest.approx(cm.speedup_layer(d_in, deg))
    assert cm.speedup_layer(d_in, 0.0) == pytest.approx(cm.speedup_feature_extraction(d_in))
