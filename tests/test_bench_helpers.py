"""Host-side logic of bench.py that needs no GPU: the tracked traffic file, the cache model that
is printed beside the headline figure, and the per-launch bounds."""
import os

import numpy as np
import pytest

import bench

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_traffic_file_names_kernel_commit_and_bytes():
    t = bench.measured_traffic("c5")
    assert t is not None and t["bytes"] > 1e9
    assert "spmm_kernel" in t["kernel"] and len(t["measured_at_commit"]) >= 7
    assert bench.measured_traffic("no-such-workload") is None


def test_cache_model_limits():
    """Everything fits -> every request hits; a tiny cache -> (nearly) none; more cache never hurts;
    with equal degrees the hit rate is the resident share of the rows."""
    rng = np.random.default_rng(0)
    deg = rng.integers(1, 200, size=20000)
    row_ptr = np.concatenate([[0], np.cumsum(deg)])
    assert bench.infinity_cache_model(row_ptr, 256, cache_bytes=1 << 40)["hit_rate"] == 1.0
    tiny = bench.infinity_cache_model(row_ptr, 256, cache_bytes=256 * 4)["hit_rate"]
    half = bench.infinity_cache_model(row_ptr, 256, cache_bytes=256 * 10000)["hit_rate"]
    most = bench.infinity_cache_model(row_ptr, 256, cache_bytes=256 * 18000)["hit_rate"]
    assert 0.0 <= tiny < 0.01 and tiny < half < most < 1.0
    assert half > 0.5          # the cache keeps the rows that are asked for most: better than a random half
    flat = np.arange(0, 10001 * 7, 7)
    got = bench.infinity_cache_model(flat, 128, cache_bytes=128 * 2500)["hit_rate"]
    assert got == pytest.approx(0.25, abs=1e-6)
    # rows shorter than a cache line still cost a line each
    assert bench.infinity_cache_model(flat, 64, cache_bytes=128 * 2500)["hit_rate"] == pytest.approx(0.25, abs=1e-6)


class _FakeBinding:
    GEMM_FP4, GEMM_VALU = 3, 1

    @staticmethod
    def bigcn_forward_row_bytes(d_in, d_out):
        return 256 if d_out > 64 else 64, True

    @staticmethod
    def bigcn_forward_row_layout(d_in, d_out):
        return {"groups": 32 if d_out > 64 else 8, "vec": 8, "kind": 0, "k_eff": d_in, "fold_last": 0,
                "scale_place": 2 if d_out > 64 else 3, "escape": 0, "alt_kind": 0}

    @staticmethod
    def bigcn_forward_gemm_path(n, d_in, d_out):
        return 3 if n > 32768 else 1


def test_slot_bounds_and_cache_resident_rule():
    from workloads import get_config
    cfg = get_config("c5")
    nnz = cfg.nnz
    launch_ms = [0.25, 0.18, 4.6, 0.25, 4.7, 0.07, 2.5]
    slots = bench.slot_bounds(cfg, cfg.n_nodes, nnz, _FakeBinding, launch_ms)
    assert [s["slot"] for s in slots] == ["pack", "bit_gemm[0]", "aggregation[0]", "bit_gemm[1]", "aggregation[1]",
                                          "bit_gemm[2]", "aggregation[2]"]
    assert slots[5]["bound"] == "hbm" and slots[5]["algorithmic_bytes"] == cfg.n_nodes * (8 * 4 + 64)
    agg1 = slots[4]
    assert agg1["algorithmic_bytes"] == nnz * (4 + 256) + cfg.n_nodes * (8 + 4 + 4 + 8 * 4 + 4)
    assert agg1["frac"] == pytest.approx(agg1["algorithmic_bytes"] / 4.7e-3 / 8e12)
    assert not agg1["rows_fit_infinity_cache"] and slots[6]["rows_fit_infinity_cache"]
    # the cache-resident launch is compared with the plain gather, not with HBM
    bench.apply_cache_bound(slots, {"128": 2.3})
    assert slots[6]["frac"] == pytest.approx(2.3 / 2.5) and "cache-resident" in slots[6]["bound"]
    assert slots[4]["bound"] == "hbm"
    dom = bench.dominant_roofline(slots)
    assert dom["kernel"] == "aggregation[1]" and dom["bound"] == "hbm" and dom["peak"] == 8000.0


def test_more_than_one_gpu_is_refused_with_a_message():
    """`bench.py --gpus N` with N above 1 exits before touching a device and says why."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    run = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                         timeout=120)
    assert run.returncode != 0 and run.stdout.strip() == ""
    assert "ONE GPU" in run.stderr
