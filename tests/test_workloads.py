"""Structure and determinism of the seeded synthetic inputs."""
import numpy as np
import pytest

from workloads import (CONFIGS, chung_lu_csr, csr_from_undirected_edges, get_config,
                       make_features, make_workload, scaled_config)


def _check_pattern(rp, ci, n, n_edges):
    assert rp.dtype == np.int64 and ci.dtype == np.int32
    assert rp.shape == (n + 1,) and rp[0] == 0 and rp[-1] == ci.size == 2 * n_edges + n
    rows = np.repeat(np.arange(n), np.diff(rp))
    key = rows.astype(np.int64) * n + ci
    assert np.all(np.diff(key) > 0)                      # sorted columns, no duplicates
    assert np.count_nonzero(rows == ci) == n             # exactly one self-loop per node
    assert np.array_equal(np.sort(ci.astype(np.int64) * n + rows), key)   # symmetric


@pytest.mark.parametrize("name", ["c1", "c2", "c3"])
def test_small_configs_have_the_stated_shape(name):
    cfg = get_config(name)
    w = make_workload(name)
    _check_pattern(w.row_ptr, w.col_idx, cfg.n_nodes, cfg.n_edges)
    assert w.x.shape == (cfg.n_nodes, cfg.dims[0]) and w.x.dtype == np.float32
    assert [m.shape for m in w.weights] == list(zip(cfg.dims[:-1], cfg.dims[1:]))
    deg = np.diff(w.row_ptr)
    assert deg.min() >= 1 and deg.max() > 10 * np.median(deg)      # heavy tail
    if cfg.feature_kind == "bernoulli":
        assert set(np.unique(w.x)) <= {0.0, 1.0}
        assert abs(w.x.mean() - cfg.feature_density) < 0.1 * cfg.feature_density
    else:
        assert w.x.min() >= 0 and abs((w.x > 0).mean() - cfg.feature_density) < 0.01
        sums = w.x.sum(axis=1)
        assert np.allclose(sums[sums > 0], 1.0, atol=1e-5)
    for m, (a, b) in zip(w.weights, zip(cfg.dims[:-1], cfg.dims[1:])):
        assert np.abs(m).max() <= np.sqrt(6.0 / (a + b))


def test_generation_is_deterministic_and_seed_dependent():
    a = chung_lu_csr(500, 2000, 2.5, 3.0, seed=7)
    b = chung_lu_csr(500, 2000, 2.5, 3.0, seed=7)
    c = chung_lu_csr(500, 2000, 2.5, 3.0, seed=8)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    assert not np.array_equal(a[1], c[1])
    w1, w2 = make_workload("c1"), make_workload("c1")
    assert np.array_equal(w1.x, w2.x) and all(np.array_equal(p, q) for p, q in zip(w1.weights, w2.weights))


def test_dense_graph_reaches_its_edge_count():
    rp, ci = chung_lu_csr(300, 300 * 299 // 4, 2.5, 5.0, seed=3)
    _check_pattern(rp, ci, 300, 300 * 299 // 4)


def test_csr_builder_rejects_bad_edges():
    with pytest.raises(ValueError):
        csr_from_undirected_edges(3, np.array([0, 0]), np.array([1, 1]))
    with pytest.raises(ValueError):
        csr_from_undirected_edges(3, np.array([0]), np.array([0]))
    with pytest.raises(ValueError):
        csr_from_undirected_edges(3, np.array([0]), np.array([3]))


def test_scaled_config_keeps_the_recipe():
    cfg = scaled_config("c5", 20000)
    full = CONFIGS["c5"]
    assert cfg.dims == full.dims and cfg.feature_kind == full.feature_kind
    assert abs(cfg.n_edges / cfg.n_nodes - full.n_edges / full.n_nodes) < 0.01
    w = make_workload(cfg)
    _check_pattern(w.row_ptr, w.col_idx, 20000, cfg.n_edges)


def test_normal_features_are_standard():
    x = make_features("normal", 2000, 50, 1.0, np.random.default_rng(1))
    assert x.dtype == np.float32 and abs(x.mean()) < 0.02 and abs(x.std() - 1) < 0.02
