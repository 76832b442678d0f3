"""Pins of the oracle's Bi-GAT layer (Sec. 4.4.1) against things other than itself: the uniform-
attention special case (equal to the mean aggregator, an independently pinned routine), a
hand-worked graph, dense linear algebra with a library softmax, and structural properties."""
import numpy as np
import pytest
import scipy.sparse as sp
from scipy.special import softmax

import oracle
from workloads import chung_lu_csr

RNG = np.random.default_rng(441_2022)


def _case(n=50, n_edges=160, d_in=13, d_out=8, seed=2):
    rp, ci = chung_lu_csr(n, n_edges, 2.5, 2.0, seed=seed)
    h = RNG.standard_normal((n, d_in)).astype(np.float32)
    w = RNG.standard_normal((d_in, d_out)).astype(np.float32)
    return rp, ci, h, w


def test_zero_attention_vector_gives_the_mean_over_the_row():
    rp, ci, h, w = _case()
    zero = np.zeros((2, 4))
    rec = oracle.gat_layer(rp, ci, h, w, zero, zero, heads=2)
    want = oracle.aggregate(rp, ci, oracle.mean_norm(rp, ci), rec["zeta"])
    assert np.allclose(rec["out"], want, rtol=1e-13, atol=1e-15)
    fwd = oracle.layer(rp, ci, oracle.gcn_norm(rp, ci), h, w)
    assert np.array_equal(rec["zeta"], fwd["zeta"])          # z_j is the binarised product of Sec. 4.2


def test_hand_worked_two_neighbours():
    """Node 0 with N_0 = {0, 1}; one input feature, one output column, one head.
    h = (2, -1): signs (+, -), beta = (2, 1); W = (0.5): B = +, alpha = 0.5; z = (1, -0.5).
    a_src = 1, a_dst = 2: e_00 = 1 + 2 = 3, e_01 = 1 - 1 = 0 (LeakyReLU leaves both).
    softmax(3, 0) = (e^3, 1) / (e^3 + 1); out_0 = (e^3 - 0.5) / (e^3 + 1).
    Node 1 with N_1 = {0, 1}: e_10 = -0.5 + 2 = 1.5, e_11 = -0.5 - 1 = -1.5 -> slope 0.2 -> -0.3;
    out_1 = (e^1.5 - 0.5 e^-0.3) / (e^1.5 + e^-0.3)."""
    rp = np.array([0, 2, 4], dtype=np.int64)
    ci = np.array([0, 1, 0, 1], dtype=np.int32)
    h = np.array([[2.0], [-1.0]], dtype=np.float32)
    w = np.array([[0.5]], dtype=np.float32)
    rec = oracle.gat_layer(rp, ci, h, w, np.array([[1.0]]), np.array([[2.0]]), heads=1, negative_slope=0.2)
    e3 = np.exp(3.0)
    assert rec["out"][0, 0] == pytest.approx((e3 - 0.5) / (e3 + 1.0), rel=1e-13)
    a, b = np.exp(1.5), np.exp(-0.3)
    assert rec["out"][1, 0] == pytest.approx((a - 0.5 * b) / (a + b), rel=1e-13)


@pytest.mark.parametrize("heads", [1, 2, 4])
def test_against_dense_algebra_with_a_library_softmax(heads):
    rp, ci, h, w = _case(n=30, n_edges=90, d_in=9, d_out=8, seed=5)
    n, d_out = 30, 8
    dh = d_out // heads
    a_src = RNG.standard_normal((heads, dh))
    a_dst = RNG.standard_normal((heads, dh))
    rec = oracle.gat_layer(rp, ci, h, w, a_src, a_dst, heads=heads, negative_slope=0.1)
    # z from float matmuls of the +-1 matrices
    h64, w64 = h.astype(np.float64), w.astype(np.float64)
    z = (np.abs(h64).mean(axis=1)[:, None] * (np.where(h64 >= 0, 1.0, -1.0) @ np.where(w64 >= 0, 1.0, -1.0))
         * np.abs(w64).mean(axis=0)[None, :])
    mask = sp.csr_matrix((np.ones(ci.size), ci, rp), shape=(n, n)).toarray() > 0
    want = np.zeros((n, d_out))
    for hd in range(heads):
        zh = z[:, hd * dh:(hd + 1) * dh]
        e = (zh @ a_src[hd])[:, None] + (zh @ a_dst[hd])[None, :]
        e = np.where(e > 0, e, 0.1 * e)
        e = np.where(mask, e, -np.inf)
        want[:, hd * dh:(hd + 1) * dh] = softmax(e, axis=1) @ zh
    assert np.allclose(rec["out"], want, rtol=1e-11, atol=1e-13)
    # attention weights of every row sum to one per head
    sums = np.add.reduceat(rec["att"], rp[:-1], axis=0)
    assert np.allclose(sums, 1.0, rtol=1e-13)


def test_source_and_destination_vectors_play_different_roles_and_shift_invariance():
    rp, ci, h, w = _case()
    a_src = RNG.standard_normal((1, 8))
    a_dst = RNG.standard_normal((1, 8))
    rec = oracle.gat_layer(rp, ci, h, w, a_src, a_dst)
    swapped = oracle.gat_layer(rp, ci, h, w, a_dst, a_src)
    assert not np.allclose(rec["out"], swapped["out"])
    # with slope 1 the LeakyReLU is the identity and a_src . z_i is constant inside row i's
    # softmax: it cancels
    lin = oracle.gat_layer(rp, ci, h, w, a_src, a_dst, negative_slope=1.0)
    lin0 = oracle.gat_layer(rp, ci, h, w, 0 * a_src, a_dst, negative_slope=1.0)
    assert np.allclose(lin["out"], lin0["out"], rtol=1e-10, atol=1e-13)


def test_empty_row_and_single_neighbour():
    # node 2 has no entries; node 0 lists only node 1
    rp = np.array([0, 1, 3, 3], dtype=np.int64)
    ci = np.array([1, 0, 1], dtype=np.int32)
    h = RNG.standard_normal((3, 5)).astype(np.float32)
    w = RNG.standard_normal((5, 4)).astype(np.float32)
    rec = oracle.gat_layer(rp, ci, h, w, RNG.standard_normal((2, 2)), RNG.standard_normal((2, 2)), heads=2)
    assert np.array_equal(rec["out"][2], np.zeros(4))
    assert np.allclose(rec["out"][0], rec["zeta"][1], rtol=1e-15)


def test_gat_on_a_subset_of_nodes_equals_the_rows_of_the_full_result():
    rng = np.random.default_rng(21)
    n, d_in, d_out, heads = 60, 20, 8, 2
    u = rng.integers(0, n, 200)
    v = rng.integers(0, n, 200)
    keep = u != v
    pairs = np.unique(np.sort(np.stack([u[keep], v[keep]], axis=1), axis=1), axis=0)
    from workloads import csr_from_undirected_edges
    rp, ci = csr_from_undirected_edges(n, pairs[:, 0], pairs[:, 1])
    x = rng.standard_normal((n, d_in))
    w = rng.standard_normal((d_in, d_out))
    a_src = rng.standard_normal((heads, d_out // heads))
    a_dst = rng.standard_normal((heads, d_out // heads))
    full = oracle.gat_layer(rp, ci, x, w, a_src, a_dst, heads=heads)
    nodes = np.array([3, 17, 59, 0])
    part = oracle.gat_layer(rp, ci, x, w, a_src, a_dst, heads=heads, nodes=nodes)
    assert np.array_equal(part["out"][nodes], full["out"][nodes])
    rest = np.setdiff1d(np.arange(n), nodes)
    assert not part["out"][rest].any()
    assert np.array_equal(part["zeta"], full["zeta"])
