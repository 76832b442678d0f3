"""Pins of the oracle's Bi-GraphSAGE layer (Sec. 4.4.2) against things other than itself: a
hand-worked graph, the lossless special case in which the binarised layer equals the
full-precision mean-aggregator layer evaluated with library routines, and structural invariants."""
import numpy as np
import pytest
import scipy.sparse as sp

import oracle
from workloads import csr_from_undirected_edges

RNG = np.random.default_rng(4420221013)


def _graph(n, edges):
    """Neighbour-list CSR (no self-loops) of the distinct undirected edges in `edges`."""
    e = np.asarray(edges, dtype=np.int64).reshape(-1, 2)
    e = e[e[:, 0] != e[:, 1]]
    e = np.unique(np.sort(e, axis=1), axis=0)
    return csr_from_undirected_edges(n, e[:, 0], e[:, 1], self_loops=False)


def _lossless_inputs(n, d_in, d_out):
    """Inputs that binarisation represents exactly: every row of h has one magnitude, every
    column of each weight has one magnitude, so sign * scale reproduces the matrix."""
    h = RNG.choice([-1.0, 1.0], size=(n, d_in)) * RNG.uniform(0.5, 2.0, size=(n, 1))
    w_self = RNG.choice([-1.0, 1.0], size=(d_in, d_out)) * RNG.uniform(0.1, 1.0, size=(1, d_out))
    w_nbr = RNG.choice([-1.0, 1.0], size=(d_in, d_out)) * RNG.uniform(0.1, 1.0, size=(1, d_out))
    return h.astype(np.float32), w_self.astype(np.float32), w_nbr.astype(np.float32)


def test_mean_norm_hand_graph():
    # path 0-1-2 plus an isolated node 3: degrees 1, 2, 1, 0
    row_ptr, col_idx = _graph(4, [(0, 1), (1, 2)])
    assert row_ptr.tolist() == [0, 1, 3, 4, 4]
    assert col_idx.tolist() == [1, 0, 2, 1]
    assert oracle.mean_norm(row_ptr, col_idx).tolist() == [1.0, 0.5, 0.5, 1.0]


def test_sage_layer_hand_worked():
    """Star with centre 0 and leaves 1, 2; two input features, one output column.
    h rows: (2, -4), (1, 1), (-3, 1)  ->  signs (+,-), (+,+), (-,+); beta = 3, 1, 2.
    W_theta = (0.5, -1.5)^T -> signs (+,-), alpha = 1;  W_n = (-2, -4)^T -> signs (-,-), alpha = 3.
    Sign inner products with W_theta: 2, 0, -2; with W_n: 0, -2, 0.
    zeta_self = beta * 1 * (2, 0, -2) = (6, 0, -4); zeta_nbr = beta * 3 * (0, -2, 0) = (0, -6, 0).
    out_0 = 6 + (zeta_nbr_1 + zeta_nbr_2)/2 = 6 - 3 = 3; out_1 = 0 + zeta_nbr_0 = 0; out_2 = -4 + 0."""
    row_ptr, col_idx = _graph(3, [(0, 1), (0, 2)])
    h = np.array([[2, -4], [1, 1], [-3, 1]], dtype=np.float32)
    w_self = np.array([[0.5], [-1.5]], dtype=np.float32)
    w_nbr = np.array([[-2.0], [-4.0]], dtype=np.float32)
    rec = oracle.sage_layer(row_ptr, col_idx, oracle.mean_norm(row_ptr, col_idx), h, w_self, w_nbr)
    assert rec["out"][:, 0].tolist() == [3.0, 0.0, -4.0]


@pytest.mark.parametrize("n,d_in,d_out", [(40, 9, 5), (150, 70, 33)])
def test_lossless_case_equals_full_precision_mean_aggregator(n, d_in, d_out):
    """With inputs that binarisation reproduces exactly, the binarised layer is the layer it
    approximates (Sec. 4.4.2, the full-precision mean-aggregator layer without its ReLU):
    H W_theta + D^-1 A (H W_n), here with scipy's sparse product and numpy's matmul."""
    edges = RNG.integers(0, n, size=(4 * n, 2))
    edges = edges[edges[:, 0] != edges[:, 1]]
    row_ptr, col_idx = _graph(n, edges)
    h, w_self, w_nbr = _lossless_inputs(n, d_in, d_out)
    rec = oracle.sage_layer(row_ptr, col_idx, oracle.mean_norm(row_ptr, col_idx), h, w_self, w_nbr)
    adj = sp.csr_matrix((np.ones(col_idx.size), col_idx, row_ptr), shape=(n, n))
    deg = np.asarray(adj.sum(axis=1)).ravel()
    inv = np.where(deg > 0, 1.0 / np.maximum(deg, 1), 0.0)
    h64 = h.astype(np.float64)
    want = h64 @ w_self.astype(np.float64) + sp.diags(inv) @ (adj @ (h64 @ w_nbr.astype(np.float64)))
    assert np.allclose(rec["out"], want, rtol=1e-12, atol=1e-12)
    # the two weights play different roles: swapping them must change the result
    swapped = oracle.sage_layer(row_ptr, col_idx, oracle.mean_norm(row_ptr, col_idx), h, w_nbr, w_self)
    assert not np.allclose(swapped["out"], want, rtol=1e-6)


def test_isolated_node_keeps_only_its_own_term_and_identical_neighbours_average_to_one():
    # node 4 isolated; nodes 1, 2, 3 carry the same features and are the neighbours of node 0
    row_ptr, col_idx = _graph(5, [(0, 1), (0, 2), (0, 3)])
    d_in, d_out = 19, 7
    h = RNG.standard_normal((5, d_in)).astype(np.float32)
    h[2] = h[1]
    h[3] = h[1]
    w_self = RNG.standard_normal((d_in, d_out)).astype(np.float32)
    w_nbr = RNG.standard_normal((d_in, d_out)).astype(np.float32)
    rec = oracle.sage_layer(row_ptr, col_idx, oracle.mean_norm(row_ptr, col_idx), h, w_self, w_nbr)
    assert np.array_equal(rec["out"][4], rec["zeta_self"][4])
    # mean of three identical neighbour terms is that term
    assert np.allclose(rec["out"][0], rec["zeta_self"][0] + rec["zeta_nbr"][1], rtol=1e-13, atol=0)
    # a leaf sees exactly its single neighbour
    assert np.allclose(rec["out"][1], rec["zeta_self"][1] + rec["zeta_nbr"][0], rtol=1e-13, atol=0)


def test_terms_are_the_binary_products_of_sec_4_2():
    """Each term is beta_i * alpha_j * (sign inner product): checked against float matmuls of the
    +-1 matrices (a library routine) rather than the oracle's integer loop."""
    n, d_in, d_out = 30, 45, 11
    row_ptr, col_idx = _graph(n, RNG.integers(0, n, size=(60, 2)))
    h = RNG.standard_normal((n, d_in)).astype(np.float32)
    w_self = RNG.standard_normal((d_in, d_out)).astype(np.float32)
    w_nbr = RNG.standard_normal((d_in, d_out)).astype(np.float32)
    rec = oracle.sage_layer(row_ptr, col_idx, oracle.mean_norm(row_ptr, col_idx), h, w_self, w_nbr)
    h64 = h.astype(np.float64)
    s = np.where(h64 >= 0, 1.0, -1.0)
    beta = np.abs(h64).mean(axis=1)
    for w, key in ((w_self, "zeta_self"), (w_nbr, "zeta_nbr")):
        w64 = w.astype(np.float64)
        want = beta[:, None] * (s @ np.where(w64 >= 0, 1.0, -1.0)) * np.abs(w64).mean(axis=0)[None, :]
        assert np.allclose(rec[key], want, rtol=1e-12, atol=1e-12)


def test_permutation_equivariance():
    n, d_in, d_out = 25, 12, 6
    edges = RNG.integers(0, n, size=(50, 2))
    edges = edges[edges[:, 0] != edges[:, 1]]
    row_ptr, col_idx = _graph(n, edges)
    h = RNG.standard_normal((n, d_in)).astype(np.float32)
    w = (RNG.standard_normal((d_in, d_out)).astype(np.float32),
         RNG.standard_normal((d_in, d_out)).astype(np.float32))
    out, _ = oracle.sage_forward(row_ptr, col_idx, h, [w])
    perm = RNG.permutation(n)            # new label of node v is perm[v]
    row_ptr_p, col_idx_p = _graph(n, perm[edges])
    h_p = np.empty_like(h)
    h_p[perm] = h
    out_p, _ = oracle.sage_forward(row_ptr_p, col_idx_p, h_p, [w])
    assert np.allclose(out_p[perm], out, rtol=1e-12, atol=1e-13)


def test_two_layer_forward_chains_the_layers_and_standardises_inputs():
    n, dims = 60, (20, 16, 5)
    edges = RNG.integers(0, n, size=(150, 2))
    edges = edges[edges[:, 0] != edges[:, 1]]
    row_ptr, col_idx = _graph(n, edges)
    x = RNG.standard_normal((n, dims[0])).astype(np.float32) + 3.0     # far from zero mean
    ws = [(RNG.standard_normal((dims[l], dims[l + 1])).astype(np.float32),
           RNG.standard_normal((dims[l], dims[l + 1])).astype(np.float32)) for l in range(2)]
    out, used = oracle.sage_forward(row_ptr, col_idx, x, ws, calibrate=[True, True])
    coeff = oracle.mean_norm(row_ptr, col_idx)
    # first layer's standardisation is the column mean / variance of x (numpy, independent)
    assert np.allclose(used[0][0], x.astype(np.float64).mean(axis=0), rtol=1e-6)
    assert np.allclose(used[0][1], 1 / np.sqrt(x.astype(np.float64).var(axis=0) + 1e-5), rtol=1e-6)
    h1 = oracle.sage_layer(row_ptr, col_idx, coeff, x, ws[0][0], ws[0][1], *used[0])["out"]
    h2 = oracle.sage_layer(row_ptr, col_idx, coeff, h1, ws[1][0], ws[1][1], *used[1])["out"]
    assert np.array_equal(out, h2)
    # without the shift every sign of the first layer would be +1: the result must differ
    plain, _ = oracle.sage_forward(row_ptr, col_idx, x, ws)
    assert not np.allclose(plain, out)
