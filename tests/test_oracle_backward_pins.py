"""Pins of the oracle's back propagation through one binarised layer (Sec. 4.3, Algorithm 1)
against things other than itself: adjoint identities with the forward routines, finite
differences of the functions that are truly differentiable, dense linear algebra, and hand-worked
values for the two straight-through rules."""
import numpy as np
import pytest
import scipy.sparse as sp

import oracle
from workloads import chung_lu_csr

RNG = np.random.default_rng(43_2022)


def _small(n=60, n_edges=200, d_in=11, d_out=5, seed=1):
    rp, ci = chung_lu_csr(n, n_edges, 2.5, 2.0, seed=seed)
    a = oracle.gcn_norm(rp, ci)
    h = RNG.standard_normal((n, d_in)).astype(np.float32)
    w = (RNG.standard_normal((d_in, d_out)) * 0.8).astype(np.float32)
    g = RNG.standard_normal((n, d_out)) * 0.05
    return rp, ci, a, h, w, g


def test_aggregate_transposed_is_the_adjoint_of_aggregate_on_an_asymmetric_matrix():
    # arbitrary (non-symmetric) coefficients on a symmetric pattern, and a dense reference
    rp, ci, _, _, _, _ = _small()
    n = rp.size - 1
    coeff = RNG.standard_normal(ci.size)
    z = RNG.standard_normal((n, 4))
    g = RNG.standard_normal((n, 4))
    lhs = np.sum(oracle.aggregate(rp, ci, coeff, z) * g)
    rhs = np.sum(z * oracle.aggregate_transposed(rp, ci, coeff, g))
    assert lhs == pytest.approx(rhs, rel=1e-12)
    dense = sp.csr_matrix((coeff, ci, rp), shape=(n, n)).toarray()
    assert np.allclose(oracle.aggregate_transposed(rp, ci, coeff, g), dense.T @ g, rtol=1e-12, atol=1e-13)
    # and it differs from the untransposed product: a transposed operand would be caught
    assert not np.allclose(dense.T @ g, dense @ g)


def test_gradients_of_the_binarised_operands_by_finite_differences():
    """With H~ and W~ as free real matrices, L = <g_out, A~ (H~ W~)> is bilinear: its exact
    partial derivatives are what Algorithm 1 calls dL/dW~ and dL/dH~."""
    rp, ci, a, h, w, g_out = _small()
    sign, beta = oracle.binarize_rows(h)
    rec = oracle.layer_backward(rp, ci, a, g_out, sign, beta, w)
    h_t, w_t = rec["h_tilde"], rec["w_tilde"]

    def loss(ht, wt):
        return float(np.sum(g_out * oracle.aggregate(rp, ci, a, ht @ wt)))

    eps = 1e-6
    for (i, j) in [(0, 0), (3, 2), (10, 4)]:
        d = np.zeros_like(w_t)
        d[i, j] = eps
        fd = (loss(h_t, w_t + d) - loss(h_t, w_t - d)) / (2 * eps)
        assert rec["g_wt"][i, j] == pytest.approx(fd, rel=1e-6, abs=1e-9)
    for (i, t) in [(0, 0), (17, 5), (59, 10)]:
        d = np.zeros_like(h_t)
        d[i, t] = eps
        fd = (loss(h_t + d, w_t) - loss(h_t - d, w_t)) / (2 * eps)
        assert rec["g_ht"][i, t] == pytest.approx(fd, rel=1e-6, abs=1e-9)
    # the binarised operands are the forward's: H~ W~ is zeta
    fwd = oracle.layer(rp, ci, a, h, w)
    assert np.allclose(h_t @ w_t, fwd["zeta"], rtol=1e-12, atol=1e-12)


def test_weight_gradient_equals_the_true_derivative_where_sign_is_locally_constant():
    """For |W_ij| >= 1 the straight-through term vanishes and dL/dW_ij is an ordinary derivative
    of L(W~(W)) = <g_wt, alpha(W) B(W)> (the sign does not change under a small step): finite
    differences of the oracle's own weight binarisation."""
    d_in, d_out = 9, 4
    w = RNG.uniform(1.0, 3.0, size=(d_in, d_out)) * RNG.choice([-1.0, 1.0], size=(d_in, d_out))
    w = w.astype(np.float32)
    g_wt = RNG.standard_normal((d_in, d_out))
    got = oracle.weight_gradient(w, g_wt)

    def surrogate(wm):
        bt, alpha = oracle.binarize_weight(wm.astype(np.float32))
        return float(np.sum(g_wt * (alpha[None, :] * bt.T)))

    eps = 1e-3          # exactly representable steps keep fp32 rounding out of the difference
    for (i, j) in [(0, 0), (4, 1), (8, 3)]:
        d = np.zeros((d_in, d_out))
        d[i, j] = eps
        fd = (surrogate(w.astype(np.float64) + d) - surrogate(w.astype(np.float64) - d)) / (2 * eps)
        assert got[i, j] == pytest.approx(fd, rel=2e-4)


def test_weight_gradient_hand_worked_with_straight_through_term():
    """One column, d_in = 2: W = (0.5, -2)^T -> B = (+1, -1), alpha = 1.25.  g_wt = (4, 1)^T.
    Column sum: 4*1 + 1*(-1) = 3.  First term: B_i * 3 / 2 = (1.5, -1.5).
    Straight-through term: alpha * g_wt_i * 1[|W_i| < 1] = (1.25*4, 0) = (5, 0).
    dL/dW = (6.5, -1.5)."""
    got = oracle.weight_gradient(np.array([[0.5], [-2.0]], dtype=np.float32), np.array([[4.0], [1.0]]))
    assert got[:, 0].tolist() == [6.5, -1.5]
    # |W| exactly 1 is outside the open interval
    edge = oracle.weight_gradient(np.array([[1.0], [-1.0]], dtype=np.float32), np.array([[4.0], [1.0]]))
    assert edge[:, 0].tolist() == [1.5, -1.5]


def test_clipped_straight_through_rule_on_the_input_gradient():
    rp, ci, a, h, w, g_out = _small()
    sign, beta = oracle.binarize_rows(h)
    rec = oracle.layer_backward(rp, ci, a, 40.0 * g_out, sign, beta, w)   # gradients on both sides of 1
    big = np.abs(rec["g_ht"]) >= 1.0
    assert big.any() and (~big).any()
    assert np.all(rec["g_h"][big] == 0.0)
    assert np.array_equal(rec["g_h"][~big], rec["g_ht"][~big])
    # frozen standardisation of the layer input: one more per-column factor
    mul = RNG.uniform(0.5, 2.0, size=h.shape[1]).astype(np.float32)
    rec2 = oracle.layer_backward(rp, ci, a, 40.0 * g_out, sign, beta, w, mul=mul)
    assert np.allclose(rec2["g_in"], rec["g_h"] * mul[None, :].astype(np.float64), rtol=1e-15)
    assert np.array_equal(rec["g_in"], rec["g_h"])


def test_layer_backward_against_dense_algebra():
    rp, ci, a, h, w, g_out = _small(n=40, n_edges=120, d_in=7, d_out=3, seed=9)
    n = rp.size - 1
    sign, beta = oracle.binarize_rows(h)
    rec = oracle.layer_backward(rp, ci, a, g_out, sign, beta, w)
    a_dense = sp.csr_matrix((a, ci, rp), shape=(n, n)).toarray()
    h_t = np.abs(h.astype(np.float64)).mean(axis=1)[:, None] * np.where(h >= 0, 1.0, -1.0)
    w64 = w.astype(np.float64)
    w_t = np.abs(w64).mean(axis=0)[None, :] * np.where(w64 >= 0, 1.0, -1.0)
    g_zeta = a_dense.T @ g_out
    assert np.allclose(rec["g_zeta"], g_zeta, rtol=1e-12, atol=1e-14)
    assert np.allclose(rec["g_wt"], h_t.T @ g_zeta, rtol=1e-12, atol=1e-14)
    assert np.allclose(rec["g_ht"], g_zeta @ w_t.T, rtol=1e-12, atol=1e-14)
