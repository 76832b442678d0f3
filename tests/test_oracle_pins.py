"""Pins of the CPU oracle against things other than itself: brute force on tiny inputs, closed
forms of Sec. 4.1, hand-built graphs, dense linear algebra and library routines."""
import itertools

import numpy as np
import pytest
import scipy.sparse as sp

import oracle
from workloads import chung_lu_csr, csr_from_undirected_edges

RNG = np.random.default_rng(20221013)


# ----------------------------------------------------------------------------------------
# vector binarisation (Sec. 4.1): V_B = sign(V), alpha = ||V||_1 / t minimise ||V - alpha V_B||^2
# ----------------------------------------------------------------------------------------
def test_binarize_hand_example():
    x = np.array([[1.0, -2.0, 0.5, -0.5], [3.0, 3.0, -1.0, 1.0]], dtype=np.float32)
    sign, scale = oracle.binarize_rows(x)
    assert sign.tolist() == [[1, -1, 1, -1], [1, 1, -1, 1]]
    assert scale.tolist() == [1.0, 2.0]


def test_binarize_zero_and_negative_zero_are_plus_one():
    x = np.array([[0.0, -0.0, -1e-30, 1e-30]], dtype=np.float32)
    sign, scale = oracle.binarize_rows(x)
    assert sign.tolist() == [[1, 1, -1, 1]]
    assert scale[0] == pytest.approx(0.5e-30, rel=1e-6)


def test_binarize_is_the_least_squares_optimum():
    x = RNG.standard_normal((16, 37)).astype(np.float32)
    sign, scale = oracle.binarize_rows(x)
    x64 = x.astype(np.float64)
    for r in range(x.shape[0]):
        t = x.shape[1]
        cost = lambda a, s=sign[r]: float(np.sum((x64[r] - a * s) ** 2))
        j_star = cost(scale[r])
        # closed-form minimum  ||V||_2^2 - ||V||_1^2 / t
        assert j_star == pytest.approx(np.sum(x64[r] ** 2) - np.sum(np.abs(x64[r])) ** 2 / t,
                                       rel=1e-12)
        for eps in (1e-3, -1e-3):
            assert cost(scale[r] + eps) > j_star
        # any other sign pattern with its own best scale is no better
        for _ in range(20):
            flip = sign[r].copy()
            flip[RNG.integers(0, t)] *= -1
            a = float(np.dot(x64[r], flip)) / t
            assert float(np.sum((x64[r] - a * flip) ** 2)) >= j_star - 1e-12


def test_binarize_scale_invariances():
    x = RNG.standard_normal((8, 70)).astype(np.float32)
    x[x == 0] = 1.0
    s0, a0 = oracle.binarize_rows(x)
    s1, a1 = oracle.binarize_rows((4.0 * x).astype(np.float32))
    assert np.array_equal(s0, s1) and np.allclose(a1, 4.0 * a0, rtol=1e-12)
    s2, a2 = oracle.binarize_rows(-x)
    assert np.array_equal(s2, -s0) and np.allclose(a2, a0, rtol=1e-12)


def test_binarize_weight_uses_columns_and_divides_by_d_in():
    # 3 inputs, 2 outputs: column 0 = (1, -2, 3), column 1 = (-4, 0, 2)
    w = np.array([[1.0, -4.0], [-2.0, 0.0], [3.0, 2.0]], dtype=np.float32)
    bt, alpha = oracle.binarize_weight(w)
    assert bt.shape == (2, 3)
    assert bt.tolist() == [[1, -1, 1], [-1, 1, 1]]
    assert alpha.tolist() == [2.0, 2.0]            # 6/3 and 6/3, not 6/2
    w2 = RNG.standard_normal((50, 7)).astype(np.float32)
    bt2, alpha2 = oracle.binarize_weight(w2)
    assert np.array_equal(bt2, np.where(w2.T >= 0, 1, -1))
    assert np.allclose(alpha2, np.abs(w2.astype(np.float64)).sum(axis=0) / 50, rtol=1e-13)


def test_binarize_with_standardisation():
    x = np.array([[1.0, 5.0, 2.0], [3.0, 1.0, 2.0]], dtype=np.float32)
    shift = np.array([2.0, 3.0, 2.0], dtype=np.float32)
    mul = np.array([0.5, 2.0, 10.0], dtype=np.float32)
    sign, scale = oracle.binarize_rows(x, shift, mul)
    assert sign.tolist() == [[-1, 1, 1], [1, -1, 1]]
    assert scale.tolist() == [(0.5 + 4.0 + 0.0) / 3, (0.5 + 4.0 + 0.0) / 3]
    # fp64 input path takes the sign on the fp32-rounded value and the same scale
    sign64, scale64 = oracle.binarize_rows(x.astype(np.float64), shift, mul)
    assert np.array_equal(sign, sign64) and np.array_equal(scale, scale64)
    # a value that rounds up to the threshold in fp32 counts as +1
    th = np.array([1.0], dtype=np.float32)
    s, _ = oracle.binarize_rows(np.array([[1.0 - 1e-12]], dtype=np.float64), th, None)
    assert s.tolist() == [[1]]


def test_column_standardisation_closed_form():
    h = np.array([[1.0, 10.0], [3.0, 10.0], [5.0, 16.0]], dtype=np.float64)
    shift, mul = oracle.column_standardisation(h, eps=0.0)
    assert shift.tolist() == [3.0, 12.0]
    assert np.allclose(mul, [1 / np.sqrt(8 / 3), 1 / np.sqrt(8.0)], rtol=1e-6)
    x = RNG.standard_normal((500, 9)) * 3 + 2
    shift, mul = oracle.column_standardisation(x)
    y = (x - shift) * mul
    assert np.allclose(y.mean(axis=0), 0, atol=1e-5) and np.allclose(y.var(axis=0), 1, atol=1e-4)


# ----------------------------------------------------------------------------------------
# packed layout
# ----------------------------------------------------------------------------------------
def test_pack_hand_written_row():
    sign = -np.ones((1, 70), dtype=np.int8)
    sign[0, [0, 3, 63, 64, 69]] = 1
    words = oracle.pack_bits(sign)
    assert words.shape == (1, 2) and words.dtype == np.dtype("<u8")
    assert int(words[0, 0]) == (1 << 0) | (1 << 3) | (1 << 63)
    assert int(words[0, 1]) == (1 << 0) | (1 << 5)          # bits 6.. are padding = 0


@pytest.mark.parametrize("cols", [1, 63, 64, 65, 100, 1433])
def test_pack_round_trip(cols):
    sign = RNG.choice(np.array([-1, 1], dtype=np.int8), size=(5, cols))
    words = oracle.pack_bits(sign)
    assert words.shape == (5, (cols + 63) // 64)
    assert np.array_equal(oracle.unpack_bits(words, cols), sign)
    pad = words.shape[1] * 64 - cols
    if pad:
        assert np.all(words[:, -1] >> np.uint64(64 - pad) == 0)


# ----------------------------------------------------------------------------------------
# +-1 inner products (Sec. 4.2.3): equal to K - 2 popcount(a xor b) on the packed words
# ----------------------------------------------------------------------------------------
def _popcount_dot(wa, wb, k):
    x = 0
    for a, b in zip(wa.tolist(), wb.tolist()):
        x += bin(int(a) ^ int(b)).count("1")
    return k - 2 * x


@pytest.mark.parametrize("k", [1, 2, 3, 5, 8])
def test_sign_matmul_all_pairs_brute_force(k):
    vecs = np.array(list(itertools.product([-1, 1], repeat=k)), dtype=np.int8)
    acc = oracle.sign_matmul(vecs, vecs)
    words = oracle.pack_bits(vecs)
    for i in range(vecs.shape[0]):
        for j in range(vecs.shape[0]):
            expect = sum(int(a) * int(b) for a, b in zip(vecs[i], vecs[j]))
            assert acc[i, j] == expect == _popcount_dot(words[i], words[j], k)


@pytest.mark.parametrize("k", [1, 63, 64, 65, 100, 1433, 3703])
def test_sign_matmul_against_integer_matmul_and_popcount(k):
    f = RNG.choice(np.array([-1, 1], dtype=np.int8), size=(9, k))
    bt = RNG.choice(np.array([-1, 1], dtype=np.int8), size=(4, k))
    acc = oracle.sign_matmul(f, bt)
    assert acc.shape == (9, 4) and acc.dtype == np.int32
    assert np.array_equal(acc, f.astype(np.int64) @ bt.astype(np.int64).T)
    wf, wb = oracle.pack_bits(f), oracle.pack_bits(bt)
    for i in range(9):
        for j in range(4):
            assert acc[i, j] == _popcount_dot(wf[i], wb[j], k)
    assert np.all((acc - k) % 2 == 0) and np.all(np.abs(acc) <= k)
    perm = RNG.permutation(k)
    assert np.array_equal(oracle.sign_matmul(f[:, perm], bt[:, perm]), acc)


def test_rescale():
    acc = np.array([[3, -1, 0], [-5, 7, 2]], dtype=np.int32)
    ones = oracle.rescale(acc, np.ones(2), np.ones(3))
    assert np.array_equal(ones, acc.astype(np.float64))
    z = oracle.rescale(acc, np.array([2.0, 0.5]), np.array([1.0, 10.0, -3.0]))
    assert z.tolist() == [[6.0, -20.0, -0.0], [-2.5, 35.0, -3.0]]


# ----------------------------------------------------------------------------------------
# normalised adjacency (Sec. 3.1 / Eq. (1)) on hand-built graphs
# ----------------------------------------------------------------------------------------
def _graph(n, edges):
    u = np.array([e[0] for e in edges], dtype=np.int64)
    v = np.array([e[1] for e in edges], dtype=np.int64)
    return csr_from_undirected_edges(n, u, v)


def _dense(row_ptr, col_idx, vals):
    n = row_ptr.size - 1
    return sp.csr_matrix((vals, col_idx, row_ptr), shape=(n, n)).toarray()


def test_gcn_norm_complete_graph_k4():
    rp, ci = _graph(4, [(0, 1), (0, 2), (0, 3), (1, 2), (1, 3), (2, 3)])
    a = oracle.gcn_norm(rp, ci)
    assert a.shape == (16,) and np.allclose(a, 0.25, rtol=1e-15)


def test_gcn_norm_six_cycle():
    rp, ci = _graph(6, [(i, (i + 1) % 6) for i in range(6)])
    assert np.allclose(oracle.gcn_norm(rp, ci), 1.0 / 3.0, rtol=1e-15)


def test_gcn_norm_path_p4():
    rp, ci = _graph(4, [(0, 1), (1, 2), (2, 3)])
    dense = _dense(rp, ci, oracle.gcn_norm(rp, ci))
    r6 = 1 / np.sqrt(6.0)
    expect = np.array([[1 / 2, r6, 0, 0], [r6, 1 / 3, 1 / 3, 0], [0, 1 / 3, 1 / 3, r6],
                       [0, 0, r6, 1 / 2]])
    assert np.allclose(dense, expect, rtol=1e-15)


def test_gcn_norm_star_s5_and_triangle_with_pendant():
    rp, ci = _graph(5, [(0, 1), (0, 2), (0, 3), (0, 4)])
    dense = _dense(rp, ci, oracle.gcn_norm(rp, ci))
    assert dense[0, 0] == pytest.approx(1 / 5) and dense[1, 1] == pytest.approx(1 / 2)
    assert np.allclose(dense[0, 1:], 1 / np.sqrt(10.0)) and np.allclose(dense[1:, 0], 1 / np.sqrt(10.0))
    rp, ci = _graph(4, [(0, 1), (1, 2), (0, 2), (2, 3)])   # degrees with loops: 3, 3, 4, 2
    dense = _dense(rp, ci, oracle.gcn_norm(rp, ci))
    assert dense[2, 3] == pytest.approx(1 / np.sqrt(8.0)) and dense[0, 2] == pytest.approx(1 / np.sqrt(12.0))
    assert dense[0, 3] == 0 and dense[0, 1] == pytest.approx(1 / 3)


def test_gcn_norm_random_graph_matches_dense_definition():
    n = 200
    rp, ci = chung_lu_csr(n, 700, 2.5, 2.0, seed=5)
    a_hat = _dense(rp, ci, np.ones(ci.size))
    assert np.array_equal(a_hat, a_hat.T) and np.all(np.diag(a_hat) == 1)
    d = a_hat.sum(axis=1)
    expect = np.diag(d ** -0.5) @ a_hat @ np.diag(d ** -0.5)
    dense = _dense(rp, ci, oracle.gcn_norm(rp, ci))
    assert np.allclose(dense, expect, rtol=1e-13, atol=0)
    assert np.allclose(dense, dense.T, rtol=0, atol=0)
    # sqrt(d) is an eigenvector of A~ with eigenvalue 1
    assert np.allclose(dense @ np.sqrt(d), np.sqrt(d), rtol=1e-12)


# ----------------------------------------------------------------------------------------
# aggregation (Sec. 4.2.3)
# ----------------------------------------------------------------------------------------
def test_aggregate_against_dense_and_scipy():
    n, d = 300, 13
    rp, ci = chung_lu_csr(n, 1500, 2.5, 3.0, seed=9)
    a = oracle.gcn_norm(rp, ci)
    z = RNG.standard_normal((n, d))
    out = oracle.aggregate(rp, ci, a, z)
    assert np.allclose(out, _dense(rp, ci, a) @ z, rtol=1e-12, atol=1e-14)
    assert np.allclose(out, sp.csr_matrix((a, ci, rp), shape=(n, n)) @ z, rtol=1e-12, atol=1e-14)
    # identity input returns the matrix itself; sqrt(degree) column reproduces itself
    assert np.array_equal(oracle.aggregate(rp, ci, a, np.eye(n)), _dense(rp, ci, a))
    rootd = np.sqrt(np.diff(rp).astype(np.float64))[:, None]
    assert np.allclose(oracle.aggregate(rp, ci, a, rootd), rootd, rtol=1e-12)


def test_aggregate_is_not_symmetric_in_its_operands():
    # unsymmetric coefficients: a transposed access would give a different answer
    rp, ci = _graph(3, [(0, 1), (1, 2)])
    vals = np.arange(1.0, ci.size + 1)
    z = np.array([[1.0, 0.0], [0.0, 1.0], [2.0, 2.0]])
    out = oracle.aggregate(rp, ci, vals, z)
    assert np.array_equal(out, _dense(rp, ci, vals) @ z)
    assert not np.array_equal(out, _dense(rp, ci, vals).T @ z)


# ----------------------------------------------------------------------------------------
# whole layer / forward against dense fp64 linear algebra
# ----------------------------------------------------------------------------------------
def _dense_forward(rp, ci, x, weights, bn):
    n = rp.size - 1
    a_hat = _dense(rp, ci, np.ones(ci.size))
    d = a_hat.sum(axis=1)
    a_t = a_hat / np.sqrt(np.outer(d, d))
    h = x.astype(np.float64)
    for w, p in zip(weights, bn):
        w = w.astype(np.float64)
        shift, mul = (np.zeros(h.shape[1]), np.ones(h.shape[1])) if p is None else (
            p[0].astype(np.float64), p[1].astype(np.float64))
        f = np.where(h.astype(np.float32) >= shift.astype(np.float32), 1.0, -1.0)
        beta = np.abs((h - shift) * mul).mean(axis=1)
        b = np.where(w >= 0, 1.0, -1.0)
        alpha = np.abs(w).mean(axis=0)
        h = a_t @ ((beta[:, None] * f) @ (b * alpha[None, :]))
    return h


def test_forward_matches_dense_linear_algebra():
    n, dims = 150, (45, 19, 6, 4)
    rp, ci = chung_lu_csr(n, 500, 2.5, 2.0, seed=21)
    x = RNG.standard_normal((n, dims[0])).astype(np.float32)
    weights = [RNG.uniform(-1, 1, size=(dims[l], dims[l + 1])).astype(np.float32) for l in range(3)]
    logits, recs = oracle.forward(rp, ci, x, weights, calibrate=[True, True, False], keep_trace=True)
    bn = [(r["shift"], r["mul"]) if r["shift"] is not None else None for r in recs]
    assert bn[2] is None and bn[1] is not None
    expect = _dense_forward(rp, ci, x, weights, bn)
    assert logits.shape == (n, 4)
    assert np.allclose(logits, expect, rtol=1e-10, atol=1e-13)
    # handing back the recorded parameters reproduces the same result without calibration
    again, _ = oracle.forward(rp, ci, x, weights, bn=bn)
    assert np.array_equal(again, logits)


def test_forward_equivariances():
    n, dims = 120, (33, 16, 5)
    rp, ci = chung_lu_csr(n, 400, 2.5, 2.0, seed=22)
    x = RNG.standard_normal((n, dims[0])).astype(np.float32)
    weights = [RNG.uniform(-1, 1, size=(dims[l], dims[l + 1])).astype(np.float32) for l in range(2)]
    base, _ = oracle.forward(rp, ci, x, weights)
    # permuting the output channels permutes the logits
    perm = RNG.permutation(dims[-1])
    out, _ = oracle.forward(rp, ci, x, [weights[0], weights[1][:, perm]])
    assert np.array_equal(out, base[:, perm])
    # relabelling the nodes permutes the rows (up to the order of the neighbour sum)
    relabel = RNG.permutation(n)                       # new id of old node i
    rows = np.repeat(np.arange(n), np.diff(rp))
    keep = rows < ci
    rp2, ci2 = csr_from_undirected_edges(n, relabel[rows[keep]], relabel[ci[keep]])
    x2 = np.empty_like(x)
    x2[relabel] = x
    out2, _ = oracle.forward(rp2, ci2, x2, weights)
    assert np.allclose(out2[relabel], base, rtol=1e-9, atol=1e-12)


# ----------------------------------------------------------------------------------------
# prediction (Sec. 3.2): softmax of the last layer's output, class = largest entry
# ----------------------------------------------------------------------------------------
def test_predict_hand_example_and_ties():
    h = np.array([[0.0, np.log(3.0)], [2.0, 2.0], [-1.0, -5.0]], dtype=np.float32)
    labels, probs = oracle.predict(h)
    assert labels.tolist() == [1, 0, 0]                       # tie -> lowest class
    assert np.allclose(probs[0], [0.25, 0.75], rtol=1e-6)     # fp32 log(3) in the input
    assert np.allclose(probs[1], [0.5, 0.5], rtol=1e-15)


def test_predict_matches_library_softmax_and_is_shift_invariant():
    from scipy.special import softmax
    h = (RNG.standard_normal((200, 47)) * 8).astype(np.float32)
    labels, probs = oracle.predict(h)
    assert np.allclose(probs, softmax(h.astype(np.float64), axis=1), rtol=1e-12, atol=1e-300)
    assert np.allclose(probs.sum(axis=1), 1.0, rtol=1e-14)
    assert np.array_equal(labels, probs.argmax(axis=1))
    shifted_labels, shifted = oracle.predict(h.astype(np.float64) + 1000.0)
    assert np.array_equal(shifted_labels, labels) and np.allclose(shifted, probs, rtol=1e-9)
    # large logits do not overflow
    _, big = oracle.predict(np.array([[1e4, 1e4 - 1.0]], dtype=np.float32))
    assert np.allclose(big[0], [1 / (1 + np.exp(-1.0)), 1 / (1 + np.exp(1.0))], rtol=1e-12)


# ----------------------------------------------------------------------------------------
# entropy of a hidden layer by binning (Sec. 6.2)
# ----------------------------------------------------------------------------------------
def test_binned_entropy_closed_forms():
    n, bins = 4096, 16
    uniform = (np.arange(n) % bins).astype(np.float32)               # every bin equally often
    two = np.where(np.arange(n) % 2 == 0, -3.0, 5.0).astype(np.float32)
    const = np.full(n, 2.5, dtype=np.float32)
    skew = np.where(np.arange(n) % 4 == 0, 1.0, 0.0).astype(np.float32)   # p = 1/4, 3/4
    h = np.stack([uniform, two, const, skew], axis=1)
    per, total, counts = oracle.binned_entropy(h, bins)
    want = [4.0, 1.0, 0.0, 2.0 - 0.75 * np.log2(3.0)]
    assert np.allclose(per, want, rtol=1e-12, atol=1e-15)
    assert total == pytest.approx(sum(want), rel=1e-12)
    assert counts.sum(axis=1).tolist() == [n] * 4
    assert counts[2, 0] == n and counts[1, 0] == n // 2 and counts[1, bins - 1] == n // 2


def test_binned_entropy_matches_library_histogram_and_entropy():
    from scipy.stats import entropy
    x = RNG.standard_normal((5000, 3)).astype(np.float32) * np.array([1.0, 7.0, 0.01], dtype=np.float32)
    bins = 50
    per, total, counts = oracle.binned_entropy(x, bins)
    for c in range(3):
        col = x[:, c].astype(np.float64)
        ref_counts, _ = np.histogram(col, bins=bins, range=(col.min(), col.max()))
        # fp32 and fp64 bin edges may disagree on a value that sits on an edge: at most a handful
        assert np.abs(ref_counts - counts[c]).sum() <= 6
        assert per[c] == pytest.approx(entropy(counts[c], base=2), rel=1e-12)
    assert total == pytest.approx(per.sum(), rel=1e-15)
    # more samples of the same law, finer bins: entropy grows by about log2 of the refinement
    per2, _, _ = oracle.binned_entropy(x, 2 * bins)
    assert np.all(per2 > per) and np.all(per2 < per + 1.0 + 1e-9)
