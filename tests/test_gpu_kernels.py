"""Kernel-level parity of the HIP library against the CPU oracle, through the C ABI.

Integer work (packed sign bits, +-1 product accumulators) must match bit for bit; fp32
outputs must agree within 1e-5 relative with a 1e-6 absolute floor (tests/helpers.py).
"""
import numpy as np
import pytest

import oracle
from helpers import assert_close, to_device, words_to_numpy
from workloads import chung_lu_csr, csr_from_undirected_edges

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import torch
    from paper_2210_13149_amd import binding
    assert torch.cuda.is_available()
    binding.lib()          # fails loudly when the HIP library is missing
    return binding


def _rng(seed):
    return np.random.default_rng(seed)


# ------------------------------------------------------------------------------------------
# kernel 1: binarise + pack
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("rows,cols", [(1, 1), (3, 63), (5, 64), (7, 65), (1001, 100), (513, 128),
                                       (130, 200), (257, 256), (66, 602), (31, 1433), (9, 3703),
                                       (4, 4097), (2, 8192), (8193, 1100), (9000, 1024), (300, 1023)])
@pytest.mark.parametrize("bn", [False, True])
def test_pack_rows(B, rows, cols, bn):
    import torch
    rng = _rng(rows * 10007 + cols)
    x = rng.standard_normal((rows, cols)).astype(np.float32)
    x[rng.random(x.shape) < 0.05] = 0.0          # exact zeros and ties with the threshold
    shift = mul = None
    if bn:
        shift = rng.standard_normal(cols).astype(np.float32) * 0.3
        mul = (0.5 + rng.random(cols)).astype(np.float32)
        x[0, : min(cols, 8)] = shift[: min(cols, 8)]        # x == threshold -> +1
    sign, scale = oracle.binarize_rows(x, shift, mul)
    dx, dshift, dmul = to_device(x, shift, mul)
    bits, dscale = B.bigcn_pack(dx, dshift, dmul)
    torch.cuda.synchronize()
    assert np.array_equal(words_to_numpy(bits), oracle.pack_bits(sign))
    assert_close(dscale.cpu().numpy(), scale, "scale")


def test_pack_special_values_and_strides(B):
    import torch
    x = np.array([[0.0, -0.0, 1e-30, -1e-30, 5.0, -5.0, 0.0]], dtype=np.float32)
    sign, scale = oracle.binarize_rows(x)
    bits, dscale = B.bigcn_pack(to_device(x))
    assert int(words_to_numpy(bits)[0, 0]) == 0b1010111
    assert_close(dscale.cpu().numpy(), scale)
    # a padded row stride, a wider output leading dimension
    big = _rng(3).standard_normal((40, 300)).astype(np.float32)
    view = to_device(big)[:, 10:150]
    sign, scale = oracle.binarize_rows(big[:, 10:150])
    bits, dscale = B.bigcn_pack(view, ld_words=5)
    torch.cuda.synchronize()
    got = words_to_numpy(bits)
    assert got.shape == (40, 5)
    assert np.array_equal(got[:, :3], oracle.pack_bits(sign)) and np.all(got[:, 3:] == 0)
    assert_close(dscale.cpu().numpy(), scale)


@pytest.mark.parametrize("d_in,d_out", [(1433, 64), (64, 7), (100, 256), (3703, 64), (602, 128), (5, 3)])
def test_pack_weight_columns(B, d_in, d_out):
    rng = _rng(d_in + d_out)
    w = rng.uniform(-1, 1, size=(d_in, d_out)).astype(np.float32)
    bt, alpha = oracle.binarize_weight(w)
    bits, dalpha = B.pack_weight(to_device(w))
    assert np.array_equal(words_to_numpy(bits), oracle.pack_bits(bt))
    assert_close(dalpha.cpu().numpy(), alpha, "alpha")


# ------------------------------------------------------------------------------------------
# kernel 2: bit-GEMM
# ------------------------------------------------------------------------------------------
GEMM_SHAPES = [(1, 1, 1), (5, 3, 64), (67, 7, 65), (300, 41, 128), (1000, 47, 256), (130, 64, 1433),
               (77, 64, 3703), (1025, 128, 602), (513, 256, 100), (260, 256, 256), (33, 300, 500),
               (19, 512, 256), (21, 700, 130), (9, 64, 8192), (4099, 64, 64), (50, 130, 4096),
               (4099, 130, 1433), (4200, 49, 1024), (4500, 64, 8192), (300, 70, 640),
               # more than 32768 rows: the kernels for large row counts (up to 32768 rows one
               # wavefront takes one row at a time)
               (33001, 7, 64), (33003, 64, 500), (32800, 256, 256), (32801, 64, 1433), (32769, 300, 200),
               (40000, 47, 256), (33000, 130, 3703),
               # at least 4096 rows, more than 64 columns, 512 bits or more: the FP4 path with one
               # 128 x 128 tile per wavefront (256-bit chunks of K, partial last chunk, ragged tiles)
               (4160, 256, 4096), (4200, 257, 512), (5000, 129, 8192), (4097, 128, 768), (4300, 384, 1000),
               (4100, 65, 515)]


@pytest.mark.parametrize("variant", ["auto", "valu", "mfma", "fp4"])
@pytest.mark.parametrize("m,n,k", GEMM_SHAPES)
def test_binary_gemm(B, m, n, k, variant):
    import torch
    rng = _rng(m * 31 + n * 7 + k)
    f = rng.choice(np.array([-1, 1], dtype=np.int8), size=(m, k))
    bt = rng.choice(np.array([-1, 1], dtype=np.int8), size=(n, k))
    if m > 2 and n > 2:
        f[1] = bt[1]            # identical vectors: product = +K
        f[2] = -bt[2]           # opposite vectors:  product = -K
    beta = (0.1 + rng.random(m)).astype(np.float32)
    alpha = (0.01 + rng.random(n)).astype(np.float32)
    acc = oracle.sign_matmul(f, bt)
    zeta = oracle.rescale(acc, beta.astype(np.float64), alpha.astype(np.float64))
    a_bits, b_bits, dbeta, dalpha = to_device(oracle.pack_bits(f).view(np.int64),
                                              oracle.pack_bits(bt).view(np.int64), beta, alpha)
    v = {"auto": B.GEMM_AUTO, "valu": B.GEMM_VALU, "mfma": B.GEMM_MFMA, "fp4": B.GEMM_FP4}[variant]
    dacc, dout = B.bigcn_binary_gemm(a_bits, dbeta, b_bits, dalpha, k, variant=v)
    torch.cuda.synchronize()
    assert np.array_equal(dacc.cpu().numpy(), acc)
    assert_close(dout.cpu().numpy(), zeta, "zeta")
    # each output alone
    only_acc, none = B.bigcn_binary_gemm(a_bits, None, b_bits, None, k, want_out=False, variant=v)
    assert none is None and np.array_equal(only_acc.cpu().numpy(), acc)
    none, only_out = B.bigcn_binary_gemm(a_bits, dbeta, b_bits, dalpha, k, want_acc=False, variant=v)
    assert none is None and np.array_equal(only_out.cpu().numpy(), dout.cpu().numpy())


@pytest.mark.parametrize("seed", range(4))
def test_binary_gemm_random_shapes(B, seed):
    """Seeded random shapes on either side of the tile sizes of the four evaluation paths (32-row
    and 128-row tiles, 32 / 64 / 128 columns, 64 / 256 / 512-bit chunks of K, the 32768-row switch)."""
    rng = _rng(900 + seed)
    for _ in range(12):
        m = int(rng.choice([1, 31, 32, 33, 127, 128, 129, 255, 257, 1000, 4099, int(rng.integers(1, 5000)),
                            32769 + int(rng.integers(0, 3000))]))
        n = int(rng.choice([1, 2, 31, 32, 33, 47, 63, 64, 65, 127, 128, 129, 255, 256, 257, 300, 512, 700]))
        k = int(rng.choice([1, 63, 64, 65, 127, 128, 129, 255, 256, 257, 511, 512, 513, 767, 768, 1023, 1024,
                            1025, 2047, 2048, 2049, 4096, int(rng.integers(1, 6000))]))
        if m * n * k > 3e9:
            continue
        for variant in ("auto", "valu", "mfma", "fp4"):
            test_binary_gemm(B, m, n, k, variant)


def test_binary_gemm_strided_operands_on_every_path(B):
    """Rows that start on 8-byte but not 16-byte boundaries and leading dimensions larger than the
    row (the tile path reads 16 bytes per lane straight from the operands)."""
    import torch
    m, n, k = 4200, 200, 1100
    words = (k + 63) // 64
    rng = _rng(4242)
    f = rng.choice(np.array([-1, 1], dtype=np.int8), size=(m, k))
    bt = rng.choice(np.array([-1, 1], dtype=np.int8), size=(n, k))
    acc = oracle.sign_matmul(f, bt)
    fa = np.full((m, words + 3), -1, dtype=np.int64)          # garbage beyond the row
    fb = np.full((n, words + 1), 0x5555555555555555, dtype=np.int64)
    fa[:, 1:1 + words] = oracle.pack_bits(f).view(np.int64)
    fb[:, 1:1 + words] = oracle.pack_bits(bt).view(np.int64)
    da, db = to_device(fa, fb)
    a_view, b_view = da[:, 1:1 + words], db[:, 1:1 + words]
    for v in (B.GEMM_AUTO, B.GEMM_VALU, B.GEMM_MFMA, B.GEMM_FP4):
        dacc, _ = B.bigcn_binary_gemm(a_view, None, b_view, None, k, want_out=False, variant=v)
        torch.cuda.synchronize()
        assert np.array_equal(dacc.cpu().numpy(), acc), f"variant {v}"


def test_binary_gemm_unit_scales_give_exact_integers(B):
    rng = _rng(5)
    f = rng.choice(np.array([-1, 1], dtype=np.int8), size=(64, 1433))
    bt = rng.choice(np.array([-1, 1], dtype=np.int8), size=(64, 1433))
    a_bits, b_bits = to_device(oracle.pack_bits(f).view(np.int64), oracle.pack_bits(bt).view(np.int64))
    import torch
    ones = torch.ones(64, device="cuda")
    acc, out = B.bigcn_binary_gemm(a_bits, ones, b_bits, ones, 1433)
    assert np.array_equal(out.cpu().numpy(), acc.cpu().numpy().astype(np.float32))
    assert np.array_equal(acc.cpu().numpy(), oracle.sign_matmul(f, bt))


# ------------------------------------------------------------------------------------------
# graph helpers and kernel 3: SpMM
# ------------------------------------------------------------------------------------------
def _hub_graph(seed=11):
    """Power-law graph with rows on both sides of the workgroup-per-row thresholds (1024 for the
    aggregation of the Bi-GCN path, 256 for the Bi-GAT kernels)."""
    n = 3000
    rp, ci = chung_lu_csr(n, 60000, 2.2, 1.5, seed=seed)
    deg = np.diff(rp)
    assert (deg >= 1024).sum() >= 3 and ((deg >= 256) & (deg < 1024)).sum() >= 5 and deg.min() <= 8
    return rp, ci


def test_gcn_norm(B):
    rp, ci = _hub_graph()
    a = oracle.gcn_norm(rp, ci)
    drp, dci = to_device(rp, ci)
    dinv, vals = B.bigcn_gcn_norm(drp, dci, want_vals=True)
    assert_close(dinv.cpu().numpy(), 1.0 / np.sqrt(np.diff(rp).astype(np.float64)), "dinv_sqrt")
    assert_close(vals.cpu().numpy(), a, "a_tilde")
    dinv2, none = B.bigcn_gcn_norm(drp, dci)
    assert none is None and np.array_equal(dinv2.cpu().numpy(), dinv.cpu().numpy())


@pytest.mark.parametrize("d", [1, 3, 4, 7, 8, 41, 47, 64, 100, 128, 256, 260, 301, 600])
@pytest.mark.parametrize("weighted", [True, False])
def test_spmm(B, d, weighted):
    import torch
    rp, ci = _hub_graph()
    n = rp.size - 1
    rng = _rng(d)
    # without coefficients a hub row adds ~1000 O(1) terms: keep them of one sign so that the
    # relative tolerance is not asked to resolve fp32 cancellation
    z = (rng.standard_normal((n, d)) if weighted else rng.random((n, d))).astype(np.float32)
    a = oracle.gcn_norm(rp, ci) if weighted else np.ones(ci.size)
    ref = oracle.aggregate(rp, ci, a, z.astype(np.float64))
    drp, dci, dz = to_device(rp, ci, z)
    plan = B.Plan(drp, dci)
    assert plan.nnz == ci.size
    vals = to_device(a.astype(np.float32)) if weighted else None
    out = B.bigcn_spmm(plan, drp, dci, vals, dz)
    torch.cuda.synchronize()
    # the fp32 coefficients themselves carry a relative rounding error of 2^-24
    ref32 = oracle.aggregate(rp, ci, a.astype(np.float32).astype(np.float64), z.astype(np.float64))
    assert_close(out.cpu().numpy(), ref32, "spmm")
    assert np.allclose(ref, ref32, rtol=1e-6, atol=1e-7)
    again = B.bigcn_spmm(plan, drp, dci, vals, dz)
    assert torch.equal(out, again)                       # fixed summation order
    plan.destroy()


def test_spmm_invariants(B):
    """A~ sqrt(d) = sqrt(d) and A~ I = A~ on a graph with long rows."""
    rp, ci = _hub_graph(seed=12)
    n = rp.size - 1
    drp, dci = to_device(rp, ci)
    plan = B.Plan(drp, dci)
    _, vals = B.bigcn_gcn_norm(drp, dci, want_vals=True)
    rootd = np.sqrt(np.diff(rp).astype(np.float32))[:, None]
    out = B.bigcn_spmm(plan, drp, dci, vals, to_device(np.ascontiguousarray(rootd)))
    assert_close(out.cpu().numpy(), rootd.astype(np.float64))
    eye = np.eye(n, 256, dtype=np.float32)
    out = B.bigcn_spmm(plan, drp, dci, vals, to_device(eye)).cpu().numpy()
    import scipy.sparse as sp
    dense = sp.csr_matrix((oracle.gcn_norm(rp, ci), ci, rp), shape=(n, n)).toarray()[:, :256]
    assert_close(out, dense)


def test_spmm_tiny_and_degenerate_graphs(B):
    # isolated nodes (self-loop only) and a single edge
    rp, ci = csr_from_undirected_edges(5, np.array([0]), np.array([3]))
    z = np.arange(15, dtype=np.float32).reshape(5, 3)
    drp, dci, dz = to_device(rp, ci, z)
    plan = B.Plan(drp, dci)
    out = B.bigcn_spmm(plan, drp, dci, None, dz).cpu().numpy()
    expect = z.copy()
    expect[0] += z[3]
    expect[3] += z[0]
    assert np.array_equal(out, expect)


def test_plan_validation_rejects_bad_patterns(B):
    rp, ci = csr_from_undirected_edges(4, np.array([0, 1]), np.array([1, 2]))
    drp, dci = to_device(rp, ci)
    B.Plan(drp, dci).destroy()

    def status(rp_, ci_):
        with pytest.raises(B.BigcnError) as e:
            B.Plan(*to_device(rp_, ci_))
        return e.value.status

    bad = ci.copy(); bad[0] = 9
    assert status(rp, bad) == B.BIGCN_EGRAPH                       # column out of range
    bad = ci.copy(); bad[[0, 1]] = bad[[1, 0]]
    assert status(rp, bad) == B.BIGCN_EGRAPH                       # unsorted
    # missing self-loop on node 3: rows (0:0,1) (1:0,1,2) (2:1,2) (3:) -> use an asymmetric entry
    rp2 = np.array([0, 2, 5, 7, 8], dtype=np.int64)
    ci2 = np.array([0, 1, 0, 1, 2, 1, 2, 0], dtype=np.int32)       # row 3 holds (3,0) only
    assert status(rp2, ci2) == B.BIGCN_EGRAPH
    bad_rp = rp.copy(); bad_rp[2] = bad_rp[1] - 1
    assert status(bad_rp, ci) == B.BIGCN_EINVAL
    # validation can be switched off
    B.Plan(*to_device(rp2, ci2), validate=False).destroy()


def test_multiply_rate_probes_run_and_count_their_work(B):
    """The two measurement launches behind the bit-GEMM's ceilings: both complete, report the
    multiply-accumulates of their grid, and leave finite sums (every product is +-1)."""
    import torch
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    sink = torch.full((cus * 256,), float("nan"), dtype=torch.float32, device="cuda")
    for probe in (B.bigcn_probe_fp4_multiply_rate, B.bigcn_probe_fp4_expand_multiply_rate):
        sink.fill_(float("nan"))
        macs = probe(3, sink)
        torch.cuda.synchronize()
        assert macs == cus * 4 * 3 * 16 * 32 * 32 * 64
        got = sink.cpu().numpy()
        # a lane's 256 accumulators hold sums of 3 * 64 products of +-1 each
        assert np.isfinite(got).all() and (np.abs(got) <= 256 * 3 * 64).all() and np.array_equal(got, np.rint(got))
    with pytest.raises(Exception):
        B.bigcn_probe_fp4_expand_multiply_rate(3, sink[:16])


def test_stream_read_probe_reads_what_it_says(B):
    """The read-only measurement launch: completes on a buffer whose length is not a multiple of
    its pieces, reports the bytes it read, and refuses a sink that is too small."""
    import torch
    src = torch.arange(0, 3_000_003, dtype=torch.int32, device="cuda")
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    sink = torch.full((cus * 32 * 256,), float("nan"), dtype=torch.float32, device="cuda")
    assert B.bigcn_probe_stream_read(src, sink) == 3_000_003 * 4 // 16 * 16
    torch.cuda.synchronize()
    assert bool(torch.isfinite(sink).all())
    with pytest.raises(Exception):
        B.bigcn_probe_stream_read(src, sink[:1024])
