"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, and rejects bad arguments before touching the device."""
import numpy as np
import ctypes
import os
import re

import pytest

from paper_2210_13149_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "bigcn.h")

pytestmark = pytest.mark.skipif(not os.path.exists(binding.LIBRARY),
                                reason="libbigcn.so not built (run __graft_entry__.build())")


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(bigcn_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_four_north_star_entry_points():
    names = _declared_functions()
    for required in ("bigcn_pack", "bigcn_binary_gemm", "bigcn_spmm", "bigcn_forward"):
        assert required in names


def test_library_exports_every_declared_symbol():
    L = binding.lib()
    for name in _declared_functions():
        assert hasattr(L, name), f"{name} declared in bigcn.h but not exported"
    assert set(binding.EXPORTS) == set(_declared_functions())


def test_version_and_status_strings():
    assert binding.version() >= 100
    seen = set()
    for code in range(0, -7, -1):
        s = binding.status_string(code)
        assert s and s != "unknown status" and s not in seen
        seen.add(s)
    assert binding.status_string(-99) == "unknown status"
    assert binding.status_string(0) == "ok"


FAKE = 0x1000  # a non-NULL address that is never dereferenced: argument checks come first


def test_pack_rejects_bad_arguments():
    L = binding.lib()
    assert L.bigcn_pack(None, 4, 8, 8, 1, None, None, FAKE, 1, FAKE, None) == binding.BIGCN_ENULL
    assert L.bigcn_pack(FAKE, 4, 8, 8, 1, None, None, None, 1, FAKE, None) == binding.BIGCN_ENULL
    assert L.bigcn_pack(FAKE, 4, 8, 8, 1, None, None, FAKE, 1, None, None) == binding.BIGCN_ENULL
    assert L.bigcn_pack(FAKE, -1, 8, 8, 1, None, None, FAKE, 1, FAKE, None) == binding.BIGCN_EINVAL
    assert L.bigcn_pack(FAKE, 4, 0, 8, 1, None, None, FAKE, 1, FAKE, None) == binding.BIGCN_EINVAL
    assert L.bigcn_pack(FAKE, 4, 8, 0, 1, None, None, FAKE, 1, FAKE, None) == binding.BIGCN_EINVAL
    assert L.bigcn_pack(FAKE, 4, 65, 65, 1, None, None, FAKE, 1, FAKE, None) == binding.BIGCN_EINVAL
    assert L.bigcn_pack(FAKE, 0, 8, 8, 1, None, None, FAKE, 1, FAKE, None) == binding.BIGCN_OK


def test_binary_gemm_rejects_bad_arguments():
    L = binding.lib()
    ok = dict(a=FAKE, sa=FAKE, m=4, lda=2, b=FAKE, sb=FAKE, n=3, ldb=2, k=100, acc=FAKE, ldacc=3,
              out=FAKE, ldout=3)

    def call(**kw):
        p = dict(ok, **kw)
        return L.bigcn_binary_gemm(p["a"], p["sa"], p["m"], p["lda"], p["b"], p["sb"], p["n"], p["ldb"],
                                   p["k"], p["acc"], p["ldacc"], p["out"], p["ldout"], None)

    assert call(a=None) == binding.BIGCN_ENULL
    assert call(b=None) == binding.BIGCN_ENULL
    assert call(acc=None, out=None) == binding.BIGCN_ENULL
    assert call(sa=None) == binding.BIGCN_ENULL
    assert call(sb=None) == binding.BIGCN_ENULL
    assert call(m=-1) == binding.BIGCN_EINVAL
    assert call(k=0) == binding.BIGCN_EINVAL
    assert call(lda=1) == binding.BIGCN_EINVAL
    assert call(ldb=1) == binding.BIGCN_EINVAL
    assert call(ldacc=2) == binding.BIGCN_EINVAL
    assert call(ldout=2) == binding.BIGCN_EINVAL
    assert call(k=binding.MAX_K_BITS + 1, lda=200, ldb=200) == binding.BIGCN_ESHAPE
    assert call(m=0) == binding.BIGCN_OK
    assert call(n=0, ldacc=0, ldout=0) == binding.BIGCN_OK
    p = ok
    for variant, expect in ((4, binding.BIGCN_EINVAL), (-1, binding.BIGCN_EINVAL)):
        assert L.bigcn_binary_gemm_variant(p["a"], p["sa"], p["m"], p["lda"], p["b"], p["sb"], p["n"],
                                           p["ldb"], p["k"], p["acc"], p["ldacc"], p["out"], p["ldout"],
                                           variant, None) == expect
    assert L.bigcn_binary_gemm_variant(None, p["sa"], p["m"], p["lda"], p["b"], p["sb"], p["n"], p["ldb"],
                                       p["k"], p["acc"], p["ldacc"], p["out"], p["ldout"],
                                       binding.GEMM_MFMA, None) == binding.BIGCN_ENULL


def test_graph_entry_points_reject_bad_arguments():
    L = binding.lib()
    assert L.bigcn_gcn_norm(None, FAKE, 4, FAKE, None, None) == binding.BIGCN_ENULL
    assert L.bigcn_gcn_norm(FAKE, FAKE, 4, None, None, None) == binding.BIGCN_ENULL
    assert L.bigcn_gcn_norm(FAKE, None, 4, FAKE, FAKE, None) == binding.BIGCN_ENULL
    assert L.bigcn_gcn_norm(FAKE, FAKE, -4, FAKE, None, None) == binding.BIGCN_EINVAL
    assert L.bigcn_gcn_norm(FAKE, FAKE, 0, FAKE, None, None) == binding.BIGCN_OK
    handle = ctypes.c_void_p()
    assert L.bigcn_plan_create(None, FAKE, 4, 1, ctypes.byref(handle), None) == binding.BIGCN_ENULL
    assert L.bigcn_plan_create(FAKE, FAKE, 4, 1, None, None) == binding.BIGCN_ENULL
    assert L.bigcn_plan_create(FAKE, FAKE, -1, 1, ctypes.byref(handle), None) == binding.BIGCN_EINVAL
    assert L.bigcn_plan_create(FAKE, FAKE, 1 << 31, 1, ctypes.byref(handle), None) == binding.BIGCN_EINVAL
    assert handle.value is None
    L.bigcn_plan_destroy(None)
    assert L.bigcn_plan_rows(None) == -1 and L.bigcn_plan_nnz(None) == -1
    assert L.bigcn_spmm(None, FAKE, FAKE, None, 4, FAKE, 8, 8, FAKE, 8, None) == binding.BIGCN_ENULL


def _layers(dims, ld=None):
    arr = (binding.LayerDesc * (len(dims) - 1))()
    for l in range(len(dims) - 1):
        arr[l] = binding.LayerDesc(FAKE, FAKE, dims[l], dims[l + 1],
                                   (dims[l] + 63) // 64 if ld is None else ld, None, None)
    return arr


def test_forward_workspace_size_and_argument_checks():
    L = binding.lib()
    n = 1000
    layers = _layers((100, 256, 256, 47))
    need = L.bigcn_forward_workspace_bytes(n, layers, 3)
    # packed signs (4 words), two scale vectors, 256 one-byte products per node (K <= 256) and the
    # alternate one-byte array of the K = 256 layer (rows that do not fit the 7-bit form)
    assert need >= n * (4 * 8 + 2 * 4 + 2 * 256)
    assert need <= n * (4 * 8 + 2 * 4 + 2 * 256) + 5 * 256
    small = L.bigcn_forward_workspace_bytes(n, _layers((100, 256, 47)), 2)
    assert small <= n * (4 * 8 + 2 * 4 + 256) + 4 * 256   # K = 100 -> 256 provably fits: no alternate array
    mid = L.bigcn_forward_workspace_bytes(n, _layers((602, 128, 41)), 2)
    assert mid >= n * (10 * 8 + 8 + 128 + 128 * 2)    # 256 < K <= 1024: 7-bit products, fp16 alternates
    wide = L.bigcn_forward_workspace_bytes(n, _layers((3703, 64, 6)), 2)
    assert wide >= n * (58 * 8 + 8 + 64 * 4)          # K > 2048: products kept in fp32
    assert L.bigcn_forward_workspace_bytes(n, None, 3) == 0
    assert L.bigcn_forward_workspace_bytes(n, _layers((100, 64, 32)), 0) == 0
    bad_chain = _layers((100, 64, 7))
    bad_chain[1].d_in = 65
    assert L.bigcn_forward_workspace_bytes(n, bad_chain, 2) == 0
    assert L.bigcn_forward_workspace_bytes(n, _layers((100, 513, 7)), 2) == 0
    assert L.bigcn_forward_workspace_bytes(n, _layers((100, 64, 7), ld=1), 2) == 0

    def fwd(plan=FAKE, rp=FAKE, ci=FAKE, dinv=FAKE, x=FAKE, lay=layers, nl=3, logits=FAKE):
        return L.bigcn_forward(plan, rp, ci, dinv, n, x, 100, lay, nl, logits, 47, FAKE, need, None)

    assert fwd(plan=None) == binding.BIGCN_ENULL
    assert fwd(x=None) == binding.BIGCN_ENULL
    assert fwd(logits=None) == binding.BIGCN_ENULL
    assert fwd(lay=None) == binding.BIGCN_ENULL
    assert fwd(nl=0) == binding.BIGCN_EINVAL
    assert fwd(lay=_layers((100, 513, 47)), nl=2) == binding.BIGCN_ESHAPE
    assert fwd(lay=_layers((9000, 64, 47), ld=200), nl=2) == binding.BIGCN_ESHAPE


def test_product_row_formats_by_layer_shape():
    """The per-node product row of the fused forward, by (input bits, columns): one byte per
    product up to 1024 input bits (rows of 2..64 lanes of 8 values, the source scale inside the
    row: in its tail, in the last bytes of four lanes for 40..60 columns, or in the spare top
    bits), fp16 products up to 2048 bits and fp32 beyond (scale gathered separately).  A host
    function: no GPU needed."""
    B = binding
    expect = {
        (100, 256): (256, True), (256, 256): (256, True), (100, 512): (512, True), (1024, 512): (512, True),
        # the class counts of the large workloads: 64-byte rows up to 256 input bits
        (128, 41): (64, True), (256, 47): (64, True), (256, 39): (64, True), (256, 40): (64, True),
        (256, 60): (64, True), (256, 61): (128, True), (256, 64): (128, True),
        # beyond 256 bits: 64-byte rows up to 60 columns (8-bit values, the scale in the last bytes of
        # four lanes), else at least 16 lanes, for the bits of the scale
        (257, 47): (64, True), (512, 47): (64, True), (1024, 60): (64, True), (1024, 7): (64, True),
        (512, 61): (128, True), (602, 128): (128, True),
        (64, 7): (16, True), (100, 3): (16, True), (100, 79): (128, True), (100, 80): (128, True),
        (1025, 64): (128, False), (2048, 64): (128, False), (2049, 64): (256, False), (3703, 64): (256, False),
    }
    for (d_in, d_out), want in expect.items():
        assert B.bigcn_forward_row_bytes(d_in, d_out) == want, (d_in, d_out)


def test_binding_refuses_host_tensors():
    import torch
    with pytest.raises(TypeError):
        binding.bigcn_pack(torch.zeros(2, 3))


def test_static_forward_rejects_oversized_problems_on_the_host():
    """bigcn_forward_static checks the workspace the problem needs against its fixed array before
    it touches the device: ESHAPE for a graph that does not fit, ENULL for missing layers."""
    L = binding.lib()
    desc = (binding.LayerDesc * 1)()
    desc[0].w_bits, desc[0].alpha, desc[0].d_in, desc[0].d_out, desc[0].ld_words = FAKE, FAKE, 100, 256, 2
    n = 3_000_000
    assert L.bigcn_forward_workspace_bytes(n, desc, 1) > binding.STATIC_WORKSPACE_BYTES
    assert L.bigcn_forward_static(FAKE, FAKE, FAKE, FAKE, n, FAKE, 100, desc, 1, FAKE, 256, None) == binding.BIGCN_ESHAPE
    assert L.bigcn_forward_static(FAKE, FAKE, FAKE, FAKE, n, FAKE, 100, None, 1, FAKE, 256, None) == binding.BIGCN_ENULL
    assert L.bigcn_forward_static(FAKE, FAKE, FAKE, FAKE, -1, FAKE, 100, desc, 1, FAKE, 256, None) == binding.BIGCN_EINVAL
    text = open(HEADER).read()
    assert f"#define BIGCN_STATIC_WORKSPACE_BYTES ({binding.STATIC_WORKSPACE_BYTES >> 20}u << 20)" in text


def test_binary_gemm_column_limit_matches_the_header():
    """n up to BIGCN_MAX_GEMM_N is a shape error beyond, and the limit is what one launch can cover
    (65535 column blocks of 64)."""
    L = binding.lib()
    text = open(HEADER).read()
    limit = int(re.search(r"#define BIGCN_MAX_GEMM_N (\d+)", text).group(1))
    assert limit == 65535 * 64
    assert L.bigcn_binary_gemm(FAKE, FAKE, 4, 2, FAKE, FAKE, limit + 1, 2, 100, FAKE, limit + 1, None, 0, None) == binding.BIGCN_ESHAPE


def test_every_product_row_layout_is_consistent():
    """All layer shapes up to 1100 input bits (and a few beyond) x every column count the fused
    forward takes: the layout the library reports must have room for every column, keep the bytes
    it uses for the scale clear of live columns, and use a value width that holds the product
    (or an escape).  Pure host logic."""
    B = binding
    d_ins = list(range(1, 300)) + [300, 511, 512, 513, 602, 1000, 1023, 1024, 1025, 1433, 2048, 2049, 3703, 8191, 8192]
    for d_in in d_ins:
        for d_out in list(range(1, 130)) + [191, 192, 193, 255, 256, 257, 300, 500, 511, 512]:
            lay = B.bigcn_forward_row_layout(d_in, d_out)
            G, V, kind, k_eff = lay["groups"], lay["vec"], lay["kind"], lay["k_eff"]
            place, escape, alt = lay["scale_place"], lay["escape"], lay["alt_kind"]
            what = (d_in, d_out, lay)
            assert G in (2, 4, 8, 16, 32, 64) and V in (4, 8), what
            assert G * V >= d_out, what
            assert k_eff == d_in - lay["fold_last"] and lay["fold_last"] in (0, 1), what
            col = (np.arange(G)[:, None] + G * np.arange(V)[None, :]).reshape(-1)     # column of every position
            if kind == 0:
                assert V == 8, what
                if place == 2:
                    assert G >= 16 and (k_eff <= 127 or escape), what                 # 7 bits: |q| <= 63, or an escape
                elif not escape:
                    assert k_eff <= 255, what                                         # q = floor(K'/2) - popcount fits int8
                if place == 1:
                    assert (col[-4:] >= d_out).all(), what                            # the tail holds the scale
                if place == 3:
                    assert G == 8 and (col[[39, 47, 55, 63]] >= d_out).all(), what    # last byte of lanes 4..7
                if escape:
                    assert place in (2, 3) and alt in (0, 1), what
                    assert alt == 1 or k_eff <= 255, what                             # one-byte alternates hold q
                    assert alt == 0 or k_eff <= 4096, what                            # fp16 holds integers up to 2048
            elif kind == 1:
                assert d_in <= 2048 and place == 0 and not escape, what
            else:
                assert kind == 2 and place == 0 and not escape, what
            bytes_, embedded = B.bigcn_forward_row_bytes(d_in, d_out)
            assert bytes_ == G * V * {0: 1, 1: 2, 2: 4}[kind] and embedded == (place != 0), what
