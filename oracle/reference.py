"""numpy front-end of the plain CPU oracle (``bigcn_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke()`` and by the
``cpu_baseline`` leg of ``bench.py``; never by the product package.  It shares no code with the
HIP library.  Each function states the passage of the paper it follows.

Pinned by ``tests/test_oracle_pins.py`` and ``tests/test_oracle_sage_pins.py`` (brute force,
closed forms, hand-built graphs, library routines, the cost figures the paper prints).  Not pinned by anything: accuracy on the real
datasets (parity unpinned: neither datasets nor trained weights are available).
"""

from __future__ import annotations

import ctypes
import os
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

from . import build as _build

_LIB = None

_i64p = ctypes.POINTER(ctypes.c_int64)
_i32p = ctypes.POINTER(ctypes.c_int32)
_i8p = ctypes.POINTER(ctypes.c_int8)
_f32p = ctypes.POINTER(ctypes.c_float)
_f64p = ctypes.POINTER(ctypes.c_double)


def _lib():
    global _LIB
    if _LIB is None:
        path = _build.LIBRARY
        if not os.path.exists(path):
            path = _build.build()
        lib = ctypes.CDLL(path)
        lib.oracle_gcn_norm.argtypes = [ctypes.c_int64, _i64p, _i32p, _f64p]
        lib.oracle_binarize_rows_f32.argtypes = [_f32p, ctypes.c_int64, ctypes.c_int64,
                                                 ctypes.c_int64, ctypes.c_int64, _f32p, _f32p,
                                                 _i8p, _f64p]
        lib.oracle_binarize_rows_f64.argtypes = [_f64p, ctypes.c_int64, ctypes.c_int64, _f32p,
                                                 _f32p, _i8p, _f64p]
        lib.oracle_sign_matmul.argtypes = [_i8p, _i8p, ctypes.c_int64, ctypes.c_int64,
                                           ctypes.c_int64, _i32p]
        lib.oracle_rescale.argtypes = [_i32p, _f64p, _f64p, ctypes.c_int64, ctypes.c_int64, _f64p]
        lib.oracle_aggregate.argtypes = [ctypes.c_int64, _i64p, _i32p, _f64p, _f64p,
                                         ctypes.c_int64, _f64p]
        lib.oracle_aggregate_transposed.argtypes = [ctypes.c_int64, _i64p, _i32p, _f64p, _f64p,
                                                    ctypes.c_int64, _f64p]
        lib.oracle_aggregate_transposed.restype = None
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_set_num_threads.argtypes = [ctypes.c_int]
        for name in ("oracle_gcn_norm", "oracle_binarize_rows_f32", "oracle_binarize_rows_f64",
                     "oracle_sign_matmul", "oracle_rescale", "oracle_aggregate",
                     "oracle_set_num_threads"):
            getattr(lib, name).restype = None
        _LIB = lib
    return _LIB


def _ptr(a: Optional[np.ndarray], typ):
    if a is None:
        return ctypes.cast(None, typ)
    return a.ctypes.data_as(typ)


def num_threads() -> int:
    return int(_lib().oracle_num_threads())


def set_num_threads(t: int) -> None:
    _lib().oracle_set_num_threads(int(t))


def _check_csr(row_ptr: np.ndarray, col_idx: np.ndarray) -> Tuple[np.ndarray, np.ndarray, int]:
    row_ptr = np.ascontiguousarray(row_ptr, dtype=np.int64)
    col_idx = np.ascontiguousarray(col_idx, dtype=np.int32)
    n = row_ptr.size - 1
    if n < 0 or row_ptr[0] != 0 or row_ptr[-1] != col_idx.size or np.any(np.diff(row_ptr) < 0):
        raise ValueError("malformed CSR row pointer")
    if col_idx.size and (col_idx.min() < 0 or col_idx.max() >= n):
        raise ValueError("CSR column out of range")
    return row_ptr, col_idx, n


def gcn_norm(row_ptr: np.ndarray, col_idx: np.ndarray) -> np.ndarray:
    """Coefficients of A~ = D^-1/2 (A+I) D^-1/2 (Sec. 3.1 Notations, Eq. (1)) for the stored
    entries of the CSR pattern of A+I: ``a_tilde[p] = 1/sqrt(deg_i * deg_k)``, fp64."""
    row_ptr, col_idx, n = _check_csr(row_ptr, col_idx)
    out = np.empty(col_idx.size, dtype=np.float64)
    _lib().oracle_gcn_norm(n, _ptr(row_ptr, _i64p), _ptr(col_idx, _i32p), _ptr(out, _f64p))
    return out


def _col_params(shift, mul, cols):
    s = None if shift is None else np.ascontiguousarray(shift, dtype=np.float32)
    m = None if mul is None else np.ascontiguousarray(mul, dtype=np.float32)
    for v in (s, m):
        if v is not None and v.shape != (cols,):
            raise ValueError("per-column parameter has the wrong length")
    return s, m


def binarize_rows(x: np.ndarray, shift=None, mul=None) -> Tuple[np.ndarray, np.ndarray]:
    """Row-wise vector binarisation (Sec. 4.1; Sec. 4.2.2 for node features): returns
    ``(sign int8 (rows, cols) in {-1,+1}, scale fp64 (rows,))`` with sign = +1 iff
    ``x >= shift[c]`` and scale = mean_c |(x - shift[c]) * mul[c]|.  ``x`` may be any strided 2-D
    fp32 view (e.g. ``W.T``) or a contiguous fp64 matrix."""
    if x.ndim != 2:
        raise ValueError("expected a matrix")
    rows, cols = x.shape
    s, m = _col_params(shift, mul, cols)
    sign = np.empty((rows, cols), dtype=np.int8)
    scale = np.empty(rows, dtype=np.float64)
    if x.dtype == np.float32:
        if x.strides[0] % 4 or x.strides[1] % 4:
            x = np.ascontiguousarray(x)
        _lib().oracle_binarize_rows_f32(_ptr(x, _f32p), rows, cols, x.strides[0] // 4,
                                        x.strides[1] // 4, _ptr(s, _f32p), _ptr(m, _f32p),
                                        _ptr(sign, _i8p), _ptr(scale, _f64p))
    elif x.dtype == np.float64:
        x = np.ascontiguousarray(x)
        _lib().oracle_binarize_rows_f64(_ptr(x, _f64p), rows, cols, _ptr(s, _f32p),
                                        _ptr(m, _f32p), _ptr(sign, _i8p), _ptr(scale, _f64p))
    else:
        raise TypeError("binarize_rows takes fp32 or fp64 input")
    return sign, scale


def binarize_weight(w: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Sec. 4.2.1: each column of W (d_in, d_out) is one bucket.  Returns
    ``(bt int8 (d_out, d_in), alpha fp64 (d_out,))``: row j of ``bt`` is B_j = sign(W[:, j]) and
    alpha_j = ||W[:, j]||_1 / d_in."""
    w = np.asarray(w, dtype=np.float32)
    return binarize_rows(w.T)


def sign_matmul(f: np.ndarray, bt: np.ndarray) -> np.ndarray:
    """Sec. 4.2.3: literal inner products of +-1 vectors, ``acc[i, j] = sum_t f[i,t]*bt[j,t]``."""
    f = np.ascontiguousarray(f, dtype=np.int8)
    bt = np.ascontiguousarray(bt, dtype=np.int8)
    if f.ndim != 2 or bt.ndim != 2 or f.shape[1] != bt.shape[1]:
        raise ValueError("shape mismatch")
    m, k = f.shape
    n = bt.shape[0]
    acc = np.empty((m, n), dtype=np.int32)
    _lib().oracle_sign_matmul(_ptr(f, _i8p), _ptr(bt, _i8p), m, k, n, _ptr(acc, _i32p))
    return acc


def rescale(acc: np.ndarray, beta: np.ndarray, alpha: np.ndarray) -> np.ndarray:
    """Sec. 4.2.3: ``zeta[i, j] = beta[i] * alpha[j] * acc[i, j]`` in fp64."""
    acc = np.ascontiguousarray(acc, dtype=np.int32)
    beta = np.ascontiguousarray(beta, dtype=np.float64)
    alpha = np.ascontiguousarray(alpha, dtype=np.float64)
    m, n = acc.shape
    if beta.shape != (m,) or alpha.shape != (n,):
        raise ValueError("shape mismatch")
    zeta = np.empty((m, n), dtype=np.float64)
    _lib().oracle_rescale(_ptr(acc, _i32p), _ptr(beta, _f64p), _ptr(alpha, _f64p), m, n,
                          _ptr(zeta, _f64p))
    return zeta


def aggregate(row_ptr, col_idx, a_tilde: np.ndarray, z: np.ndarray) -> np.ndarray:
    """Sec. 4.2.3, H_b = A~ zeta: explicit sum over each node's stored neighbours, fp64."""
    row_ptr, col_idx, n = _check_csr(row_ptr, col_idx)
    a_tilde = np.ascontiguousarray(a_tilde, dtype=np.float64)
    z = np.ascontiguousarray(z, dtype=np.float64)
    if z.ndim != 2 or z.shape[0] != n or a_tilde.shape != (col_idx.size,):
        raise ValueError("shape mismatch")
    out = np.empty_like(z)
    _lib().oracle_aggregate(n, _ptr(row_ptr, _i64p), _ptr(col_idx, _i32p), _ptr(a_tilde, _f64p),
                            _ptr(z, _f64p), z.shape[1], _ptr(out, _f64p))
    return out


def column_standardisation(h: np.ndarray, eps: float = 1e-5) -> Tuple[np.ndarray, np.ndarray]:
    """Sec. 4.4 step 1 ("zero mean and variance one" over the nodes), frozen into a per-column
    affine map: ``shift = mean_i h[i, c]``, ``mul = 1/sqrt(var_c + eps)`` (biased variance), both
    rounded to fp32 because they are handed to the forward pass as fp32 inputs."""
    h64 = np.asarray(h, dtype=np.float64)
    mean = h64.mean(axis=0)
    var = h64.var(axis=0)
    return mean.astype(np.float32), (1.0 / np.sqrt(var + eps)).astype(np.float32)


def pack_bits(sign: np.ndarray) -> np.ndarray:
    """Packed layout of a +-1 matrix: uint64 words, LSB first; bit l of word w of a row is 1 iff
    element 64*w + l is +1; bits past the last column are 0."""
    sign = np.asarray(sign)
    rows, cols = sign.shape
    words = (cols + 63) // 64
    bits = np.zeros((rows, words * 64), dtype=np.uint8)
    bits[:, :cols] = sign > 0
    packed = np.packbits(bits, axis=1, bitorder="little")
    return np.ascontiguousarray(packed).view("<u8").reshape(rows, words)


def unpack_bits(words: np.ndarray, cols: int) -> np.ndarray:
    """Inverse of :func:`pack_bits` (returns int8 +-1, shape (rows, cols))."""
    words = np.ascontiguousarray(words, dtype="<u8")
    rows = words.shape[0]
    bits = np.unpackbits(words.view(np.uint8).reshape(rows, -1), axis=1, bitorder="little")
    return (bits[:, :cols].astype(np.int8) * 2 - 1).astype(np.int8)


def layer(row_ptr, col_idx, a_tilde, h: np.ndarray, w: np.ndarray, shift=None, mul=None
          ) -> Dict[str, np.ndarray]:
    """One binarised graph-convolution layer (Sec. 4.2):  binarise the rows of ``h`` and the
    columns of ``w``, take the +-1 inner products, rescale by beta_i alpha_j, aggregate with A~.
    Returns every intermediate: sign, beta, bt, alpha, acc, zeta, out."""
    sign, beta = binarize_rows(h, shift, mul)
    bt, alpha = binarize_weight(w)
    acc = sign_matmul(sign, bt)
    zeta = rescale(acc, beta, alpha)
    out = aggregate(row_ptr, col_idx, a_tilde, zeta)
    return {"sign": sign, "beta": beta, "bt": bt, "alpha": alpha, "acc": acc, "zeta": zeta,
            "out": out}


def forward(row_ptr, col_idx, x: np.ndarray, weights: Sequence[np.ndarray],
            bn: Optional[Sequence[Optional[Tuple[np.ndarray, np.ndarray]]]] = None,
            calibrate: Optional[Sequence[bool]] = None, keep_trace: bool = False):
    """L-layer Bi-GCN forward (Eq. (1) with H^(0) = X; Sec. 4.2.3 per layer); returns the
    fp64 logits H^(L) and a list with one record per layer.

    ``bn[l]`` is the frozen standardisation ``(shift, mul)`` applied to the input of layer l, or
    None.  ``calibrate[l] = True`` computes it here from the oracle's own input of that layer
    (:func:`column_standardisation`); the parameters used are returned in the records so that
    the same fp32 values can be given to any other implementation.
    """
    n_layers = len(weights)
    bn = list(bn) if bn is not None else [None] * n_layers
    calibrate = list(calibrate) if calibrate is not None else [False] * n_layers
    a_tilde = gcn_norm(row_ptr, col_idx)
    h = np.asarray(x, dtype=np.float32)
    records: List[Dict[str, np.ndarray]] = []
    for l in range(n_layers):
        params = bn[l]
        if calibrate[l]:
            params = column_standardisation(h)
        shift, mul = params if params is not None else (None, None)
        rec = layer(row_ptr, col_idx, a_tilde, h, weights[l], shift, mul)
        rec["shift"], rec["mul"] = shift, mul
        if keep_trace:
            rec["input"] = h
        h = rec["out"]
        if not keep_trace:
            rec = {k: rec[k] for k in ("shift", "mul", "beta", "alpha")}
        records.append(rec)
    return h, records


def predict(h: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Prediction from the last layer's output (Sec. 3.2: Y~ = softmax(H^(L)), the class of a
    node being the largest entry of its row): returns ``(labels int32 (n,), probs fp64 (n, C))``.
    The label is decided on the values as given (fp32 logits stay fp32 for the comparison); among
    equal maxima the lowest class index wins.  The softmax is evaluated as
    exp(h - max_row) / sum, which equals the definition for every finite input."""
    h = np.asarray(h)
    if h.ndim != 2 or h.shape[1] == 0:
        raise ValueError("expected a matrix with at least one column")
    labels = np.argmax(h, axis=1).astype(np.int32)
    h64 = h.astype(np.float64)
    e = np.exp(h64 - h64.max(axis=1, keepdims=True))
    return labels, e / e.sum(axis=1, keepdims=True)


def binned_entropy(h: np.ndarray, bins: int) -> Tuple[np.ndarray, float, np.ndarray]:
    """Entropy estimate of a hidden layer by binning (Sec. 6.2): each neuron (column of ``h``,
    one row per input sample) is discretised into ``bins`` intervals, its empirical distribution
    ``p_m = count_m / N`` gives ``H^(h_i) = - sum_m p_m log2 p_m``, and the layer's estimate is the
    sum over its neurons (the independence estimate of that section).  Returns
    ``(per-neuron entropies fp64, their sum, counts int64 (neurons, bins))``.

    The intervals are equal-width over each neuron's own [min, max]; the bin of a value is decided
    in fp32, the precision of the activations: ``m = min(bins - 1, floor((x - lo) * (bins / (hi - lo))))``
    with every operation rounded to fp32; a constant neuron falls into bin 0.  Entropies are in
    bits."""
    h = np.ascontiguousarray(h, dtype=np.float32)
    if h.ndim != 2 or h.shape[0] == 0 or bins < 1:
        raise ValueError("expected a non-empty matrix and at least one bin")
    n, d = h.shape
    lo = h.min(axis=0)
    hi = h.max(axis=0)
    width = (hi - lo).astype(np.float32)
    with np.errstate(divide="ignore"):
        scale = np.where(width > 0, np.float32(bins) / width, np.float32(0)).astype(np.float32)
    idx = np.floor(((h - lo[None, :]).astype(np.float32) * scale[None, :]).astype(np.float32))
    idx = np.minimum(idx, bins - 1).astype(np.int64)
    counts = np.zeros((d, bins), dtype=np.int64)
    for c in range(d):
        counts[c] = np.bincount(idx[:, c], minlength=bins)
    p = counts.astype(np.float64) / n
    with np.errstate(divide="ignore", invalid="ignore"):
        terms = np.where(p > 0, -p * np.log2(p), 0.0)
    per = terms.sum(axis=1)
    return per, float(per.sum()), counts


# ---- back propagation through one binarised layer (Sec. 4.3, Algorithm 1) -----------------------

def aggregate_transposed(row_ptr, col_idx, a_tilde: np.ndarray, g: np.ndarray) -> np.ndarray:
    """Algorithm 1, first line: ``A~^T g`` as the literal transpose of :func:`aggregate` (entry p
    of row i sends ``a_tilde[p] * g[i]`` to row ``col_idx[p]``), fp64."""
    row_ptr, col_idx, n = _check_csr(row_ptr, col_idx)
    a_tilde = np.ascontiguousarray(a_tilde, dtype=np.float64)
    g = np.ascontiguousarray(g, dtype=np.float64)
    if g.ndim != 2 or g.shape[0] != n or a_tilde.shape != (col_idx.size,):
        raise ValueError("shape mismatch")
    out = np.empty_like(g)
    _lib().oracle_aggregate_transposed(n, _ptr(row_ptr, _i64p), _ptr(col_idx, _i32p),
                                       _ptr(a_tilde, _f64p), _ptr(g, _f64p), g.shape[1],
                                       _ptr(out, _f64p))
    return out


def weight_gradient(w: np.ndarray, g_wt: np.ndarray) -> np.ndarray:
    """Sec. 4.3, the gradient of the full-precision weights from the gradient of the binarised
    ones (W~_:,j = alpha_j B_:,j, alpha_j = ||W_:,j||_1 / d_in, B = sign(W)):
    ``dL/dW_ij = (1/d_in) B_ij sum_k g_wt[k, j] B_kj  +  alpha_j g_wt[i, j] 1[|W_ij| < 1]``
    (first term: alpha_j depends on every entry of its column; second term: the straight-through
    estimate d sign(r)/dr = 1[|r| < 1])."""
    w = np.asarray(w, dtype=np.float32)
    g_wt = np.asarray(g_wt, dtype=np.float64)
    if w.shape != g_wt.shape:
        raise ValueError("shape mismatch")
    bt, alpha = binarize_weight(w)
    b = bt.T.astype(np.float64)                      # (d_in, d_out)
    d_in = w.shape[0]
    column = (g_wt * b).sum(axis=0)                  # sum_k g_wt[k, j] B_kj
    ste = (np.abs(w.astype(np.float64)) < 1.0).astype(np.float64)
    return b * column[None, :] / d_in + alpha[None, :] * g_wt * ste


def layer_backward(row_ptr, col_idx, a_tilde, g_out: np.ndarray, sign: np.ndarray, beta: np.ndarray,
                   w: np.ndarray, mul=None) -> Dict[str, np.ndarray]:
    """Back propagation through one binarised graph-convolution layer (Sec. 4.3, Algorithm 1),
    fp64.  ``g_out`` = dL/dH^(l+1); ``sign``, ``beta`` are the layer's binarised input as the
    forward produced them (H~ = beta_i F_i); ``w`` the full-precision weights.

      g_zeta = A~^T g_out;   g_wt = H~^T g_zeta;   g_ht = g_zeta W~^T      (Algorithm 1)
      g_h    = g_ht * 1[|g_ht| < 1]                                       (the clipped
               straight-through estimate of Sec. 4.3, with the indicator on the gradient as
               the paper prints it)
      g_w    = weight_gradient(w, g_wt)

    With ``mul`` (the layer input was standardised by a frozen per-column affine map) ``g_in`` is
    the gradient with respect to the values before that map, ``g_h * mul``; else ``g_in = g_h``.
    Returns every intermediate."""
    sign = np.asarray(sign, dtype=np.float64)
    beta = np.asarray(beta, dtype=np.float64)
    bt, alpha = binarize_weight(w)
    h_tilde = beta[:, None] * sign                                   # (n, d_in)
    w_tilde = alpha[None, :] * bt.T.astype(np.float64)               # (d_in, d_out)
    g_zeta = aggregate_transposed(row_ptr, col_idx, a_tilde, g_out)
    g_wt = h_tilde.T @ g_zeta
    g_ht = g_zeta @ w_tilde.T
    g_h = g_ht * (np.abs(g_ht) < 1.0)
    g_in = g_h if mul is None else g_h * np.asarray(mul, dtype=np.float64)[None, :]
    return {"g_zeta": g_zeta, "g_wt": g_wt, "g_ht": g_ht, "g_h": g_h, "g_in": g_in,
            "g_w": weight_gradient(w, g_wt), "h_tilde": h_tilde, "w_tilde": w_tilde}


# ---- Bi-GraphSAGE, mean aggregator (Sec. 4.4.2) ------------------------------------------------

def mean_norm(row_ptr: np.ndarray, col_idx: np.ndarray) -> np.ndarray:
    """Coefficients of the mean aggregator of Sec. 4.4.2: row i of the CSR lists N_i and every
    stored entry of that row gets ``1/|N_i|`` (fp64).  A node without neighbours has no entries,
    so its neighbour term is an empty sum."""
    row_ptr, col_idx, n = _check_csr(row_ptr, col_idx)
    deg = np.diff(row_ptr)
    return np.repeat(1.0 / np.maximum(deg, 1).astype(np.float64), deg)


def sage_layer(row_ptr, col_idx, mean_coeff, h: np.ndarray, w_self: np.ndarray, w_nbr: np.ndarray,
               shift=None, mul=None) -> Dict[str, np.ndarray]:
    """One Bi-GraphSAGE layer (Sec. 4.4.2, the binarised form of the mean-aggregator layer):
    ``out_i = W~_theta (*) h~_i + (1/|N_i|) sum_{j in N_i} W~_n (*) h~_j`` where (*) is the
    binarised product of Sec. 4.2 (signs, row scale beta, column scale alpha); no non-linearity.
    Returns every intermediate."""
    sign, beta = binarize_rows(h, shift, mul)
    bt_self, alpha_self = binarize_weight(w_self)
    bt_nbr, alpha_nbr = binarize_weight(w_nbr)
    zeta_self = rescale(sign_matmul(sign, bt_self), beta, alpha_self)
    zeta_nbr = rescale(sign_matmul(sign, bt_nbr), beta, alpha_nbr)
    out = zeta_self + aggregate(row_ptr, col_idx, mean_coeff, zeta_nbr)
    return {"sign": sign, "beta": beta, "alpha_self": alpha_self, "alpha_nbr": alpha_nbr,
            "zeta_self": zeta_self, "zeta_nbr": zeta_nbr, "out": out}


def sage_forward(row_ptr, col_idx, x: np.ndarray, weights: Sequence[Tuple[np.ndarray, np.ndarray]],
                 bn: Optional[Sequence[Optional[Tuple[np.ndarray, np.ndarray]]]] = None,
                 calibrate: Optional[Sequence[bool]] = None):
    """L-layer Bi-GraphSAGE forward (Sec. 4.4.2; h^(L) is the prediction input): ``weights[l]``
    is the pair ``(W_theta, W_n)`` of layer l; ``bn`` / ``calibrate`` as in :func:`forward`
    (standardisation before each binarised layer, Sec. 7.2 Setups).  Returns the
    fp64 output and the standardisation parameters used per layer."""
    n_layers = len(weights)
    bn = list(bn) if bn is not None else [None] * n_layers
    calibrate = list(calibrate) if calibrate is not None else [False] * n_layers
    coeff = mean_norm(row_ptr, col_idx)
    h = np.asarray(x, dtype=np.float32)
    used = []
    for l in range(n_layers):
        params = bn[l]
        if calibrate[l]:
            params = column_standardisation(h)
        shift, mul = params if params is not None else (None, None)
        h = sage_layer(row_ptr, col_idx, coeff, h, weights[l][0], weights[l][1], shift, mul)["out"]
        used.append(params)
    return h, used


# ---- Bi-GAT (Sec. 4.4.1) ------------------------------------------------------------------------

def gat_layer(row_ptr, col_idx, h: np.ndarray, w: np.ndarray, a_src: np.ndarray, a_dst: np.ndarray,
              heads: int = 1, negative_slope: float = 0.2, shift=None, mul=None,
              nodes=None) -> Dict[str, np.ndarray]:
    """One Bi-GAT layer (Sec. 4.4.1): with z_j = W~ (*) h~_j (the binarised product of Sec. 4.2,
    ``heads`` blocks of d_out / heads columns, one weight block and one attention vector per
    head),

        e_ij  = LeakyReLU(a_src . z_i + a_dst . z_j)        (a^T (z_i || z_j), a not binarised)
        a_ij  = softmax over j in N_i of e_ij               (row i of the CSR lists N_i)
        out_i = sum_{j in N_i} a_ij z_j                     (no further non-linearity)

    per head, the heads' outputs side by side.  ``a_src``, ``a_dst``: (heads, d_out / heads).
    fp64 throughout; a node with an empty row gives zeros.  Returns every intermediate.
    ``nodes``: if given, ``out`` and ``att`` are computed for these nodes only (the other rows
    stay zero); ``zeta``, ``s`` and ``t`` always cover every node."""
    row_ptr, col_idx, n = _check_csr(row_ptr, col_idx)
    sign, beta = binarize_rows(h, shift, mul)
    bt, alpha = binarize_weight(w)
    zeta = rescale(sign_matmul(sign, bt), beta, alpha)               # (n, d_out)
    d_out = zeta.shape[1]
    if d_out % heads:
        raise ValueError("d_out must be a multiple of heads")
    dh = d_out // heads
    a_src = np.asarray(a_src, dtype=np.float64).reshape(heads, dh)
    a_dst = np.asarray(a_dst, dtype=np.float64).reshape(heads, dh)
    z3 = zeta.reshape(n, heads, dh)
    s = (z3 * a_src[None]).sum(axis=2)                               # (n, heads)
    t = (z3 * a_dst[None]).sum(axis=2)
    out = np.zeros((n, heads, dh), dtype=np.float64)
    att = np.zeros((col_idx.size, heads), dtype=np.float64)
    for i in (range(n) if nodes is None else (int(v) for v in nodes)):
        p0, p1 = int(row_ptr[i]), int(row_ptr[i + 1])
        if p0 == p1:
            continue
        nb = col_idx[p0:p1]
        e = s[i][None, :] + t[nb]                                    # (deg, heads)
        e = np.where(e > 0, e, negative_slope * e)
        e = np.exp(e - e.max(axis=0, keepdims=True))
        a = e / e.sum(axis=0, keepdims=True)
        att[p0:p1] = a
        out[i] = np.einsum("kh,khd->hd", a, z3[nb])
    return {"sign": sign, "beta": beta, "alpha": alpha, "zeta": zeta, "s": s, "t": t, "att": att,
            "out": out.reshape(n, d_out)}
