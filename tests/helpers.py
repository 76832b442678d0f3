"""Shared pieces of the GPU parity tests: tolerance, device upload, and the protocol that
compares a multi-layer forward when fp32 rounding may legitimately flip a sign bit."""
from __future__ import annotations

import numpy as np

REL_TOL = 1e-5      # fp32 outputs: |gpu - ref| <= REL_TOL * |ref| + ABS_TOL
ABS_TOL = 1e-6


def close(gpu: np.ndarray, ref: np.ndarray):
    """Boolean mask of elements within tolerance of the fp64 reference."""
    ref = np.asarray(ref, dtype=np.float64)
    gpu = np.asarray(gpu, dtype=np.float64)
    return np.abs(gpu - ref) <= REL_TOL * np.abs(ref) + ABS_TOL


def assert_close(gpu, ref, what=""):
    ok = close(gpu, ref)
    if not ok.all():
        bad = np.argwhere(~ok)
        i = tuple(bad[0])
        raise AssertionError(f"{what}: {bad.shape[0]} of {ok.size} elements out of tolerance; "
                             f"first at {i}: gpu={np.asarray(gpu)[i]!r} ref={np.asarray(ref)[i]!r}")


def to_device(*arrays):
    import torch
    out = []
    for a in arrays:
        out.append(None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda())
    return out if len(out) > 1 else out[0]


def words_to_numpy(bits) -> np.ndarray:
    """int64 device tensor of packed words -> uint64 numpy array."""
    return bits.cpu().numpy().view(np.uint64)


def neighbours_closed(row_ptr: np.ndarray, col_idx: np.ndarray, rows_mask: np.ndarray) -> np.ndarray:
    """Mask of nodes that are marked or have a marked node among their stored entries (the
    closed neighbourhood, whether or not the pattern holds the self-loop)."""
    marked_entry = rows_mask[col_idx]
    counts = np.add.reduceat(marked_entry.astype(np.int64), row_ptr[:-1].clip(max=max(col_idx.size - 1, 0)))
    counts[np.diff(row_ptr) == 0] = 0
    return (counts > 0) | rows_mask


def sign_error_bound(row_ptr, col_idx, a_tilde, zeta) -> np.ndarray:
    """Bound on |fp32 result - exact result| of sum_k a_ik zeta_kj evaluated in fp32 in any
    order: (terms + 4) * 2^-24 * sum_k |a_ik zeta_kj|.  Elements whose distance to the sign
    threshold is below this bound may legitimately come out with either sign."""
    import oracle
    mag = oracle.aggregate(row_ptr, col_idx, a_tilde, np.abs(zeta))
    terms = np.diff(row_ptr).astype(np.float64)[:, None]
    return (terms + 4.0) * 2.0 ** -24 * mag


def inherited_scale_error(beta, in_tol, mul):
    """Relative bound on the error of a layer's row scales beta_i = mean_j |(h_ij - mu_j) s_j|
    when every input element may be off by ``in_tol[i, j]`` (the tolerance granted to the previous
    layer's output): |d beta_i| <= mean_j in_tol_ij |s_j|.  Zero for the first layer (``in_tol``
    None: X is the same fp32 array on both sides)."""
    if in_tol is None:
        return np.zeros(beta.shape[0], dtype=np.float64)
    weight = np.ones(in_tol.shape[1]) if mul is None else np.abs(np.asarray(mul, dtype=np.float64))
    d_beta = (in_tol * weight[None, :]).mean(axis=1)
    return np.where(beta > 0, d_beta / np.where(beta > 0, beta, 1.0), 0.0)


class _GcnOracle:
    """Per-layer oracle of the Bi-GCN forward, the fp32 rounding bound of its output, and the
    error its output inherits from the tolerance of its input through the row scales."""

    def __init__(self, work):
        import oracle
        self.work = work
        self.coeff = oracle.gcn_norm(work.row_ptr, work.col_idx)

    def layer(self, l, h, shift, mul, in_tol=None):
        import oracle
        w = self.work
        rec = oracle.layer(w.row_ptr, w.col_idx, self.coeff, h, w.weights[l], shift, mul)
        rel = inherited_scale_error(rec["beta"], in_tol, mul)
        inherited = oracle.aggregate(w.row_ptr, w.col_idx, self.coeff, np.abs(rec["zeta"]) * rel[:, None])
        return rec["out"], sign_error_bound(w.row_ptr, w.col_idx, self.coeff, rec["zeta"]), inherited


class _SageOracle:
    """The same for the Bi-GraphSAGE forward: the own term is one more summand of the fp32 sum."""

    def __init__(self, work):
        import oracle
        self.work = work
        self.coeff = oracle.mean_norm(work.row_ptr, work.col_idx)

    def layer(self, l, h, shift, mul, in_tol=None):
        import oracle
        w = self.work
        rec = oracle.sage_layer(w.row_ptr, w.col_idx, self.coeff, h, w.weights[l][0], w.weights[l][1],
                                shift, mul)
        mag = oracle.aggregate(w.row_ptr, w.col_idx, self.coeff, np.abs(rec["zeta_nbr"]))
        mag += np.abs(rec["zeta_self"])
        terms = np.diff(w.row_ptr).astype(np.float64)[:, None]
        rel = inherited_scale_error(rec["beta"], in_tol, mul)
        inherited = oracle.aggregate(w.row_ptr, w.col_idx, self.coeff, np.abs(rec["zeta_nbr"]) * rel[:, None])
        inherited += np.abs(rec["zeta_self"]) * rel[:, None]
        return rec["out"], (terms + 6.0) * 2.0 ** -24 * mag, inherited


def compare_forward_layerwise(work, bn, run_gpu_prefix, cancellation_aware=False, log=None):
    """Layer-by-layer parity of the fused forward against the oracle (Bi-GCN or Bi-GraphSAGE,
    as the workload's config says).

    ``bn[l]`` is the frozen standardisation ``(shift, mul)`` of layer l's input, ``None`` for no
    standardisation, or the string ``"calibrate"``: the parameters are then computed here from
    the oracle's own input of that layer and handed to the GPU side as fp32.
    ``run_gpu_prefix(l, params)`` must return the GPU result of the first ``l`` layers (fp32
    H^(l), numpy) using ``params[:l]``.  Every H^(l) is compared with the oracle's on all rows
    whose inputs were identical on both sides.  Where the GPU's fp32 value of a hidden activation
    falls on the other side of its threshold than the oracle's, the element must lie within the
    fp32 error bound of the threshold (both signs are then valid results); such rows, and the
    rows they feed, are left out of the comparison of later layers.  The oracle runs one layer at
    a time so that only one layer's intermediates are alive.  Nothing flows from the GPU into
    the oracle.  Returns per-layer statistics.

    ``cancellation_aware`` (adversarial inputs and degenerate shapes only): an element also
    passes when its error is within the fp32 rounding bound of its own sum, ``sign_error_bound``,
    plus what it inherits from its input: the row scales beta of a layer are computed from the
    previous layer's fp32 output, so the tolerance granted there (1e-5 relative, or that layer's
    own bound) reappears as a relative error of every summand beta_k alpha_j c_kj of this layer
    (``inherited_scale_error``).  With products of magnitude K next to products near 0 a neighbour
    sum can cancel to 1e-9 of its terms, which no fp32 evaluation order resolves to 1e-5 of the
    result; and a sum of 512 signed products of a 2-bit layer cancels enough for a 1e-5 error of
    its scales to show as 5e-5 of the result.
    """
    import oracle
    say = log if log is not None else (lambda *a: None)
    n_layers = len(work.weights)
    model = _SageOracle(work) if work.config.model == "sage" else _GcnOracle(work)
    tainted = np.zeros(work.n, dtype=bool)
    params = []
    stats = []
    h = work.x
    in_tol = None
    for l in range(1, n_layers + 1):
        p = bn[l - 1]
        if isinstance(p, str):
            assert p == "calibrate"
            p = oracle.column_standardisation(h)
        params.append(p)
        shift, mul = p if p is not None else (None, None)
        if l > 1:
            # signs of this layer's input as the oracle takes them, against the GPU's previous output
            th = np.zeros(h.shape[1], dtype=np.float32) if shift is None else shift
            flips = (gpu >= th[None, :]) != (h.astype(np.float32) >= th[None, :])
            margin = np.abs(h - th[None, :].astype(np.float64))
            illegal = flips & clean[:, None] & (margin > bound + 1e-30)
            assert not illegal.any(), (f"layer {l - 1}: {int(illegal.sum())} sign bits differ from "
                                       f"the oracle outside the fp32 error bound")
            stats[-1]["sign_flips"] = int((flips & clean[:, None]).sum())
            tainted = neighbours_closed(work.row_ptr, work.col_idx, tainted | flips.any(axis=1))
            del flips, margin, illegal, bound, gpu
        ref, bound, inherited = model.layer(l - 1, h, shift, mul, in_tol if cancellation_aware else None)
        say(f"oracle layer {l} done")
        gpu = run_gpu_prefix(l, params)
        say(f"gpu prefix {l} done")
        assert gpu.shape == ref.shape
        ok = close(gpu, ref)
        if cancellation_aware:
            bound = bound + inherited
            ok |= np.abs(gpu - ref) <= bound
            # what this layer's elements were allowed to be off by: the next layer's input tolerance
            in_tol = np.maximum(REL_TOL * np.abs(ref) + ABS_TOL, bound)
        clean = ~tainted
        if not ok[clean].all():
            bad = np.argwhere(~ok & clean[:, None])
            i = tuple(bad[0])
            raise AssertionError(f"layer {l}: {bad.shape[0]} elements out of tolerance on rows with "
                                 f"identical inputs; first at {i}: gpu={gpu[i]!r} ref={ref[i]!r}")
        del ok
        stats.append({"layer": l, "rows_compared": int(clean.sum()), "sign_flips": 0})
        h = ref
    return stats


def compare_forward_teacher_forced(work, bn, run_gpu_prefix, log=None, own_sum_bound=False):
    """Layer-level parity with the layer input taken from the GPU (the second mode of the parity
    protocol): the oracle evaluates layer l from the GPU's own fp32 H^(l-1) (layer 1 from X), so
    both sides binarise identical numbers, every sign bit is the same by construction, and EVERY
    row of every layer is held to the plain tolerance: no row is left out because an earlier
    layer's activation sat within rounding of its threshold, and no rounding bound is granted.

    ``bn[l]`` as in compare_forward_layerwise; "calibrate" computes the parameters from the layer's
    input as the oracle sees it here (the GPU's previous output), and both sides use them.

    One caveat is handled explicitly: the GPU binarises a hidden activation inside the aggregation
    kernel, from the value in its registers, while this comparison sees that activation as the
    fp32 output of a shorter forward.  The two are the same arithmetic; should a build ever round
    them differently in the last place, an element within 4 units in the last place of its
    threshold could take the other sign.  Rows fed by such an element (``ambiguous_rows``) are
    reported and excused if, and only if, they fail; their number must stay below 1e-5 of the rows.

    ``own_sum_bound`` (adversarial inputs only: rows equal to a weight column, layers of one or two
    bits): an element also passes inside the worst-case rounding bound of ITS OWN fp32 neighbour
    sum, (terms + 4) 2^-24 sum_k |a_ik zeta_kj| (``sign_error_bound``): products of magnitude K
    next to products near 0 cancel to 1e-9 of their terms, which no fp32 summation order resolves
    to 1e-5 of the result.  Nothing is granted for errors inherited from earlier layers: there are
    none in this mode.  The number of elements that needed the bound is returned.
    """
    import oracle
    say = log if log is not None else (lambda *a: None)
    n_layers = len(work.weights)
    model = _SageOracle(work) if work.config.model == "sage" else _GcnOracle(work)
    params, stats = [], []
    h = work.x
    for l in range(1, n_layers + 1):
        p = bn[l - 1]
        if isinstance(p, str):
            assert p == "calibrate"
            p = oracle.column_standardisation(h)
        params.append(p)
        shift, mul = p if p is not None else (None, None)
        ref, bound, _ = model.layer(l - 1, h, shift, mul, None)
        say(f"teacher-forced oracle layer {l} done")
        gpu = run_gpu_prefix(l, params)
        say(f"gpu prefix {l} done")
        assert gpu.shape == ref.shape
        ok = close(gpu, ref)
        by_bound = 0
        if own_sum_bound:
            inside = np.abs(gpu - ref) <= bound
            by_bound = int((inside & ~ok).sum())
            ok |= inside
        del bound
        excused = 0
        if not ok.all() and l > 1:
            th = np.zeros(h.shape[1], dtype=np.float64) if shift is None else np.asarray(shift, dtype=np.float64)
            near = np.abs(h - th[None, :]) <= 4 * 2.0 ** -23 * np.maximum(np.abs(h), np.abs(th)[None, :])
            ambiguous = neighbours_closed(work.row_ptr, work.col_idx, near.any(axis=1))
            bad_rows = ~ok.all(axis=1)
            excused = int((bad_rows & ambiguous).sum())
            ok[ambiguous] = True
            assert excused <= 1e-5 * work.n + 1, f"layer {l}: {excused} rows differ next to a threshold"
        if not ok.all():
            bad = np.argwhere(~ok)
            i = tuple(bad[0])
            raise AssertionError(f"teacher-forced layer {l}: {bad.shape[0]} of {ok.size} elements out of the plain "
                                 f"tolerance; first at {i}: gpu={gpu[i]!r} ref={ref[i]!r}")
        stats.append({"layer": l, "rows_compared": int(work.n), "excused_rows": excused,
                      "passed_by_own_sum_bound": by_bound})
        h = gpu.astype(np.float64) if l < n_layers else None
        del ref, ok
    return stats


def decode_product_rows(workspace: np.ndarray, offsets: dict, layout: dict, n: int, d_out: int):
    """The integer products that a one-layer bigcn_forward left in its workspace, decoded from the
    documented row format (include/bigcn.h, bigcn_forward_row_layout): returns (values, k_eff,
    escaped) where values[i, j] is the product over the first k_eff input bits, c'_ij = sum_{k<k_eff}
    F_ik B_kj, as int64, and escaped[i] says that row i was read from the alternate array.
    Pure byte manipulation; shares nothing with the library."""
    G, V, kind, k_eff = layout["groups"], layout["vec"], layout["kind"], layout["k_eff"]
    place, escape, alt_kind = layout["scale_place"], layout["escape"], layout["alt_kind"]
    pos = G * V
    elem = {0: 1, 1: 2, 2: 4}[kind]
    raw = workspace[offsets["rows"]: offsets["rows"] + n * pos * elem]
    escaped = np.zeros(n, dtype=bool)
    if kind == 0:
        b = raw.view(np.uint8).reshape(n, pos)
        if place == 2:
            # 7-bit two's complement in bits 0..6; bit 7 of the carrier bytes belongs to the scale
            q = ((b & 0x7f).astype(np.int64) ^ 0x40) - 0x40
            seg = b.reshape(n, G, V)
            if G >= 32:
                bits = (seg[:, :32, 0] >> 7).astype(np.uint32)
                scale_word = (bits << np.arange(32, dtype=np.uint32)[None, :]).sum(axis=1, dtype=np.uint64)
            else:
                assert G == 16
                lo = (seg[:, :, 0] >> 7).astype(np.uint32)
                hi = (seg[:, :, 4] >> 7).astype(np.uint32)
                scale_word = ((lo << np.arange(16, dtype=np.uint32)[None, :]).sum(axis=1, dtype=np.uint64)
                              | (hi << np.arange(16, 32, dtype=np.uint32)[None, :]).sum(axis=1, dtype=np.uint64))
            scale = scale_word.astype(np.uint32).view(np.float32)
        else:
            q = b.view(np.int8).astype(np.int64)
            scale = None
            if place == 3:
                # 8 lanes of 8 values: byte i of the scale is the last byte of lane 4 + i
                assert G == 8 and V == 8
                seg = b.reshape(n, G, V)
                scale_word = sum(seg[:, 4 + i, 7].astype(np.uint64) << np.uint64(8 * i) for i in range(4))
                scale = scale_word.astype(np.uint32).view(np.float32)
        if escape:
            assert scale is not None
            escaped = np.isnan(scale)
            alt_elem = 1 if alt_kind == 0 else 2
            alt = workspace[offsets["alt_rows"]: offsets["alt_rows"] + n * pos * alt_elem]
            if alt_kind == 0:
                alt_q = alt.view(np.int8).reshape(n, pos).astype(np.int64)
            else:
                alt_q = alt.view(np.float16).reshape(n, pos).astype(np.float64)
                assert np.array_equal(alt_q[escaped], np.rint(alt_q[escaped]))
                alt_q = alt_q.astype(np.int64)
            q = np.where(escaped[:, None], alt_q, q)
        elif scale is not None:
            assert not np.isnan(scale).any()
        stored = 2 * q + (k_eff & 1)
    elif kind == 1:
        f = raw.view(np.float16).reshape(n, pos).astype(np.float64)
        stored = f.astype(np.int64)
    else:
        f = raw.view(np.float32).reshape(n, pos).astype(np.float64)
        stored = f.astype(np.int64)
    # stored position g * V + v holds output column g + G * v
    g = np.arange(G)[:, None]
    v = np.arange(V)[None, :]
    col = (g + G * v).reshape(-1)
    values = np.zeros((n, d_out), dtype=np.int64)
    keep = col < d_out
    values[:, col[keep]] = stored[:, np.nonzero(keep)[0]]
    return values, k_eff, escaped
