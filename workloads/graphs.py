"""Seeded Chung-Lu power-law graphs in symmetric CSR form.

The CSR produced here is the *pattern* of A + I (paper, Notations: the adjacency
matrix of an undirected graph plus the identity) or, with ``self_loops=False``,
of A alone (row i lists the neighbours N_i).  No normalisation coefficient is
computed in this module.
"""

from __future__ import annotations

import numpy as np


def csr_from_undirected_edges(n: int, u: np.ndarray, v: np.ndarray, self_loops: bool = True):
    """Pattern of A + I (or of A, ``self_loops=False``) from a list of distinct undirected
    edges {u, v}, u != v.

    Returns (row_ptr int64[n+1], col_idx int32[nnz]) with both directions of every edge,
    one self-loop per node unless switched off, and strictly increasing columns inside each row.
    """
    u = np.asarray(u, dtype=np.int64)
    v = np.asarray(v, dtype=np.int64)
    if u.shape != v.shape or u.ndim != 1:
        raise ValueError("u and v must be 1-D arrays of equal length")
    if u.size and (min(u.min(), v.min()) < 0 or max(u.max(), v.max()) >= n):
        raise ValueError("edge endpoint out of range")
    if np.any(u == v):
        raise ValueError("self-pairs are not edges; the self-loop is added here")
    loops = np.arange(n if self_loops else 0, dtype=np.int64)
    key = np.concatenate([u * n + v, v * n + u, loops * n + loops])
    key.sort()
    if key.size > 1 and np.any(key[1:] == key[:-1]):
        raise ValueError("duplicate edges")
    rows = key // n
    col_idx = (key - rows * n).astype(np.int32)
    counts = np.bincount(rows, minlength=n)
    row_ptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(counts, out=row_ptr[1:])
    return row_ptr, col_idx


def _draw_endpoints(rng: np.random.Generator, n: int, gamma: float, i0: float, m: int) -> np.ndarray:
    """m node ranks in [0, n): rank i is drawn with probability proportional to the integral
    of (x + i0)^(-1/(gamma-1)) over [i, i+1), by inverting that law's distribution function."""
    e = 1.0 / (gamma - 1.0)
    if abs(e - 1.0) < 1e-12:
        raise ValueError("gamma = 2 is not supported")
    q = 1.0 - e
    a = i0 ** q
    b = (n + i0) ** q
    x = rng.random(m)
    x *= (b - a)
    x += a
    np.power(x, 1.0 / q, out=x)
    x -= i0
    idx = x.astype(np.int64)
    np.clip(idx, 0, n - 1, out=idx)
    return idx


def _sorted_unique_inplace(keys: np.ndarray) -> np.ndarray:
    keys.sort()
    if keys.size < 2:
        return keys
    keep = np.empty(keys.size, dtype=bool)
    keep[0] = True
    np.not_equal(keys[1:], keys[:-1], out=keep[1:])
    return keys[keep]


def chung_lu_edges(n: int, n_edges: int, gamma: float, i0: float, rng: np.random.Generator,
                   shuffle_ids: bool = True):
    """Exactly ``n_edges`` distinct undirected edges whose two endpoints are drawn
    independently from a power law over node ranks, w_i ~ (i + i0)^(-1/(gamma-1)).

    Pairs with equal endpoints and repeated pairs are rejected and redrawn, so the
    heaviest nodes end up somewhat below their expected degree when the graph is dense.
    Node ids are randomly relabelled afterwards (real datasets are not degree-sorted) unless
    ``shuffle_ids`` is False, in which case ids follow decreasing expected degree.
    """
    if n < 2:
        raise ValueError("need at least two nodes")
    if n_edges > n * (n - 1) // 2:
        raise ValueError("more edges than a simple graph can hold")
    keys = np.empty(0, dtype=np.int64)
    while keys.size < n_edges:
        m = int((n_edges - keys.size) * 1.15) + 1024
        a = _draw_endpoints(rng, n, gamma, i0, m)
        b = _draw_endpoints(rng, n, gamma, i0, m)
        lo = np.minimum(a, b)
        np.maximum(a, b, out=b)
        ok = lo != b
        lo *= n
        lo += b
        batch = _sorted_unique_inplace(lo[ok])
        del a, b, lo, ok
        if keys.size:
            pos = np.searchsorted(keys, batch)
            pos[pos == keys.size] = keys.size - 1
            batch = batch[keys[pos] != batch]
            keys = np.concatenate([keys, batch])
            keys.sort()
        else:
            keys = batch
    if keys.size > n_edges:
        drop = rng.choice(keys.size, size=keys.size - n_edges, replace=False)
        keep = np.ones(keys.size, dtype=bool)
        keep[drop] = False
        keys = keys[keep]
    lo = keys // n
    hi = keys - lo * n
    if not shuffle_ids:
        return lo, hi
    relabel = rng.permutation(n)
    return relabel[lo], relabel[hi]


def chung_lu_csr(n: int, n_edges: int, gamma: float = 2.5, i0: float = 1.0, seed: int = 0,
                 shuffle_ids: bool = True, self_loops: bool = True):
    """Symmetric CSR pattern of A + I (of A with ``self_loops=False``) for a seeded Chung-Lu
    graph.

    Returns (row_ptr int64[n+1], col_idx int32[2*n_edges (+ n)]).
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    u, v = chung_lu_edges(n, n_edges, gamma, i0, rng, shuffle_ids)
    return csr_from_undirected_edges(n, u, v, self_loops)
