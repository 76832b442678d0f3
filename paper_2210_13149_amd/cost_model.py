"""Closed-form storage and work counts of Sec. 5 ("Analysis of Efficiency").

These are the paper's *theoretical* figures (it reports no measured time): sizes in bytes,
work in "cycle operations" (one fp multiply plus one add), with 64 binary operations counted
as one cycle operation (Sec. 5.3).  The benchmark prints them beside measured numbers as
context only.
"""

from __future__ import annotations

from typing import Dict, Sequence


def _layers(dims: Sequence[int]):
    return list(zip(dims[:-1], dims[1:]))


def model_size_bytes(dims: Sequence[int]) -> float:
    """fp32 GCN parameters, no bias (Sec. 5.1)."""
    return 4.0 * sum(a * b for a, b in _layers(dims))


def model_size_bytes_binary(dims: Sequence[int]) -> float:
    """d_in*d_out bits plus d_out fp32 scales per layer (Sec. 5.1)."""
    return sum(a * b / 8.0 + 4.0 * b for a, b in _layers(dims))


def data_size_bytes(n: int, d: int) -> float:
    """fp32 node features (Sec. 5.2)."""
    return 4.0 * n * d


def data_size_bytes_binary(n: int, d: int) -> float:
    """N*d bits plus N fp32 scales (Sec. 5.2)."""
    return n * d / 8.0 + 4.0 * n


def cycle_ops(n: int, n_edges: int, dims: Sequence[int]) -> float:
    """N*d_in*d_out multiply-adds for the transform plus |E|*d_out for the aggregation
    (Sec. 5.3), summed over layers."""
    return float(sum(n * a * b + n_edges * b for a, b in _layers(dims)))


def cycle_ops_binary(n: int, n_edges: int, dims: Sequence[int]) -> float:
    """N*d_in*d_out binary operations at 1/64 of a cycle operation each, 2*N*d_out fp
    multiplications for the scales, and the unchanged aggregation (Sec. 5.3)."""
    return float(sum(n * a * b / 64.0 + 2.0 * n * b + n_edges * b for a, b in _layers(dims)))


def parameter_compression(d_in: int) -> float:
    """PC = 32 d_in / (d_in + 32) (Sec. 5.1)."""
    return 32.0 * d_in / (d_in + 32.0)


def data_compression(d: int) -> float:
    """DC = 32 d / (d + 32) (Sec. 5.2)."""
    return 32.0 * d / (d + 32.0)


def speedup_feature_extraction(d_in: int) -> float:
    """S_fe = 64 d_in / (d_in + 128) (Sec. 5.3)."""
    return 64.0 * d_in / (d_in + 128.0)


def speedup_layer(d_in: int, mean_degree: float) -> float:
    """S_full = (64 d_in + 32 deg) / (d_in + 128 + 32 deg) (Sec. 5.3)."""
    return (64.0 * d_in + 32.0 * mean_degree) / (d_in + 128.0 + 32.0 * mean_degree)


def sage_summary(n: int, n_edges: int, dims: Sequence[int]) -> Dict[str, float]:
    """The same counts for the mean-aggregator GraphSAGE layer and its binarised form
    (Sec. 4.4.2): two weight matrices per layer, so parameters and transform work double while
    the aggregation term |E|*d_out and the loaded features stay as they are."""
    ms, msb = 2.0 * model_size_bytes(dims), 2.0 * model_size_bytes_binary(dims)
    co = float(sum(2 * n * a * b + n_edges * b for a, b in _layers(dims)))
    cob = float(sum(2.0 * (n * a * b / 64.0 + 2.0 * n * b) + n_edges * b for a, b in _layers(dims)))
    return {"model_size_bytes": ms, "model_size_bytes_binary": msb, "model_size_ratio": ms / msb,
            "cycle_ops": co, "cycle_ops_binary": cob, "cycle_ops_ratio": co / cob}


def summary(n: int, n_edges: int, dims: Sequence[int]) -> Dict[str, float]:
    ms, msb = model_size_bytes(dims), model_size_bytes_binary(dims)
    ds, dsb = data_size_bytes(n, dims[0]), data_size_bytes_binary(n, dims[0])
    co, cob = cycle_ops(n, n_edges, dims), cycle_ops_binary(n, n_edges, dims)
    return {
        "model_size_bytes": ms, "model_size_bytes_binary": msb, "model_size_ratio": ms / msb,
        "data_size_bytes": ds, "data_size_bytes_binary": dsb, "data_size_ratio": ds / dsb,
        "cycle_ops": co, "cycle_ops_binary": cob, "cycle_ops_ratio": co / cob,
    }
