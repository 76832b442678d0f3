"""The benchmark workloads, as data.

Shapes follow the datasets table of the paper's evaluation section (Cora,
CiteSeer, PubMed, Reddit, OGBN-Products); none of those datasets is reproduced:
graphs are Chung-Lu random graphs and features are drawn from simple
distributions with the same dimensions and density.  c1..c5 are Bi-GCN models
(graph stored as A + I); s4 and s5 are Bi-GraphSAGE models (graph stored as the
neighbour lists, two weight matrices per layer) with the hidden widths of the
paper's set-up: 256 on Reddit, 512 and three layers on OGBN-Products.
"""

from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Tuple

BASE_SEED = 221013149


@dataclass(frozen=True)
class WorkloadConfig:
    name: str
    stands_in_for: str
    n_nodes: int
    n_edges: int               # undirected edges, self-loops not counted
    i0: float                  # offset of the power-law weight sequence (sets the max degree)
    dims: Tuple[int, ...]      # d_0 -> d_1 -> ... -> d_L
    feature_kind: str          # "bernoulli" | "tfidf" | "normal"
    feature_density: float     # fraction of non-zeros (bernoulli / tfidf)
    bn_layers: str             # "first" (input features only) or "all" (before every layer)
    seed: int
    gamma: float = 2.5         # power-law exponent of the expected-degree sequence
    shuffle_ids: bool = True   # random node relabelling (False: ids by decreasing expected degree)
    model: str = "gcn"         # "gcn": pattern of A + I, one weight per layer
                               # "sage": pattern of A, a (W_theta, W_n) pair per layer

    @property
    def n_layers(self) -> int:
        return len(self.dims) - 1

    @property
    def nnz(self) -> int:
        return 2 * self.n_edges + (self.n_nodes if self.model == "gcn" else 0)


CONFIGS = {
    "c1": WorkloadConfig("c1", "Cora", 2708, 5278, 2.1, (1433, 64, 7),
                         "bernoulli", 0.0127, "first", BASE_SEED + 1),
    "c2": WorkloadConfig("c2", "CiteSeer", 3327, 4552, 3.4, (3703, 64, 6),
                         "bernoulli", 0.0085, "first", BASE_SEED + 2),
    "c3": WorkloadConfig("c3", "PubMed", 19717, 44324, 19.0, (500, 64, 3),
                         "tfidf", 0.10, "first", BASE_SEED + 3),
    "c4": WorkloadConfig("c4", "Reddit", 232965, 57_300_000, 186.0, (602, 128, 41),
                         "normal", 1.0, "all", BASE_SEED + 4),
    "c5": WorkloadConfig("c5", "OGBN-Products", 2449029, 61_859_140, 77.0, (100, 256, 256, 47),
                         "normal", 1.0, "all", BASE_SEED + 5),
    "s4": WorkloadConfig("s4", "Reddit", 232965, 57_300_000, 186.0, (602, 256, 41),
                         "normal", 1.0, "all", BASE_SEED + 14, model="sage"),
    "s5": WorkloadConfig("s5", "OGBN-Products", 2449029, 61_859_140, 77.0, (100, 512, 512, 47),
                         "normal", 1.0, "all", BASE_SEED + 15, model="sage"),
}


def get_config(name: str) -> WorkloadConfig:
    try:
        return CONFIGS[name]
    except KeyError:
        raise KeyError(f"unknown workload {name!r}; choose one of {sorted(CONFIGS)}") from None


def scaled_config(name: str, n_nodes: int) -> WorkloadConfig:
    """The same recipe on fewer nodes: mean degree, dims, feature law and the head of the
    power-law weight sequence (gamma, i0) are kept; the edge count shrinks with the node count."""
    cfg = get_config(name)
    if n_nodes >= cfg.n_nodes:
        return cfg
    ratio = n_nodes / cfg.n_nodes
    n_edges = max(1, int(round(cfg.n_edges * ratio)))
    # a simple graph on n nodes holds at most n(n-1)/2 edges; stay well below that
    n_edges = min(n_edges, n_nodes * (n_nodes - 1) // 4)
    return replace(cfg, name=f"{cfg.name}@{n_nodes}", n_nodes=n_nodes, n_edges=n_edges)
