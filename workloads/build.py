"""Assemble one workload instance (graph + features + weights) from a config."""

from __future__ import annotations

from dataclasses import dataclass
from typing import List

import numpy as np

from .configs import WorkloadConfig, get_config
from .features import make_features, make_weights
from .graphs import chung_lu_csr


@dataclass
class Workload:
    config: WorkloadConfig
    row_ptr: np.ndarray        # int64 [n+1], pattern of A + I (model "gcn") or of A ("sage")
    col_idx: np.ndarray        # int32 [nnz]
    x: np.ndarray              # fp32 [n, d_0]
    weights: List              # per layer: fp32 [d_l, d_{l+1}] ("gcn") or a pair of them ("sage")

    @property
    def n(self) -> int:
        return int(self.row_ptr.size - 1)

    @property
    def nnz(self) -> int:
        return int(self.col_idx.size)


def make_workload(cfg) -> Workload:
    """Generate the instance for a config (or config name).  Graph, features and weights use
    independent streams derived from the config's seed, so each can be regenerated alone."""
    if isinstance(cfg, str):
        cfg = get_config(cfg)
    row_ptr, col_idx = chung_lu_csr(cfg.n_nodes, cfg.n_edges, cfg.gamma, cfg.i0, seed=cfg.seed,
                                    shuffle_ids=cfg.shuffle_ids, self_loops=cfg.model == "gcn")
    rng_x = np.random.Generator(np.random.PCG64([cfg.seed, 1]))
    rng_w = np.random.Generator(np.random.PCG64([cfg.seed, 2]))
    x = make_features(cfg.feature_kind, cfg.n_nodes, cfg.dims[0], cfg.feature_density, rng_x)
    weights = make_weights(cfg.dims, rng_w)
    if cfg.model == "sage":
        weights = list(zip(weights, make_weights(cfg.dims, rng_w)))
    return Workload(cfg, row_ptr, col_idx, x, weights)
