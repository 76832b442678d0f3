"""Seeded synthetic inputs for the Bi-GCN forward path.

This package only *draws inputs* (graphs, node features, weights).  It contains
none of the method's arithmetic (no binarisation, no normalisation, no
products), so that the CPU oracle and the HIP path can both be fed from it
without sharing any computation.  Everything is generated with
``numpy.random.Generator(PCG64(seed))``; one generated instance is handed to
both sides, so no cross-language generator agreement is needed.
"""

from .configs import CONFIGS, WorkloadConfig, get_config, scaled_config
from .graphs import chung_lu_csr, csr_from_undirected_edges
from .features import make_features, glorot_uniform, make_weights
from .build import Workload, make_workload

__all__ = [
    "CONFIGS", "WorkloadConfig", "get_config", "scaled_config",
    "chung_lu_csr", "csr_from_undirected_edges",
    "make_features", "glorot_uniform", "make_weights",
    "Workload", "make_workload",
]
