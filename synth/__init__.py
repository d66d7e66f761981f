"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests.

This package holds input generation only (graphs as CSR, feature matrices, weight
matrices).  None of the method's arithmetic lives here: no normalisation, no window
index, no aggregation.  Both sides receive exactly the arrays produced here.
"""
from .graphs import (Graph, csr_from_pairs, erdos_renyi, chung_lu, sbm, rmat,
                     fill_controlled, config_graph, CONFIGS)
from .features import uniform_features, normal_features, glorot_uniform

__all__ = ["Graph", "csr_from_pairs", "erdos_renyi", "chung_lu", "sbm", "rmat",
           "fill_controlled", "config_graph", "CONFIGS", "uniform_features",
           "normal_features", "glorot_uniform"]
