"""Seeded synthetic inputs (graphs, features, gradients) shared by the tests,
the bench harness and the smoke check.

This package only draws random structure and random numbers.  It contains no
aggregation arithmetic, no CSR transposition and no degree binning: those live
once in the HIP library and once, independently, in the CPU oracle.
"""
from .rng import mix64, uniform01
from .graphs import (
    EdgeList,
    erdos_renyi_directed,
    rmat_directed,
    rmat_symmetric,
    small_random_multigraph,
    regular_random_neighbours,
    relabel,
    to_csr_numpy,
)
from .features import uniform_features, normal_features, gcn_sym_edge_weights
from .workloads import WORKLOADS, make_graph, make_features

__all__ = [
    "mix64", "uniform01", "EdgeList", "erdos_renyi_directed", "rmat_directed",
    "rmat_symmetric", "small_random_multigraph", "regular_random_neighbours", "relabel", "to_csr_numpy",
    "uniform_features", "normal_features", "gcn_sym_edge_weights",
    "WORKLOADS", "make_graph", "make_features",
]
