"""Seeded synthetic inputs (graphs, features, weights, update batches).

This package is the only code shared by the CPU oracle's tests and the HIP path's
tests/benchmark.  It produces inputs only: it contains none of the method's
arithmetic (no aggregation, no transform, no event logic).
"""
from .rmat import rmat_edges, in_csr_from_edges, edge_keys, keys_to_edges
from .workloads import (CONFIGS, WorkloadConfig, get_config, make_features, make_model,
                        make_graph, BatchSampler, xavier_uniform)

__all__ = ["rmat_edges", "in_csr_from_edges", "edge_keys", "keys_to_edges", "CONFIGS",
           "WorkloadConfig", "get_config", "make_features", "make_model", "make_graph",
           "BatchSampler", "xavier_uniform"]
