"""Seeded synthetic inputs (graphs, features, edge weights) for the five workloads.

This module only *produces inputs*: CSR adjacency structures, feature matrices and
edge-weight arrays.  It contains none of the method's arithmetic (no translation, no
SpMM, no SDDMM, no softmax), and it imports neither the CPU oracle nor the HIP library,
so both can be fed from it without sharing code with each other.
"""
from .rng import splitmix64, uniform01, uniform_pm1, normal01
from .graphs import (
    CSR,
    csr_from_undirected_pairs,
    csr_from_directed_pairs,
    erdos_renyi_gnm,
    chung_lu_powerlaw,
    rmat,
    clustered_communities,
    dense_block_windows,
    window_fill,
    sym_norm_weights,
)
from .features import features_uniform, features_normal, round_to_bf16, bf16_bits
from .configs import CONFIGS, make_config

__all__ = [
    "splitmix64", "uniform01", "uniform_pm1", "normal01",
    "CSR", "csr_from_undirected_pairs", "csr_from_directed_pairs",
    "erdos_renyi_gnm", "chung_lu_powerlaw", "rmat", "clustered_communities",
    "dense_block_windows", "window_fill", "sym_norm_weights",
    "features_uniform", "features_normal", "round_to_bf16", "bf16_bits",
    "CONFIGS", "make_config",
]
