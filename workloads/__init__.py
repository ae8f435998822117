"""Seeded synthetic inputs (graphs in CSR, dense feature matrices, weights).

This package only *produces inputs*: it holds none of the SpMM / selector /
condensing arithmetic, and is the one module that both the CPU oracle's tests
and the GPU path's tests may import.
"""
from .graphs import (  # noqa: F401
    CSRGraph,
    chung_lu_graph,
    sbm_graph,
    disjoint_union,
    gcn_normalise,
    random_relabel,
    CONFIGS,
    make_config,
    dense_uniform,
    dense_normal,
    glorot_uniform,
    to_bf16_bits,
    bf16_bits_to_f32,
    to_f16_bits,
    tiny_random_csr,
)
