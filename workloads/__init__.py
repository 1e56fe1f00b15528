"""Seeded synthetic inputs (graphs, features, gradients, weights).

This package only *makes inputs*: edge lists, feature arrays and their bf16
encodings.  It holds none of the propagation arithmetic and is the one module
that both the CPU oracle's tests and the GPU path's tests/bench may import.
"""
from .graphs import (  # noqa: F401
    CONFIGS,
    bf16_bits_to_f32,
    f32_to_bf16_bits,
    make_config,
    make_edge_weights,
    make_features,
    powerlaw_bipartite,
    sample_subgraph,
    uniform_bipartite,
)
