"""Seeded synthetic inputs (forests, node features, weights).

This package only draws inputs.  It holds none of the scheduling or Tree-LSTM
arithmetic, so both the CPU oracle's tests and the HIP path's tests may use it
without sharing any of the method's code.
"""
from .forests import (  # noqa: F401
    CONFIGS,
    ForestConfig,
    make_forest,
    make_values,
    make_workload,
    relabel,
    tree_ranges,
    to_bf16_bits,
    bf16_bits_to_f32,
    chain_forest,
    star_forest,
    perfect_kary_tree,
    tree_signatures,
    node_signatures,
    bounded_arity_forest,
    arity_signatures,
    make_cell_values,
    mixed_forest,
    make_values_typed,
)
