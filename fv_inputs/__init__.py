"""Seeded synthetic inputs (shapes, weights, prefixes, draft trees).

This package is shared by the tests, the benchmark, the CPU oracle's callers and
the HIP library's callers.  It holds no arithmetic of the verification method
itself: it only draws numbers and lays out tree topologies.
"""
from .shapes import ModelShape, SHAPES, shape_by_name
from .weights import gen_weights, gen_drafter_weights, gen_features, bf16_bits_from_f32, f32_from_bf16_bits, sub_model
from .trees import gen_tree, chain_tree, gen_prefix, tree_depths, random_branching, sibling_ranks
from .drafter import draft_tree

__all__ = [
    "ModelShape", "SHAPES", "shape_by_name",
    "gen_weights", "gen_drafter_weights", "gen_features", "bf16_bits_from_f32", "f32_from_bf16_bits", "sub_model",
    "gen_tree", "chain_tree", "gen_prefix", "tree_depths", "random_branching", "sibling_ranks", "draft_tree",
]
