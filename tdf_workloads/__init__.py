"""Seeded synthetic inputs for the five workloads (integer recursion and recursive tree
networks).  This module holds input generation only: a counter-based 64-bit generator,
random binary trees, token ids and parameter tensors.  It contains none of the tagged
dataflow method's arithmetic and is the only code shared by the CPU oracle's tests and
the GPU path's tests.
"""
from .rng import SplitMix64
from .trees import Forest, random_split_tree, left_chain_tree, complete_tree, build_forest, permuted
from .configs import make_config, CONFIG_NAMES, BASE_SEED, round_to_bf16

__all__ = [
    "SplitMix64", "Forest", "random_split_tree", "left_chain_tree", "complete_tree",
    "build_forest", "permuted", "make_config", "CONFIG_NAMES", "BASE_SEED", "round_to_bf16",
]
