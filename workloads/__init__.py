"""Seeded synthetic inputs (tree shapes and tensors) shared by the tests, the
benchmark and the CPU oracle.

This package only draws random structure and random numbers.  It contains none
of the attention arithmetic and imports neither the HIP binding nor the oracle.
"""
from .trees import (CONFIGS, config_tree, config_heads, random_tree, chain_tree,
                    scaled_config_tree)
from .tensors import make_inputs_numpy, round_to_bf16

__all__ = ["CONFIGS", "config_tree", "config_heads", "random_tree", "chain_tree",
           "scaled_config_tree", "make_inputs_numpy", "round_to_bf16"]
