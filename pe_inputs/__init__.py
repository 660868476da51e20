"""Seeded synthetic inputs for the Parallel Evoformer block.

This module holds workload shapes and random-number recipes only.  It contains
none of the block's arithmetic and is the single piece of code used both by the
float64 CPU oracle's tests and by the HIP path's tests and benchmark.
"""
from .configs import CONFIGS, dims_for, TINY_TEST_DIMS
from .generate import make_inputs, round_to_bf16, res_mask_for

__all__ = ["CONFIGS", "dims_for", "TINY_TEST_DIMS", "make_inputs",
           "round_to_bf16", "res_mask_for"]
