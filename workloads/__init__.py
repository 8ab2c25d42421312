"""Seeded synthetic inputs for the fused-subgraph workloads.

This package only draws numbers and names shapes.  It contains none of the
arithmetic of the subgraphs themselves (no convolution, GEMM, activation or
softmax), so that the CPU oracle and the HIP path can both take their inputs
from it without sharing any part of the method.
"""

from .rng import uniform, normal, round_to_bf16, bf16_bits, bf16_from_bits
from .configs import (
    InvresCase, ChainCase, FfnCase, AttnCase, PairCase, QkvCase,
    baseline_case, BASELINE_NAMES, small_cases, pair_cases, network_block_cases,
)

__all__ = [
    "uniform", "normal", "round_to_bf16", "bf16_bits", "bf16_from_bits",
    "InvresCase", "ChainCase", "FfnCase", "AttnCase", "PairCase", "QkvCase",
    "baseline_case", "BASELINE_NAMES", "small_cases", "pair_cases", "network_block_cases",
]
