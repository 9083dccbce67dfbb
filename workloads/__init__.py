"""Seeded synthetic inputs for the SpecVocab draft-step hot path.

This module is the only code shared by the CPU oracle's tests and the HIP path's
tests / benchmark.  It holds no arithmetic of the method itself: only random
draws, dtype conversion of the drawn values, and the shape tables of the
workloads.
"""
from .gen import (  # noqa: F401
    CONFIGS,
    Workload,
    bf16_bits_to_f32,
    f32_to_bf16_bits,
    hidden_rows,
    make_rng,
    normal_matrix,
    tree_subsets,
    zipf_subset,
    zipf_subsets,
)
