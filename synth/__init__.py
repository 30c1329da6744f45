"""Seeded synthetic inputs shaped like the paper's Llama-class K/V workloads.

This package only draws random inputs (activations, codebooks, queries).  It
holds none of the method's arithmetic: no nearest-centroid search, no
attention, no code packing.  Both the CPU oracle's tests and the GPU path's
tests/bench feed from it so that the two sides see identical inputs.
"""
from .generator import (  # noqa: F401
    CONFIGS,
    WorkloadConfig,
    TensorRecipe,
    tensor_recipe,
    sample_activations,
    sample_codebook,
    sample_query,
    sample_activations_torch,
    mixing_block,
)
