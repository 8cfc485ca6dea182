"""Seeded synthetic inputs for the RSR++ vector-matrix product.

This package holds input generators only: random weight matrices with entries in
{0,1} or {-1,0,1} and random activation vectors, in the shapes and value
distributions of the benchmark configurations.  It contains none of the method's
arithmetic (no blocking, sorting, segment sums or products), so both the CPU
oracle's tests and the HIP path's tests may draw their inputs from it.

The paper's own timing runs use random binary/ternary matrices and random
vectors (Section 5.1); its language-model runs need trained 1.58-bit weights,
for which the "llm_block" configuration stands in by shape and value law only.
"""
from .configs import (  # noqa: F401
    CONFIGS,
    SEED_BASE,
    Workload,
    binary_matrix,
    correlated_ternary_matrix,
    get,
    llm_block_stages,
    stage_matrix,
    make_activations,
    seed_for,
    ternary_matrix,
)
