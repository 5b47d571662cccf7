"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path.

This module only *draws* data: mixture means, per-dimension spreads, base
vectors, queries and index permutations.  It holds none of the retrieval
method's arithmetic (no distances, no quantisers, no selection), so the
oracle and the HIP library can both be fed from it without sharing code.

The recipes stand in for the two public billion-scale descriptor sets the
paper evaluates on (Section 4, "Datasets"): 96-d L2-normalised CNN
descriptors ("deep-like") and 128-d non-negative uint8-valued histogram
descriptors ("sift-like").
"""
from .generators import (  # noqa: F401
    MASTER_SEED,
    Mixture,
    WorkloadSpec,
    WORKLOADS,
    stream_seed,
    make_mixture,
    draw_points,
    draw_queries,
    draw_indices,
    random_rotation,
)
