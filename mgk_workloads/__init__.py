"""Seeded synthetic graph workloads shared by the CPU oracle tests and the GPU path.

This package holds input generation only: no kernel arithmetic, no solver, no
packing.  Both the oracle and the HIP library consume the plain arrays of a
:class:`GraphBatch`; neither imports the other.
"""
from .generators import (  # noqa: F401
    GraphBatch,
    KernelParams,
    SEED_BASE,
    config0,
    config1,
    config2,
    config3,
    config4,
    erdos_renyi_batch,
    molecule_like_batch,
    morton_rank,
    geometric_batch,
    newman_watts_strogatz_batch,
    barabasi_albert_batch,
    concat_batches,
    permute_vertices,
    with_label_attributes,
    gram_pairs,
    paper_synthetic,
)
