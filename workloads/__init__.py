"""Seeded synthetic inputs shared by the oracle-side tests and the GPU-side tests.

This package only *draws and arranges numbers*: Gaussian vectors, orthonormal
column blocks, eigenvalue grids, mini-batches.  It contains none of the
method's arithmetic (no Lanczos step, no Hessian-vector product, no update
rule), so both the CPU oracle's tests and the HIP path's tests may import it
without sharing any part of what is being compared.
"""
from .generators import (  # noqa: F401
    ROOT_SEED,
    CONFIGS,
    StepParams,
    PlantedWorkload,
    GgnWorkload,
    philox,
    normal_vector,
    normal_matrix,
    orthonormal_columns,
    planted_spectrum,
    planted_workload,
    ggn_workload,
    gradient,
    padded_ld,
)
