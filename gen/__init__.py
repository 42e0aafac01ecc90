"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests.

This package draws random inputs only.  It contains none of the method's
arithmetic (no distances, no neighbourhoods, no updates) and imports neither
the oracle nor the HIP binding.
"""
from .workloads import (  # noqa: F401
    CONFIGS,
    Workload,
    dense_uniform,
    dense_mixture,
    sparse_zipf_csr,
    sparse_uniform_csr,
    codebook_uniform,
    make_workload,
    scaled_workload,
)
