"""Seeded synthetic PLAID workloads (index buffers + queries).

This package only *draws inputs*: it is the one module that both the CPU
oracle's tests and the HIP path's tests/benchmarks share.  It holds none of the
search path's arithmetic (no S_cq, no centroid interaction, no decompression,
no MaxSim, no top-k) and imports neither the oracle nor the HIP library.
"""
from .workload import (  # noqa: F401
    CONFIGS,
    WorkloadConfig,
    Workload,
    get_config,
    make_workload,
    tiny_config,
    save_index_file,
    index_nbytes,
)
