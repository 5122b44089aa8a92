"""CPU oracle for the FC-layer matrix multiplies and their operand re-storage (TEST INFRASTRUCTURE ONLY).

Nothing in the product imports this package.  Only the tests, the smoke check
and the benchmark's cpu_baseline leg may call it.  It shares no code with the
GPU library.
"""
from .reference import (  # noqa: F401
    LAYOUTS,
    build,
    gemm,
    gemm_at,
    linear_fwd,
    linear_bwd_data,
    linear_bwd_weight,
    max_threads,
    transpose,
)
