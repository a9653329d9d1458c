"""Seeded synthetic inputs for the coalesced-superkernel path.

This package only *describes* and *draws* inputs: operator shapes, dtypes,
deadlines and random tensors.  It contains none of the method's arithmetic
(no GEMM, no convolution, no tiling) and is the one module both the CPU
oracle's tests and the HIP path's tests/benchmarks take their inputs from.
"""
from .configs import (  # noqa: F401
    Problem,
    config,
    config_names,
    draw_host,
    draw_device,
    canonical_dims,
    flops,
    algorithmic_bytes,
    ELEM_SIZE,
)
