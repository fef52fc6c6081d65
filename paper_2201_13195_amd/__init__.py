"""RMM linear layer (arXiv 2201.13195, Algorithm 1) for AMD MI355X.

The arithmetic lives in librmm.so (hand-written HIP for gfx950, C ABI in
include/rmm.h).  This package only marshals arguments: PyTorch tensors supply
device memory and the current stream.
"""
from .binding import (  # noqa: F401
    GAUSSIAN, RADEMACHER, SORS, RmmError, lib_path, load_library, rmm_backward, rmm_debug_philox,
    rmm_debug_sketch_tile, rmm_forward, rmm_probe_mfma, rmm_probe_read, rmm_uses_paired_launch, rmm_sketch, rmm_sketch_static, rmm_status_string, rmm_variance_stats, rmm_version, rmm_workspace_bytes,
    STATIC_SCRATCH_BYTES, VARIANCE_FIELDS,
)
from .layer import RMMLinear, RMMLinearFunction  # noqa: F401,E402
