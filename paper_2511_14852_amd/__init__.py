"""Fused Chebyshev-KAN layer (forward + backward) for AMD MI355X.

The compute lives in libchebykan.so (hand-written HIP for gfx950, C ABI in
include/chebykan.h); this package is the thin ctypes binding plus the seeded
synthetic workloads used to test and time it.
"""
from . import workloads  # noqa: F401
from .binding import (  # noqa: F401
    CHEBYKAN_PASS_BACKWARD, CHEBYKAN_PASS_FORWARD, ChebykanError, alloc_workspace, chebykan_backward,
    chebykan_forward, chebykan_set_kernel_family, chebykan_status_string, chebykan_version,
    chebykan_workspace_bytes, library_path, load,
)
