"""Soft-DTW forward / log-space backward / barycenter step on MI355X (gfx950).

The arithmetic runs in hand-written HIP kernels behind the C-ABI declared in
``include/sdtw.h``; this package is the thin Python binding of the same names.
Importing the package does not load the library; the first call does, and it raises if
the library has not been built.
"""
from .binding import (  # noqa: F401
    FLAG_DENSE_E,
    FLAG_MIN_MEMORY,
    FLAG_VALUE_ONLY,
    FUSED,
    UNFUSED,
    SdtwError,
    Workspace,
    library_path,
    load_library,
    sdtw_backward,
    sdtw_backward_half,
    sdtw_backward_ragged,
    sdtw_barycenter_step,
    sdtw_barycenter_workspace_bytes,
    sdtw_forward,
    sdtw_forward_half,
    sdtw_forward_ragged,
    sdtw_normalized_backward,
    sdtw_normalized_forward,
    sdtw_normalized_workspace_bytes,
    sdtw_status_string,
    sdtw_version,
    sdtw_workspace_bytes,
)
