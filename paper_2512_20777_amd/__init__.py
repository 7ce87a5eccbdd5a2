"""MI355X-native batched matrix exponential (Taylor scaling and squaring, arXiv 2512.20777).

The package is a thin binding over a C-ABI shared library of hand-written HIP kernels for gfx950.
Importing it does not load the library; the first call does, and fails loudly if it is missing.
"""
from .binding import (  # noqa: F401
    DTYPE_F32,
    DTYPE_F64,
    NORM_INF,
    NORM_ONE,
    SCHEME_BASELINE,
    SCHEME_PS,
    SCHEME_SASTRE,
    ExpmError,
    expm,
    expm_get_stats,
    expm_lowrank,
    expm_lowrank_select,
    expm_noalloc,
    expm_profile_enable,
    expm_profile_read,
    expm_profile_reset,
    expm_reserve,
    expm_select,
    expm_shutdown,
    expm_status_string,
    expm_workspace_bytes,
    library_path,
    load_library,
)
