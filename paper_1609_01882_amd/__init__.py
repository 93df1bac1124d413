"""Polysemous-code search on AMD MI355X: Python face of libpsc.so (HIP, gfx950).

The compute lives in `csrc/` behind the C ABI declared in `include/psc.h`; this package only
marshals arguments (see `binding.py`).
"""
from .binding import (  # noqa: F401
    Index,
    PscError,
    PSC_MAX_K,
    exported_symbols,
    hamming_filter,
    hamming_histogram,
    last_scan_route,
    lib_path,
    scan,
    scan_static,
    scan_workspace_bytes,
    PSC_STATIC_SCRATCH_BYTES,
    set_filter_route,
    threshold_for_rate,
    version,
    workspace_status,
)
