"""MI355X-native Local SGD / Local AdamW with the Quadratic Synchronization Rule.

Everything is computed by the HIP library libqsr.so (see include/qsr.h); this package only
marshals arguments.  There is no CPU fallback: importing works without a GPU (so that the
symbols can be inspected), any compute call without the built library or a gfx950 device fails.
"""
from .binding import (QSRError, Config, Context, average_rows, clip_factors, clip_factors_static,
                      host_schedule, lib, lib_path, validate,
                      workspace_bytes, EXPORTS)

__all__ = ["QSRError", "Config", "Context", "average_rows", "clip_factors", "clip_factors_static", "host_schedule", "lib", "lib_path", "validate",
           "workspace_bytes", "EXPORTS"]
