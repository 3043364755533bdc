"""MI355X-native mixed paged attention (the GPU hot path of a Convertible Decoder iteration).

Thin ctypes binding over libtokenscale.so; every step of the pass runs in the library's HIP
kernels.  PyTorch is used by callers only for device memory and streams.
"""
from .binding import (Context, Desc, PlanInfo, Velocity, TokenScaleError, cache_bytes, check_desc,
                      library_path, load_library, plan_decode_items, plan_describe, plan_export, DTYPES, calib_copy, calib_read, calib_mfma)

from . import policy

__all__ = ["policy", "Context", "Desc", "PlanInfo", "Velocity", "TokenScaleError", "cache_bytes", "check_desc",
           "library_path", "load_library", "plan_decode_items", "plan_describe", "plan_export", "DTYPES", "calib_copy", "calib_read", "calib_mfma"]
