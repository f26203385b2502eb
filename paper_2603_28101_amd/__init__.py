"""MI355X-native paged-KV trajectory attention (decode + tool-chunk append).

Thin ctypes binding over libheddle.so; every step of the path runs in the
library's HIP kernels.  There is no CPU fallback: if the library is missing the
import of `paper_2603_28101_amd.binding` raises.
"""
from .binding import (  # noqa: F401
    HeddleError,
    Context,
    lib,
    lib_path,
    stream_read,
    placement_dp,
    placement_aggregate,
    interference_table,
    simulate_group,
    E_INVAL,
    E_NOMEM,
    E_HIP,
    E_UNSUPPORTED,
)
