"""MI355X-native quantized Adam step of STQuant: thin Python binding over the C-ABI library.

Every step of the path runs in the HIP kernels of libstq.so; this package only marshals
arguments.  PyTorch is used by callers for device memory and streams.
"""
from .binding import (  # noqa: F401
    STQ_FLAG_STATS, STQ_DECIDE_R_ALG1, StqError, Context, Bits, HParams, LayerStats, DecideState,
    load_library, library_path, state_bytes, table, decide, strerror,
)

__all__ = ["STQ_FLAG_STATS", "STQ_DECIDE_R_ALG1", "StqError", "Context", "Bits", "HParams", "LayerStats",
           "DecideState", "load_library", "library_path", "state_bytes", "table", "decide", "strerror"]
