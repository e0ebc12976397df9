"""MI355X-native quantized Adam step of STQuant: thin Python binding over the C-ABI library.

Every step of the path runs in the HIP kernels of libstq.so; this package only marshals
arguments.  PyTorch is used by callers for device memory and streams.
"""
from .binding import (  # noqa: F401
    STQ_FLAG_STATS, STQ_FLAG_STATS_GRAD, STQ_DECIDE_R_ALG1, STQ_DECIDE_NO_DUAL, STQ_DECIDE_NO_TEMPORAL, STQ_DECIDE_NO_SPATIAL,
    StqError, Context, Engine, Bits, HParams, LayerStats, DecideState,
    load_library, library_path, state_bytes, table, decide, decide_due, strerror,
)

__all__ = ["STQ_FLAG_STATS", "STQ_FLAG_STATS_GRAD", "STQ_DECIDE_R_ALG1", "STQ_DECIDE_NO_DUAL", "STQ_DECIDE_NO_TEMPORAL",
           "STQ_DECIDE_NO_SPATIAL", "decide_due", "StqError", "Context", "Engine", "Bits", "HParams", "LayerStats",
           "DecideState", "load_library", "library_path", "state_bytes", "table", "decide", "strerror"]
