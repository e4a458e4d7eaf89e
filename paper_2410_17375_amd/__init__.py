"""MI355X-native verify pass of asynchronous speculative decoding (AMUSD).

The work is done by hand-written HIP kernels for gfx950 in libamusd.so (C ABI
in include/amusd.h); this package is the thin ctypes binding with the same
names.  There is no CPU fallback: importing the binding without the built
library raises.
"""
from .binding import (AmusdError, Config, Model, LoopStats, generate_async, generate_sync,
                      generate_greedy, calibration_copy, calibration_chain, library_path, lib, TENSOR_IDS,
                      OPT_KEEP_LOGITS, OPT_TIME_STAGE, STAGES, DTYPE_FP32, DTYPE_BF16, MAX_K)

__all__ = ["AmusdError", "Config", "Model", "LoopStats", "generate_async", "generate_sync",
           "generate_greedy", "calibration_copy", "calibration_chain", "library_path", "lib", "TENSOR_IDS", "OPT_KEEP_LOGITS",
           "OPT_TIME_STAGE", "STAGES", "DTYPE_FP32", "DTYPE_BF16", "MAX_K"]
