"""MI355X-native hot path of HTS-RL: batched acting with seeded sampling, returns/GAE, A2C/PPO learner step.

Thin ctypes binding over libhts.so (hand-written HIP for gfx950, C ABI in include/hts.h).  Every step runs in
the library's kernels; this package only marshals torch device pointers.  There is no CPU fallback: importing
`binding` raises if the library has not been built (python -m paper_2012_09849_amd.build).
"""
from .binding import (ALGO_A2C, ALGO_A2C_TIS, ALGO_PPO, OPT_ADAM, OPT_RMSPROP, PRECISION_BF16, PRECISION_FP32, Context, CuRangeStream, HParams, HtsError, OptState,
                      hts_adam_apply_static, load_library, param_count)

__all__ = ["Context", "CuRangeStream", "HParams", "OptState", "HtsError", "param_count", "load_library", "hts_adam_apply_static", "PRECISION_FP32",
           "PRECISION_BF16", "ALGO_A2C", "ALGO_PPO", "ALGO_A2C_TIS", "OPT_ADAM", "OPT_RMSPROP"]
