"""MI355X-native Concurrent ALS (fused multi-model MTTKRP + batched per-model updates).

The compute lives in the HIP library behind include/cals.h; this package is a thin ctypes binding
with the same call names.  Importing the package does not load the library; the first call does and
fails loudly if it has not been built (python -m paper_2010_04678_amd.build).
"""
from .binding import (  # noqa: F401
    CalsError,
    Context,
    Result,
    Stats,
    cp_cals,
    suggest_max_total_rank,
    suggest_two_step,
    library_path,
    load_library,
    FLAG_NONNEG,
    FLAG_LINESEARCH,
    CTX_REUSE,
    CTX_TIMING,
    RUNNING,
    CONVERGED,
    MAX_ITERS,
    NUMERICAL,
    MAX_RANK,
    MAX_MODES,
)
