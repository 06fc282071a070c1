"""ScaleKV hot path for AMD MI355X: thin Python binding over libscalekv.so.

Argument marshalling only -- every step of the path (score, select, compact,
attend, and the fused step) runs in the HIP kernels behind the C ABI declared
in include/scalekv.h.  PyTorch is used for device memory and streams, nothing
else.  There is no CPU fallback: if the library cannot be loaded, importing
the binding's functions raises.
"""
from .binding import (  # noqa: F401
    ScaleKVError,
    Shape,
    lib,
    lib_path,
    version,
    workspace_bytes,
    score,
    select,
    compact,
    attend,
    step,
    step_static,
    PreparedStep,
    PreparedAppendFirst,
    step_stage_events,
    window_centroids,
    select_window,
    step_append_first,
    asi,
    drafter_set,
    allocate_budgets,
    pyramid_budgets,
    policy_table,
    select_positional,
    MAX_WINDOW,
    MAX_ASI_SAMPLES,
    MAX_POOL,
    STATIC_SCRATCH_BYTES,
    EXPORTED_SYMBOLS,
)
