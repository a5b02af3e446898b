"""MI355X (gfx950) SpecKV hot path: scoring, selection and KV-cache compaction.

Thin ctypes binding over ``libspeckv.so`` (hand-written HIP, C ABI declared in
``include/speckv.h``).  PyTorch only supplies device memory and the current
stream; every step of the path runs in the library's kernels.  There is no CPU
fallback: calling any function without the built library raises.
"""
from .binding import (  # noqa: F401
    SpecKVError,
    SpecKVParams,
    library_path,
    load_library,
    n_keep,
    plan_info,
    probe_ceiling,
    select_workspace_bytes,
    specpc_compress_prompt,
    specpc_compress_workspace_bytes,
    specpc_select_tokens,
    specpc_select_tokens_events,
    SPECPC_STAGE_NAMES,
    specpc_workspace_bytes,
    ada_workspace_bytes,
    speckv_compact,
    speckv_compact_ada,
    speckv_compress_ada,
    speckv_select_ada,
    speckv_compress,
    speckv_compress_events,
    speckv_compress_lse,
    speckv_compress_static,
    STATIC_SCRATCH_BYTES,
    speckv_score_lse,
    N_STAGE_EVENTS,
    STAGE_NAMES,
    speckv_score,
    speckv_select,
    total_keep,
    workspace_bytes,
)
