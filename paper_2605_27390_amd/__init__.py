"""MI355X-native active-vocabulary LM head (EvoSpec, Eq. 1 restricted to V_t) -- Python binding.

The package is a thin ctypes layer over `libevospec.so` (hand-written HIP for gfx950 behind the
C ABI of `include/evospec.h`).  It has no CPU fallback: importing it without the built library
raises.  Build the library with `python -m paper_2605_27390_amd.build` or `__graft_entry__.build()`.
"""
from .binding import (  # noqa: F401
    EvospecError,
    K_MAX,
    M_TILE,
    STATUS,
    ROW_MAJOR,
    PACKED,
    PackedMatrix,
    matrix_bytes,
    lib,
    lib_path,
    version,
    status_string,
    workspace_bytes,
    workspace_bytes_segmented,
    active_gather,
    active_lmhead_topk,
    active_lmhead_topk_static,
    STATIC_SCRATCH_BYTES,
    active_lmhead_topk_then_update,
    active_lmhead_partials,
    active_lmhead_merge,
    active_lmhead_topk_segmented,
    validate_ids,
    kl_gate,
    kl_gate_workspace_bytes,
)
from .arc import ArcManager, form_candidates, path_a_event, path_a_workspace_bytes  # noqa: F401,E402
