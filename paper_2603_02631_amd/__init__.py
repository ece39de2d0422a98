"""MI355X-native token-importance pass for cross-family speculative prefill.

The package is a thin ctypes binding over ``libsp_amd.so`` (hand-written HIP
kernels for gfx950 behind the C ABI declared in ``include/sp.h``). Importing
the package does not load the library; the first call does, and it raises if
the library has not been built.
"""
from .binding import (  # noqa: F401
    SP_LAYER_MAX,
    SP_LAYER_MEAN,
    SpError,
    ScoreDesc,
    library_path,
    load_library,
    sp_assemble,
    sp_assemble_workspace,
    sp_debug_fused_giveup,
    sp_hbm_read_probe,
    sp_keep_count,
    sp_last_error,
    sp_project,
    sp_project_batch,
    sp_score,
    sp_score_batch,
    sp_score_batch_is_fused,
    sp_score_fp8,
    sp_score_fp8_is_fused,
    sp_score_look,
    sp_score_paged,
    sp_score_is_fused,
    sp_score_workspace,
    sp_select,
    sp_select_batch,
    sp_select_batch_workspace,
    sp_select_budget,
    sp_select_static,
    sp_select_budget_workspace,
    sp_select_workspace,
    sp_version,
)
