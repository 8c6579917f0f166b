"""MI355X-native frequency-ranked draft LM head (FR-Spec, Section 3.2).

Thin ctypes binding over ``libfrspec.so`` (see ``include/frspec.h``).  Every step
of the path runs in the HIP kernels; this module only marshals arguments.  There
is no CPU fallback: importing the binding without the built library raises.
"""

from .binding import (  # noqa: F401
    FR_K_MAX,
    FrSpecError,
    Tuning,
    bind_draft_topk,
    fr_beam_expand,
    fr_build_subset,
    fr_build_subset_tiled,
    fr_calib_copy,
    fr_calib_read,
    fr_count_tokens,
    fr_draft_logits,
    fr_draft_step,
    fr_draft_topk,
    fr_draft_topk_multi,
    fr_draft_topk_static,
    fr_draft_topk_tiled,
    fr_full_topk,
    fr_init,
    fr_rank_tokens,
    fr_strerror,
    fr_tiled_bytes,
    fr_tree_select,
    fr_version,
    fr_workspace_bytes,
    fr_workspace_check,
    fr_workspace_init,
    lib,
    lib_path,
    new_workspace,
)
