"""MI355X-native trimmed-vocabulary draft LM head: Python binding of the C-ABI library libvt.so."""
from .binding import (  # noqa: F401
    EXPORTS, LIB_PATH, VT_MAX_K, VT_OK, VtError, Workspace, lib, status_str, vt_build_subset,
    vt_check_token_ids_host, vt_draft_head, vt_draft_head_regime, vt_draft_head_workspace_bytes,
    vt_draft_head_workspace_init, new_workspace, vt_draft_head_static, VT_STATIC_SCRATCH_BYTES, VT_Q_FP8_E4M3, VT_Q_MXFP4,
    vt_build_subset_q, vt_draft_head_q, vt_draft_head_q_workspace_bytes,
    vt_feature_fusion, vt_draft_head_fused, vt_draft_head_fused_workspace_bytes, vt_select_vocab, vt_select_vocab_workspace_bytes,
    vt_build_t2d, vt_coverage, vt_coverage_workspace_bytes,
    vt_version,
)
