"""MI355X-native hot path of AgentSAM speculative decoding (one step over a batch of sessions).

The Python layer is a thin ctypes binding over libagentsam.so (see include/agentsam.h); the
library is loaded on first use and there is no fallback when it is missing.
"""
from .binding import (  # noqa: F401
    AgentSamError, FlatSam, Sam, SamBuilder, SamDelta, attn_tuning, agentsched_pick, spec_adaptive_k, spec_choose_k, spec_switch_frontier, overlay_table, sam_append, sam_apply_delta,
    sam_build, sam_delta_export, sam_delta_sizes, sam_reflatten_due, sam_draft, sam_draft_delta, sam_draft_merged, sam_draft_step, sam_flat_sizes, sam_flatten, spec_accept, spec_verify_attn, spec_verify_attn_static, spec_verify_attn_workspace, strerror, BF16, F32,
)
