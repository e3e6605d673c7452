"""RACE Attention (arXiv 2510.04008) forward/backward for MI355X: a C-ABI HIP library plus this binding."""
from .binding import (  # noqa: F401
    RACE_BF16, RACE_ERR_HIP, RACE_ERR_INVALID_ARG, RACE_ERR_NOT_READY, RACE_ERR_UNSUPPORTED, RACE_ERR_WORKSPACE, RACE_F32, RACE_OK,
    RaceAttnDesc, RaceAttnError, lib, make_desc, race_attn_bwd, race_attn_bwd_beta, race_attn_bwd_saved, race_attn_debug_buckets, race_attn_debug_hash,
    race_attn_expand_projection, race_attn_fwd, race_attn_fwd_static, race_attn_state_bytes, race_attn_state_init, race_attn_step, race_attn_step_workspace_bytes, race_attn_calibration_copy, race_attn_calibration_mfma, race_attn_profile_enable, race_attn_profile_read, race_attn_kernel_family, race_attn_segment_tokens, race_attn_workspace_bytes,
)
