"""PaTH attention hot path for MI355X (gfx950): thin binding over the C-ABI library."""
from .binding import (  # noqa: F401
    PATH_F32, PATH_BF16, PathAttnError, library_path, load_library,
    path_attn_workspace_bytes, path_attn_fwd_workspace_layout, path_attn_fwd, path_attn_fwd_prep, path_attn_fwd_sweep, path_attn_bwd, path_status_str,
    path_attn_last_error, path_decode_workspace_bytes, path_key_prefill, path_decode_step, path_decode_step_static, path_decode_static_scratch_bytes, path_attn_fox_fwd, path_attn_fox_bwd,
    path_attn_train_fwd, path_attn_train_bwd, path_attn_train_fwd_prep, path_attn_train_fwd_sweep,
    PATH_LAYOUT_BHLD, PATH_LAYOUT_BLHD, path_attn_fwd_layout, path_attn_bwd_layout,
    path_attn_varlen_workspace_bytes, path_attn_varlen_fwd, path_attn_varlen_bwd,
    path_gate_prefill, path_decode_step_fox, path_attn_ring_state_bytes, path_attn_ring_regions, path_attn_ring_local, path_attn_ring_hop, path_attn_ring_finish,
    path_attn_train_bwd_stages, path_probe_mfma, path_attn_bwd_workspace_bytes_for_heads, path_attn_bwd_heads_per_pass, PATH_BWD_STAGE_SCAN, PATH_BWD_STAGE_KEYS_NEAR, PATH_BWD_STAGE_KEYS_FAR,
    PATH_BWD_STAGE_DDP, PATH_BWD_STAGE_CHUNK, PATH_BWD_STAGE_ALL,
)
