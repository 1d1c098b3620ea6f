"""MI355X-native Lightning Attention (arXiv 2307.14995): a C-ABI library of gfx950 HIP
kernels plus this thin binding.  Importing the package loads nothing; the shared
library is opened on first use and its absence is an error (there is no fallback).
"""
from .binding import (  # noqa: F401
    LtnError,
    library_path,
    load_library,
    ltn_attn_bwd,
    ltn_attn_check_decay,
    ltn_attn_decode_step,
    ltn_attn_decode_steps,
    ltn_attn_fwd,
    ltn_attn_fwd_gated,
    ltn_attn_fwd_tiled,
    ltn_gate_bwd,
    ltn_gate_fwd,
    ltn_attn_pick_block,
    ltn_attn_workspace_bytes,
    ltn_status_str,
    ltn_prologue_fwd,
    ltn_prologue_bwd,
    ltn_prologue_workspace_bytes,
    ltn_attn_fwd_dkdv,
    ltn_attn_bwd_dkdv,
    ltn_attn_decode_steps_dkdv,
    ltn_attn_query_plan,
    ltn_attn_set_debug_plan,
    ltn_attn_fwd_static,
    ltn_attn_bwd_tiled,
    ltn_probe_stream_read,
    ltn_attn_workspace_bytes_dkdv,
)

__all__ = [
    "LtnError", "library_path", "load_library", "ltn_attn_fwd", "ltn_attn_fwd_gated", "ltn_attn_fwd_tiled", "ltn_gate_fwd", "ltn_gate_bwd", "ltn_attn_bwd",
    "ltn_attn_decode_step", "ltn_attn_decode_steps", "ltn_attn_pick_block", "ltn_attn_workspace_bytes",
    "ltn_attn_check_decay", "ltn_status_str", "ltn_prologue_fwd", "ltn_prologue_bwd", "ltn_prologue_workspace_bytes",
    "ltn_attn_fwd_dkdv", "ltn_attn_bwd_dkdv", "ltn_attn_decode_steps_dkdv",
    "ltn_attn_query_plan", "ltn_attn_set_debug_plan", "ltn_attn_fwd_static", "ltn_attn_bwd_tiled", "ltn_probe_stream_read", "ltn_attn_workspace_bytes_dkdv",
]
