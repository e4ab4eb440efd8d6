"""Fused RMSNorm + linear for AMD MI355X (gfx950): Python face of the C-ABI library.

The computation is the case study of the Mirage superoptimizer paper: Eq. 1 (RMSNorm)
followed by a MatMul, executed as one kernel in the reordered form of Fig. 2b.
"""
from .binding import (  # noqa: F401
    LIB_PATH, VARIANTS, RmsnlError, lib, matmul, rl_autotune, rl_autotune_rotating, rl_autotune_clear, rl_autotune_get, rl_ff_rmsnorm_linear, rl_ntrans, rl_qknorm_attention, rl_get_variant, rl_last_error, rl_last_variant,
    rl_probe_copy, rl_probe_mfma, rl_probe_read, rl_set_trace, rl_set_tuning, rl_set_variant, rl_set_workspace, rl_interleave_gate_up, rl_tile_order, rl_trace_slots,
    rl_version, rl_workspace_bytes, rl_workspace_default_bytes, rmsnorm, rmsnorm_gated_mlp, rmsnorm_gated_mlp_interleaved, rmsnorm_linear, rmsnorm_linear_noalloc, rl_noalloc_scratch_bytes, rmsnorm_linear_ex, rmsnorm_gated_mlp_ex, rl_last_launch,
    rl_probe_read_strips, rl_probe_read_flat, LaunchOpts, rl_ff_pairs, rl_autotune_qknorm,
    silu_mul,
)
