"""MI355X-native LinFusion token mixer: normalized non-causal linear attention (gfx950 HIP).

The compute path is the C-ABI shared library built from csrc/ (see include/linfusion.h);
this package is only the argument-marshalling binding plus the seeded synthetic workloads.
Nothing here falls back to a CPU or PyTorch implementation: importing the binding without a
built library raises.
"""
from .binding import (  # noqa: F401
    DTYPE_BF16, DTYPE_F16, DTYPE_F32, FLAG_FORCE_FUSED, FLAG_FORCE_SOLO, FLAG_FORCE_SPLIT, FLAG_NONE, FLAG_UNNORMALIZED,
    PHI_ELU_PLUS_ONE, PHI_IDENTITY, PHI_RELU, LinFusionError, library, library_path,
    linfusion_attn_bwd, linfusion_attn_bwd_strided, linfusion_attn_bwd_workspace_bytes, linfusion_attn_fwd, linfusion_attn_fwd_mlp, linfusion_attn_fwd_mlp_strided, linfusion_attn_mlp_workspace_bytes, linfusion_attn_fwd_qv, linfusion_attn_qv_workspace_bytes, linfusion_attn_fwd_bf16, linfusion_attn_fwd_ex, linfusion_attn_fwd_ex_bound, linfusion_attn_fwd_f16,
    linfusion_attn_fwd_f32, linfusion_attn_fwd_profile, linfusion_attn_fwd_static, linfusion_attn_static_scratch_bytes, linfusion_init, linfusion_attn_fwd_strided, linfusion_attn_last_error, linfusion_attn_plan, linfusion_attn_apply_kernel, linfusion_attn_state, linfusion_attn_workspace_bytes, linfusion_attn_workspace_state_offset,
    linfusion_hbm_probe, linfusion_launch_probe, linfusion_release, linfusion_set_tuning, linfusion_status_string, linfusion_version,
)
