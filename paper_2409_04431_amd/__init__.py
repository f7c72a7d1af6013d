"""MI355X-native fused sigmoid attention (forward + recompute backward) behind a C ABI.

`binding` holds thin ctypes wrappers with the same names as the C entry points;
`workloads` holds the seeded synthetic input recipes.  Importing this package does not
load the HIP library; the first call does, and fails loudly if it is missing.
"""
from .binding import (  # noqa: F401
    SattnError,
    library_path,
    load_library,
    sigmoid_attn_bwd,
    sigmoid_attn_bwd_bias_grad,
    sigmoid_attn_bwd_compiler_scheduled,
    sigmoid_attn_bwd_dkdv,
    sigmoid_attn_bwd_dq,
    sigmoid_attn_bwd_workspace_bytes,
    sigmoid_attn_cross_bwd,
    sigmoid_attn_cross_fwd,
    sigmoid_attn_fwd,
    sigmoid_attn_fwd_compiler_scheduled,
    sigmoid_attn_mqa_bwd,
    sigmoid_attn_mqa_fwd,
    sigmoid_attn_varlen_bwd,
    sigmoid_attn_varlen_bwd_bias_grad,
    sigmoid_attn_varlen_fwd,
    softmax_attn_bwd,
    softmax_attn_bwd_noalloc,
    softmax_attn_bwd_noalloc_max_rows,
    softmax_attn_bwd_workspace_bytes,
    softmax_attn_fwd,
    softmax_attn_fwd_compiler_scheduled,
    sattn_device_info,
    sattn_fwd_v_slots,
    sattn_fwd_waves,
    sattn_headconcat_norm_bwd,
    sattn_headconcat_norm_fwd,
    sattn_mfma_bf16_probe,
    sattn_set_clock_probe,
    sattn_set_fwd_v_slots,
    sattn_set_fwd_waves,
    sattn_strerror,
    sattn_version,
    sattn_wall_clock_khz,
)
