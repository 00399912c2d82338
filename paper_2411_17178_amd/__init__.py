"""MI355X-native multi-diagonal windowed attention (LiteVAR, arXiv 2411.17178).

Thin Python binding over the C-ABI library built from csrc/ (see include/litevar.h).
PyTorch is used for device memory and streams only; every step of the path runs in
the library's HIP kernels.  There is no CPU fallback: a missing library raises.
"""
from .binding import (  # noqa: F401
    LitevarError, Plan, lib_path, litevar_mask_build, litevar_mask_export_csr,
    litevar_mask_export_dense, litevar_mask_plan_bytes, litevar_mask_plan_stats, litevar_peak_copy,
    litevar_peak_mfma_bf16, litevar_peak_read, litevar_plan_check, litevar_qkv8_dequantize,
    litevar_qkv8_quantize, litevar_scale_offsets, litevar_windowed_attn_qkv8_fwd,
    litevar_windowed_attn_qkv8_workspace_bytes,
    litevar_window_calibrate, litevar_window_calibrate_band, litevar_window_calibrate_static, litevar_window_table_export,
    litevar_windowed_attn_fwd, load_library, use_library,
)
