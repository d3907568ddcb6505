"""MI355X-native W4A16 / bf16 linear layer of a Dynamic-Mixed-Precision-Routing step.

The product is ``libdmr_qlinear.so`` (hand-written gfx950 kernels behind the C ABI declared in
``include/dmr_qlinear.h``); this package holds its sources, its build step, a thin binding with
the same names, and the seeded input generators.
"""
from .binding import (DMR_FMT_BF16, DMR_FMT_W3_G128, DMR_FMT_W4_G128, DMR_FMT_W4_PER_CHANNEL, DMR_OUT_BF16, DMR_OUT_FP32, DMR_PRO_NONE, DMR_PRO_RMSNORM, DMR_PRO_SWIGLU, DmrError, Layer,
                      dmr_glue_rmsnorm, dmr_glue_swiglu, dmr_probe_empty_launch, dmr_probe_hbm_read, dmr_qlinear_bf16_forward,
                      dmr_qlinear_bf16_forward_fused, dmr_qlinear_bf16_workspace_bytes, dmr_qlinear_create,
                      dmr_qlinear_create_per_channel, dmr_qlinear_dequantize, dmr_qlinear_per_channel_storage_bytes, dmr_qlinear_destroy,
                      dmr_qlinear_forward, dmr_qlinear_forward_fused, dmr_qlinear_forward_static, dmr_qlinear_kernel_path, dmr_qlinear_quantize,
                      dmr_qlinear_quantize_w3, dmr_qlinear_storage_bytes, dmr_qlinear_w3_create,
                      dmr_qlinear_w3_storage_bytes, dmr_qlinear_w3_workspace_bytes,
                      dmr_qlinear_workspace_bytes)

__all__ = [
    "DMR_FMT_BF16", "DMR_FMT_W3_G128", "DMR_FMT_W4_G128", "DMR_FMT_W4_PER_CHANNEL", "DMR_OUT_BF16", "DMR_OUT_FP32", "DMR_PRO_NONE", "DMR_PRO_RMSNORM", "DMR_PRO_SWIGLU", "DmrError", "Layer",
    "dmr_glue_rmsnorm", "dmr_glue_swiglu", "dmr_probe_empty_launch", "dmr_probe_hbm_read", "dmr_qlinear_bf16_forward",
    "dmr_qlinear_bf16_forward_fused", "dmr_qlinear_bf16_workspace_bytes", "dmr_qlinear_create",
    "dmr_qlinear_create_per_channel", "dmr_qlinear_dequantize", "dmr_qlinear_per_channel_storage_bytes", "dmr_qlinear_destroy", "dmr_qlinear_forward",
    "dmr_qlinear_forward_fused", "dmr_qlinear_forward_static", "dmr_qlinear_kernel_path", "dmr_qlinear_quantize", "dmr_qlinear_quantize_w3", "dmr_qlinear_storage_bytes",
    "dmr_qlinear_w3_create", "dmr_qlinear_w3_storage_bytes", "dmr_qlinear_w3_workspace_bytes",
    "dmr_qlinear_workspace_bytes",
]
