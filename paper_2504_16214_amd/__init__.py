"""MI355X-native W4A16 mixture-of-experts layer: hand-written HIP kernels (gfx950) behind a
small C ABI (include/moe_w4a16.h), with a thin Python binding of the same names.

PyTorch is used for device memory and streams only; every step of the layer runs in the HIP
library.  There is no CPU fallback: if the library has not been built the binding raises.
"""
from .binding import (  # noqa: F401
    MOE_F16, MOE_BF16, MoEError, library_path, load_library,
    moe_align_capacity, moe_align_by_expert, moe_w4a16_grouped_gemm, moe_silu_mul, moe_combine, moe_combine_masked,
    moe_w4a16_layer_workspace_bytes, moe_w4a16_layer, moe_layer_block_m,
    moe_w4a16_dense_gemm, moe_route_topk, moe_route_align, moe_probe_stream_read, moe_probe_mfma, moe_probe_issue_mix,
    moe_w4a16_routed_layer_workspace_bytes, moe_w4a16_routed_layer,
    moe_repack_qweight, moe_w4a16_layer_prepacked, moe_import_awq,
    fp8_blockwise_gemm_workspace_bytes, fp8_blockwise_gemm, fp8_moe_grouped_gemm, fp8_set_plan_override,
    fp8_probe_mfma, fp8_quantize_rows, fp8_silu_mul_quantize, fp8_moe_layer_workspace_bytes, fp8_moe_layer,
    fp8_set_layer_block_m,
    moe_set_tile_override, moe_set_scale_path, moe_set_tiles_per_workgroup, moe_set_reduction_splits, moe_set_stage_events, moe_last_error,
    moe_set_block_m_override, moe_last_gemm_plan, moe_w4a16_layer_noalloc, moe_layer_block_m_for, moe_set_wide_tiles,
)
