"""W6A16 FP6 (E3M2, 4+2 planes) linear layer for MI355X: Python binding of the HIP library."""
from .binding import (  # noqa: F401
    FP6_TILE, FP6_VARIANT_AUTO, FP6_VARIANT_DECODE, FP6_VARIANT_GEMM, Fp6Error,
    fp6_dequantize, fp6_layout_version, fp6_linear, fp6_linear_variant,
    fp6_linear_variant_workspace_bytes, fp6_linear_workspace_bytes, fp6_packed_sizes,
    fp6_quantize_pack, fp6_status_string, fp6_unpack_codes, new_workspace,
    fp6_dequantize_fgq, fp6_linear_fgq, fp6_linear_fgq_workspace_bytes, fp6_quantize_pack_fgq,
    fp6_dequantize_v2, fp6_linear_v2, fp6_linear_v2_bf16, fp6_probe_mfma, fp6_probe_read, fp6_linear_v2_workspace_bytes, fp6_quantize_pack_v2, fp6_unpack_codes_v2,
    fp6_linear_plan, plan_text, fp6_linear_group, fp6_linear_group_workspace_bytes, FP6_GROUP_MAX, fp6_linear_static, FP6_STATIC_SCRATCH_BYTES, FP6_FORMAT_E3M2, FP6_FORMAT_E3M1, FP6_FORMAT_E3M2_V2, FP6_FORMAT_E3M2_V2_BF16,
    fp5_dequantize, fp5_linear, fp5_linear_workspace_bytes, fp5_packed_sizes, fp5_quantize_pack, fp5_unpack_codes,
)
