"""MI355X-native SmoothRot W4A4 linear layer: Python binding of libsmoothrot.so."""
from .binding import (  # noqa: F401
    LIB_PATH, SR_ERR_ALIGN, SR_ERR_ARG, SR_ERR_DEVICE, SR_ERR_NULL, SR_ERR_SHAPE, SR_ERR_UNSUPPORTED_K,
    SR_ERR_WORKSPACE, SR_F16, SR_I32, SR_OK, SmoothRotError, raw, sr_calib_absmax, sr_fold_smooth_rotate_quant,
    sr_fold_workspace_bytes, sr_fwht_quant_act, sr_gemm_workspace_bytes, sr_hadamard_supported, sr_status_str,
    sr_w4a4_gemm, sr_swiglu_fwht_quant_act, sr_fwht_quant_act_heads, sr_fold_smooth_rotate_quant_ex,
    sr_kv_quant_asym, sr_w4a4_linear_decode, sr_f6_tiles_bytes, sr_pack_f6_tiles, sr_w4a4_gemm_f6, sr_w4a4_gemm_f6_warm,
    sr_fwht_quant_act_f6, sr_swiglu_fwht_quant_act_f6, sr_fwht_quant_act_f6_warm, sr_tune_set, sr_tune_get,
    SR_TUNE_AUTO, SR_TUNE_GEMM_TILE, SR_TUNE_GEMM_GRID, SR_TUNE_GEMM_XCDM, SR_TUNE_DECODE_KERNEL, SR_TUNE_FWHT4096,
    SR_TUNE_FWHT_STREAM, SR_TUNE_GEMM_WARM, SR_TUNE_KNOBS, sr_linear_decode_workspace_bytes, sr_noalloc_scratch_bytes, sr_fold_smooth_rotate_quant_noalloc,
    sr_ceiling_hbm_read, sr_ceiling_row_stream, sr_ceiling_mfma_f6, sr_ceiling_mfma_i8, sr_ceiling_valu_f32,
)
