"""MI355X-native OSC dual-path linear layer: thin Python binding of libosc (C ABI).

PyTorch is used for device memory and streams only; every step of the path runs in the
hand-written HIP kernels of ``libosc.so``.  There is no CPU fallback: calling any entry point
without the built library raises.
"""
from .binding import (  # noqa: F401
    OSC_DT_BF16, OSC_DT_F32, OSC_FMT_FP8_E4M3_TOKEN, OSC_FMT_MXFP4_OSC, OSC_FMT_MXFP4_OSC_G64, OSC_FMT_MXFP8, OscError, lib, lib_path,
    osc_act_scale_bytes, osc_unpack_act_scales,
    osc_dual_gemm, osc_fp8_gemm, osc_grouped_dual_gemm, osc_last_error, osc_pack_weight,
    osc_pack_weight_fp8, osc_packed_weight_bytes, osc_packed_weight_fp8_bytes, osc_quantize_act,
    osc_table_to_index, osc_unpack_weight, osc_unpack_weight_fp8, osc_version,
    osc_mxfp8_gemm, osc_pack_weight_mxfp8, osc_packed_weight_mxfp8_bytes, osc_unpack_weight_mxfp8,
    osc_quantize_act_dynamic, osc_rmsnorm_quantize_act, osc_swiglu_quantize_act, osc_tuning_set, osc_tuning_get, OSC_TUNE_GEMM_TILE, OSC_TUNE_GEMM_KERNEL, OSC_TUNE_GROUPED_ONE_TILE, OSC_TUNE_SWIGLU_TABLE, OSC_TUNE_GEMM_KSPLIT, osc_profile_abs_sum, osc_profile_threshold, osc_profile_hist, osc_profile_table, osc_profile_calibrate, osc_profile_calibrate_static, osc_profile_workspace_bytes,
    osc_pack_weight_g, osc_table_to_index_g, OSC_FMT16_E8M0, OSC_FMT16_NVFP4, osc_quantize_act_g16,
    osc_packed_weight_g16_bytes, osc_pack_weight_g16, osc_unpack_weight_g16, osc_dual_gemm_g16, osc_swiglu_quantize_act_fp8)
