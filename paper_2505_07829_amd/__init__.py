"""MI355X-native fused RMSNorm->FFN-SwiGLU and LayerNorm->matmul and attention (Blockbuster, Examples 3, 2 and 1)."""
from .binding import (  # noqa: F401
    BBError, OP_FFN, OP_FFN_UNFUSED, OP_LN, OP_LN_UNFUSED, VARIANT_AUTO, VARIANT_SNAPSHOT1,
    VARIANT_PRESCALE, VARIANT_NEST, VARIANT_STREAM, VARIANT_UNFUSED, bb_attention, bb_attention_workspace_bytes, bb_layernorm_matmul_tune, bb_rmsnorm_swiglu_ffn_residual, bb_rmsnorm_swiglu_ffn_tune,
    bb_tune_clear, bb_tuned_variant, bb_calib_copy, bb_calib_mfma, bb_calib_mfma_data, bb_calib_read, bb_get_variant,
    bb_last_hip_error, bb_layernorm_matmul, bb_layernorm_matmul_t, bb_rmsnorm_swiglu_ffn_t, bb_profile_enable, bb_profile_last, bb_profile_history, bb_check_fault, bb_debug_inject_fault, bb_debug_set_spin_limit, BB_ERR_TIMEOUT, BB_ERR_WORKSPACE, BB_ERR_VARIANT, BB_ERR_INIT, STATIC_SCRATCH_BYTES, bb_init, bb_rmsnorm_swiglu_ffn_static, bb_rmsnorm_swiglu_ffn, bb_set_variant,
    bb_set_workspace, bb_shutdown, bb_version, bb_workspace_bytes, load, status_string,
)
