"""MI355X-native local training step with partial parameter updates (C-ABI library + thin binding)."""
from .binding import (PP_BF16, PP_F32, PPConfig, PPMask, PPAdamW, PPOuter, PPError, LocalStepModel, lib_path, load_library,
                      pp_query_bytes, pp_init_model, pp_set_tensor, pp_get_tensor, pp_set_trainable_mask, pp_local_step,
                      pp_set_jacobian_slices, pp_outer_delta, pp_outer_delta_group, pp_synth_delta_sum, pp_get_counters, pp_get_launch_counts, pp_get_gemm_timing, pp_set_option, pp_last_error, pp_free,
                      pp_op_gemm_nt, pp_op_gemm_tn, pp_op_gemm_nt_splitk_static, PP_STATIC_SCRATCH_FLOATS, pp_op_attention_fwd, pp_op_attention_bwd)
