"""MI355X-native AMDP pipeline-stage library: thin Python binding over the
C ABI declared in include/amdp.h. Everything numerical runs in the HIP
kernels of libamdp.so; this package only marshals arguments. PyTorch is used
by callers for device memory and streams, never for arithmetic."""
from .binding import (  # noqa: F401
    AmdpError, lib, lib_path, build,
    amdp_event_t, amdp_sched_params_t, amdp_sched_stats_t, amdp_stage_config_t,
    amdp_param_desc_t, amdp_adam_t, amdp_profile_entry_t, make_config,
    amdp_sim_params_t, amdp_sim_op_t, amdp_sim_result_t, amdp_system_simulate, amdp_tie_embedding_grads, amdp_device_copy,
    amdp_layernorm_forward, amdp_layernorm_backward, amdp_column_sums_workspace_bytes, amdp_column_sums,
    amdp_column_sums_static_max_cols, amdp_column_sums_static, E_TOO_LARGE,
    amdp_strerror, amdp_schedule_generate, amdp_schedule_stats, amdp_stage_map, amdp_schedule_preset,
    PRESET_AMDP, PRESET_PIPEDREAM, PRESET_PIPEDREAM_2BW, PRESET_SYNC_1F1B, U_FLUSH,
    amdp_stage_n_params, amdp_stage_workspace_bytes, amdp_stage_param_layout,
    Stage,
    EV_F, EV_B, EV_A, EV_U, U_NEXT_BUBBLE, U_EAGER, BWD_STASHED, BWD_CURRENT,
    FLAG_LAST_USE, FLAG_PARTIAL_WINDOW, BLOCK_GPT, BLOCK_BERT, FP32, BF16, ATTN_AUTO, ATTN_UNFUSED,
    OPT_GEMM_TILE, OPT_GEMM_TRANSPOSING_READS, OPT_GEMM_DIRECT_TO_LDS, OPT_LAZY_JOIN, OPT_SPLIT_K_MIN_TOKENS, OPT_SPLIT_MAIN_MIN_K, OPT_LEAF_FORKS,
    E_INVAL, E_MB_STATE, E_NO_SLOT, E_VERSION, E_STASH_FULL, E_HIP, E_CAPACITY,
)
