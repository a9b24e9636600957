"""libonebitlamb: the 1-bit LAMB compression-stage optimizer step as HIP kernels for MI355X.

The package is a thin ctypes binding over the C ABI declared in include/onebitlamb.h; every step
of the path runs in the library's kernels.  There is no CPU fallback: loading fails loudly when
the shared library has not been built (`python -m paper_2104_06069_amd.build`).
"""
from .binding import (  # noqa: F401
    OB_OK, OB_ERR_NULL, OB_ERR_ARG, OB_ERR_ALIGN, OB_ERR_STATE, OB_ERR_HIP, ObLambConfig, ObLambError, ObLambState, lib, lib_path,
    ob_lamb_chunk_len, ob_lamb_compress_local, ob_lamb_create, ob_lamb_decompress_apply,
    ob_lamb_destroy, ob_lamb_freeze, ob_lamb_layer_ratios, ob_lamb_num_params, ob_lamb_padded_len,
    ob_lamb_padded_len_for, ob_lamb_profile_enable, ob_lamb_profile_read, ob_lamb_server_reduce,
    ob_lamb_status_string, ob_lamb_warmup_step, make_state, ob_lamb_check_device_status,
    ob_lamb_uses_single_pass, ob_lamb_server_single_pass, ob_lamb_plan_split, ob_lamb_plan_big_tiles, ob_lamb_momentum_dense, ob_lamb_momentum_scale, ob_lamb_ratios_apply, ob_lamb_fused_layers, ob_lamb_fused_params,
    OB_F32, OB_F16, OB_BF16, ob_lamb_warmup_step_lp, ob_lamb_compress_local_lp,
    ob_lamb_decompress_apply_lp, ob_lamb_ratios_apply_lp,
    ob_lamb_warmup_fused_layers, ob_lamb_warmup_fused_params,
    OB_CFG_TWO_PASS_COMPRESS, OB_CFG_NO_FUSED_APPLY, OB_CFG_TWO_PASS_WARMUP, OB_CFG_NO_BARRIERS, OB_SPIN_NONE,
    ob_lamb_server_reduce_static, ob_lamb_static_max_chunk_len, ob_lamb_diag_copy, ob_lamb_workspace_bytes, ob_lamb_error_dense, ob_lamb_server_error_dense,
    OB_VF_MAX_OLD, ObLambVfHistory, make_vf_history, ob_lamb_ratios_apply_hist, ob_lamb_ratios_apply_hist_lp, ob_lamb_variance_dense, ob_lamb_big_tile_params,
)
