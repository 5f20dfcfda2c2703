"""MI355X-native hot path of Representation Shift token pruning (HIP library + thin binding)."""
from .binding import (  # noqa: F401
    RS_BF16, RS_DIST_COS, RS_DIST_L1, RS_DIST_L2, RS_EPI_BIAS, RS_EPI_BIAS_GELU, RS_EPI_BIAS_RES, RS_ERR_DEVICE, RS_ERR_INVALID_ARG,
    RS_ERR_UNSUPPORTED, RS_ERR_WORKSPACE_TOO_SMALL, RS_F32, RS_OK, RS_SHIFT_ATTN, RS_SHIFT_BLOCK, RS_SHIFT_MLP,
    RS_SHIFT_MLP_NORMED, RS_SHIFT_MLP_STREAM, RsBlockCfg,
    RsBlockWeights, RsError, dtype_code, lib, make_cfg, make_weights, rs_attention_fwd, rs_attention_map_fwd, rs_attention_map_size, rs_attention_map_workspace_size,
    rs_block_fwd, rs_block_fwd_chained, rs_block_fwd_static, rs_build_info, rs_tune_gemm_variant, rs_block_static_scratch_size, rs_block_workspace_size, rs_grid_line_prune, rs_grid_token_prune, rs_linear_fwd, rs_pack_linear, rs_last_error, rs_pack_weights,
    rs_packed_weights_size, rs_profile_enable, rs_profile_read, rs_shift_topk, rs_shift_topk_workspace_size, rs_version)
from .runner import EncoderStack  # noqa: F401
from .schedule import keep_counts, block_flops, forward_flops  # noqa: F401
