"""MI355X-native core of Group Tree Optimization: thin Python binding over libgto.so.

The binding only marshals arguments (torch tensors -> device pointers, current stream);
every step of the path runs in the HIP kernels of libgto.so.  There is no CPU fallback:
if the library is missing, importing the binding's entry points raises.
"""
from .binding import (  # noqa: F401
    GTO_BF16, GTO_F32, GTO_REWARD_LSE, GTO_REWARD_MAX, GTO_REWARD_MEAN, GTO_REWARD_NODESUM,
    GTO_FLAG_GRAD_ZERO_FILL, GTO_FLAG_TARGET_PRUNE, GTO_PATH_GREEDY, GTO_PATH_MAX_L, GTO_PATH_SAMPLED, GtoError, make_config, lib, lib_path,
    alloc_draft_stats, alloc_target_stats, alloc_pool, alloc_tree, alloc_reward, alloc_ppo,
    gto_version, gto_strerror, gto_workspace_bytes,
    gto_draft_row_stats, gto_target_row_stats, gto_expand_tree, gto_expand_from_stats,
    gto_select_topg, gto_tree_reward, gto_reward_from_stats, gto_group_advantage,
    gto_ppo_surrogate_fwd, gto_ppo_surrogate_bwd, gto_ppo_surrogate_fwd_noalloc, gto_calibration_copy, gto_token_loss_fwd, gto_token_loss_bwd,
    gto_fused_workspace_bytes, gto_fused_draft_row_stats, gto_fused_target_row_stats,
    gto_expand_tree_fused, gto_tree_reward_fused, gto_ppo_surrogate_fwd_fused, gto_ppo_surrogate_bwd_fused,
    gto_fused_dh_workspace_bytes, gto_ppo_surrogate_bwd_fused_dh, gto_fused_token_loss_workspace_bytes,
    gto_token_loss_fwd_fused, gto_token_loss_bwd_fused,
    gto_profile_enable, gto_profile_read, gto_profile_filter,
)
