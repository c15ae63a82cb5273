"""PODS hot path on AMD MI355X: thin Python binding over the C ABI in include/pods.h.

The functions here only marshal arguments (device pointers, sizes, the current HIP stream) into
libpods_hip.so; every step of the path runs in the library's HIP kernels.  PyTorch is used for
device memory and streams only.  There is no CPU fallback: if the library is missing or a call
fails, an exception is raised.
"""
from .binding import (PodsError, load, library_path, pods_select, pods_downsample, pods_advantage,
                      pods_advantage_before, pods_gather_rows, pods_downsample_gather, grpo_token_loss_fwd_bwd, grpo_token_loss_fwd_bwd_static, grpo_token_loss_report, pods_check_rewards, grpo_token_loss_static_workspace_bytes, grpo_token_loss_workspace_bytes,
                      grpo_token_loss_workspace_min_bytes, grpo_token_loss_workspace_used_bytes, pods_last_error, pods_profile_enable,
                      pods_profile_read, pods_profile_mfma_only, PODS_F32, PODS_BF16, PODS_RULE_MAXVAR, PODS_RULE_MAXR,
                      PODS_RULE_PERC, PODS_RULE_RAND, EXPORTED_SYMBOLS)

__all__ = ["PodsError", "load", "library_path", "pods_select", "pods_downsample", "pods_advantage",
           "pods_advantage_before", "pods_gather_rows", "pods_downsample_gather", "grpo_token_loss_fwd_bwd", "grpo_token_loss_fwd_bwd_static", "grpo_token_loss_report", "pods_check_rewards", "grpo_token_loss_static_workspace_bytes", "grpo_token_loss_workspace_bytes",
           "grpo_token_loss_workspace_min_bytes", "grpo_token_loss_workspace_used_bytes", "pods_last_error", "pods_profile_enable",
           "pods_profile_read", "pods_profile_mfma_only", "PODS_F32", "PODS_BF16", "PODS_RULE_MAXVAR", "PODS_RULE_MAXR", "PODS_RULE_PERC", "PODS_RULE_RAND",
           "EXPORTED_SYMBOLS"]
