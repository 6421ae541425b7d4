"""libgrpo for MI355X: the GRPO token-level objective with two-sided clipping
(forward + fused backward over the full vocabulary) as hand-written gfx950 kernels
behind a C ABI (include/grpo.h).  This package is the thin binding plus the seeded
synthetic workloads; it has no CPU implementation of the path."""
from .binding import (COUNT_NAMES, GRPO_BF16, GRPO_F32, GrpoError, grpo_filter_groups,  # noqa: F401
                      grpo_group_advantages, grpo_total_rewards,
                      grpo_logprobs_fwd, grpo_loss_aux_fwd_bwd, grpo_loss_fwd_bwd, grpo_packed_layout,
                      grpo_loss_fwd_bwd_noalloc, NOALLOC_MAX_TOKENS,
                      grpo_workspace_bytes, grpo_row_kernel_plan,
                      grpo_workspace_error, lib, status_string,
                      grpo_lmhead_workspace_bytes, grpo_lmhead_workspace_bytes_for_chunk, grpo_lmhead_logprobs_fwd, grpo_lmhead_loss_fwd_bwd,
                      grpo_lmhead_loss_aux_fwd_bwd)
from .build import build_library  # noqa: F401
from . import workloads  # noqa: F401
