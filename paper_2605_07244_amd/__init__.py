"""MI355X-native GRPO scoring hot path: thin Python binding over the C-ABI library.

The arithmetic lives entirely in the HIP library (libmrl.so, built in-tree by
`paper_2605_07244_amd.build`).  This package only marshals arguments; PyTorch
supplies device memory and streams.
"""
from .binding import (  # noqa: F401
    ADV_BATCH_ZN, ADV_CENTER, ADV_GROUP_ZN, BF16, F32, LossConfig, MrlError, PROF_CLASSES,
    grpo_loss_fwd_bwd, grpo_loss_workspace, group_advantages, lib, library_path, profile_collect,
    dw_tail_plan, probe_mfma_rate, profile_enable, read_stats, thl_word_align, status_string, token_logprobs, token_logprobs_static, token_logprobs_workspace, token_scores, version,
)
