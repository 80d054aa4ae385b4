"""MI355X-native model-local worker step of UnityMAS-O: Python binding of libumas.

The binding only marshals arguments: every step of the path (reward composition and
placement, routing through the agent-to-model map, GAE scans, LM-head scoring, the clipped
surrogate and its backward) runs in the HIP kernels behind the C ABI of include/umas.h.
PyTorch supplies device memory and the current stream, nothing else.
"""
from .binding import (  # noqa: F401
    UmasError, Streams, lib_path, load_library,
    umas_assign_token_rewards, umas_advantages, umas_policy_logprobs, umas_ppo_loss_fwd_bwd,
    umas_policy_logprobs_static, STATIC_SCRATCH_BYTES,
    ppo_workspace_bytes, read_stats, profile_enable, profile_read,
    umas_values, umas_value_loss_fwd_bwd, read_value_stats, umas_kl_rewards, umas_whiten_advantages,
    WHITEN_MODEL, WHITEN_MODEL_ROLE, umas_ready_batch, umas_ready_batch_packed,
    PLACE_LAST, PLACE_ALL, SEG_TURN, SEG_TRAJ,
)
