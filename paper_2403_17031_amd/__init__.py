"""MI355X-native rollout generation + teacher-forced rescoring for PPO-based RLHF.

The work happens in librlhf_rollout.so (hand-written HIP kernels behind a C ABI, see
include/rlhf_rollout.h); this package only marshals arguments.
"""
from .binding import (  # noqa: F401
    LIB_PATH,
    Policy,
    RlhfError,
    load_library,
    exported_symbols,
    ppo_assemble_rewards,
    ppo_gae,
    ppo_whiten,
    ppo_loss,
    PPO_LOSS_STATS,
    adamw_step,
    attention_backward,
    linear_lr,
)
