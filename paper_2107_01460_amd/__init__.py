"""MI355X-native fused multi-agent PPO training step (IPPO / MAPPO on a grid-foraging world).

Everything is computed by hand-written HIP kernels in libmarl_gfx950.so (C ABI in include/marl.h);
this package only marshals arguments.  PyTorch is used for device memory and streams.
"""
from . import binding  # noqa: F401
from .binding import (  # noqa: F401
    Config, EnvState, Traj, MarlError, lib, make_config, query_sizes, env_reset, observe, env_step,
    policy_forward, sample_actions, rollout, rollout_static, compute_gae, ppo_update, status_string, alloc_workspace,
    timing_enable, timing_read, KERNEL_CLASSES, EvalStats, evaluate, RecState, rollout_recurrent, ppo_update_recurrent, train_step, alloc_counters,
)
from .trainer import Trainer  # noqa: F401,E402
