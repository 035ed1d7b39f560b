"""The five synthetic workloads and the seeded input generators that both the HIP path and
the CPU oracle are fed from.  Nothing of the method's arithmetic lives here: only
configuration data, parameter initialisation (which is an *input* of the training step) and
seeded random inputs (permutations, forced actions, forced uniforms).

The workloads stand in for the Level-Based-Foraging scenarios the paper measures on
(Section 4, Fig. 6: 15x15 grid / 4 players / 3 food, and 8x8 grid / 2 players): same grid
sizes, agent and food counts, but fully generated from a seed.
"""
import math

import numpy as np

N_ACTIONS = 6

_COMMON = dict(
    gamma=0.99, clip_eps=0.2, lr=3e-4,
    # The paper and the workload list give no value for these; ordinary PPO defaults are used.
    ent_coef=0.01, vf_coef=0.5, normalize_adv=1, max_grad_norm=0.5, beta1=0.9, beta2=0.999,
    adam_eps=1e-5, clip_value=0,
    env_kind=0,   # 1 / 2: the warehouse world (2: episodes also end on a collision); max_level = requested shelves
    recurrent=0,  # 1: a GRU cell in place of the second hidden layer of both networks (scaled(cfg, recurrent=1))
)
_COMMON["lambda"] = 0.95


def _cfg(**kw):
    c = dict(_COMMON)
    c.update(kw)
    return c


# 1-based config k is CONFIGS[k-1].
CONFIGS = [
    _cfg(name="c1_8x8_2ag_ippo", grid=8, n_agents=2, n_food=1, max_level=2, episode_cap=25, view=3,
         n_envs=64, rollout_len=16, actor_hidden=64, critic_hidden=64, central_critic=0, precision=0,
         n_epochs=1, n_minibatches=2, seed=0xC0FFEE + 1),
    _cfg(name="c2_10x10_3ag_ippo", grid=10, n_agents=3, n_food=3, max_level=3, episode_cap=50, view=5,
         n_envs=1024, rollout_len=128, actor_hidden=128, critic_hidden=128, central_critic=0, precision=0,
         n_epochs=4, n_minibatches=4, seed=0xC0FFEE + 2),
    _cfg(name="c3_15x15_4ag_mappo", grid=15, n_agents=4, n_food=3, max_level=3, episode_cap=70, view=5,
         n_envs=16384, rollout_len=128, actor_hidden=128, critic_hidden=256, central_critic=1, precision=0,
         n_epochs=4, n_minibatches=8, seed=0xC0FFEE + 3),
    _cfg(name="c4_20x20_8ag_ippo_bf16", grid=20, n_agents=8, n_food=6, max_level=3, episode_cap=100, view=7,
         n_envs=4096, rollout_len=128, actor_hidden=512, critic_hidden=512, central_critic=0, precision=1,
         n_epochs=4, n_minibatches=16, seed=0xC0FFEE + 4),
    _cfg(name="c5_8x8_2ag_ippo_wide", grid=8, n_agents=2, n_food=1, max_level=2, episode_cap=25, view=3,
         n_envs=131072, rollout_len=64, actor_hidden=64, critic_hidden=64, central_critic=0, precision=0,
         n_epochs=1, n_minibatches=8, seed=0xC0FFEE + 5),
]


def scaled(cfg, **kw):
    """A copy of a workload with some fields replaced (smaller N / T for CPU-sized parity cases)."""
    c = dict(cfg)
    c.update(kw)
    return c


def obs_dim(cfg):
    return 3 * cfg["view"] ** 2


def critic_in_dim(cfg):
    return obs_dim(cfg) * (cfg["n_agents"] if cfg["central_critic"] else 1)


def param_layout(cfg):
    """[(name, shape)] of the flat fp32 parameter vector: actor then critic; y = x W + b, W is [in][out]."""
    D, Ha, Hc, Dc = obs_dim(cfg), cfg["actor_hidden"], cfg["critic_hidden"], critic_in_dim(cfg)
    if cfg.get("recurrent", 0):
        def net(prefix, din, h, dout):
            return [(prefix + ".We", (din, h)), (prefix + ".be", (h,)), (prefix + ".Wi", (h, 3 * h)),
                    (prefix + ".bi", (3 * h,)), (prefix + ".Wh", (h, 3 * h)), (prefix + ".bh", (3 * h,)),
                    (prefix + ".W3", (h, dout)), (prefix + ".b3", (dout,))]
        return net("actor", D, Ha, N_ACTIONS) + net("critic", Dc, Hc, 1)
    return [("actor.W1", (D, Ha)), ("actor.b1", (Ha,)), ("actor.W2", (Ha, Ha)), ("actor.b2", (Ha,)),
            ("actor.W3", (Ha, N_ACTIONS)), ("actor.b3", (N_ACTIONS,)),
            ("critic.W1", (Dc, Hc)), ("critic.b1", (Hc,)), ("critic.W2", (Hc, Hc)), ("critic.b2", (Hc,)),
            ("critic.W3", (Hc, 1)), ("critic.b3", (1,))]


def param_count(cfg):
    return sum(int(np.prod(s)) for _, s in param_layout(cfg))


def init_params(cfg, seed=None, bias_scale=0.0):
    """Orthogonal initialisation with gain sqrt(2) of every weight matrix, biases bias_scale * N(0,1)."""
    import torch

    g = torch.Generator().manual_seed(int(cfg["seed"] if seed is None else seed))
    parts = []
    for name, shape in param_layout(cfg):
        if len(shape) == 2:
            w = torch.empty(shape[1], shape[0], dtype=torch.float32)  # torch convention [out][in]
            torch.nn.init.orthogonal_(w, gain=math.sqrt(2.0), generator=g)
            parts.append(w.t().contiguous().reshape(-1))
        else:
            parts.append(bias_scale * torch.randn(shape[0], generator=g, dtype=torch.float32))
    return torch.cat(parts).numpy().astype(np.float32)


def make_env_perm(cfg, seed=None):
    """[E][N] int32: one seeded permutation of the N environments per epoch (sequence minibatches of the
    recurrent networks)."""
    import torch

    base = int(cfg["seed"] if seed is None else seed)
    out = np.empty((cfg["n_epochs"], cfg["n_envs"]), np.int32)
    for e in range(cfg["n_epochs"]):
        g = torch.Generator().manual_seed(base + e)
        out[e] = torch.randperm(cfg["n_envs"], generator=g).numpy().astype(np.int32)
    return out


def make_perm(cfg, seed=None):
    """[E][R] int32: one seeded permutation of the R = T*N trajectory rows per epoch."""
    import torch

    R = cfg["rollout_len"] * cfg["n_envs"]
    base = int(cfg["seed"] if seed is None else seed)
    out = np.empty((cfg["n_epochs"], R), np.int32)
    for e in range(cfg["n_epochs"]):
        g = torch.Generator().manual_seed(base + e)
        out[e] = torch.randperm(R, generator=g).numpy().astype(np.int32)
    return out


def random_actions(cfg, steps, seed, p_load=None):
    """[steps][N][A] int32 uniform actions (optionally with a raised probability of 'load')."""
    rng = np.random.default_rng(seed)
    shape = (steps, cfg["n_envs"], cfg["n_agents"])
    a = rng.integers(0, N_ACTIONS, size=shape, dtype=np.int32)
    if p_load is not None:
        a = np.where(rng.random(shape) < p_load, 5, a).astype(np.int32)
    return a


def random_uniforms(cfg, steps, seed):
    """[steps][N][A][6] fp32 in (0,1)."""
    rng = np.random.default_rng(seed)
    u = rng.random((steps, cfg["n_envs"], cfg["n_agents"], N_ACTIONS), dtype=np.float32)
    return np.clip(u, 2.0 ** -24, 1.0 - 2.0 ** -24).astype(np.float32)
