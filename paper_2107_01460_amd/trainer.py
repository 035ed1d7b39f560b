"""A training run around the library: the loop of Fig. 2 (rollout -> loss -> gradient -> new parameters) with
evaluation blocks in between (Section 2: training is interleaved with evaluation blocks).

Host logic only.  Every step of the path runs in the library's kernels; this class owns the device buffers,
draws the per-epoch row permutations with torch on the device and calls the entry points in order.  The
parameters start from a seeded orthogonal initialisation (gain sqrt 2, zero biases), which is set-up, not part
of the training step.
"""
import math

import torch

from . import binding as B


def init_params(cfg, seed=0):
    """Flat fp32 parameter vector in the library's layout (feed-forward: W1 b1 W2 b2 W3 b3 per network; recurrent:
    We be Wi bi Wh bh W3 b3), every weight matrix orthogonal with gain sqrt 2, biases zero."""
    g = torch.Generator().manual_seed(int(seed))
    D = 3 * cfg["view"] ** 2
    Dc = D * cfg["n_agents"] if cfg["central_critic"] else D
    blocks = []
    for din, h, dout in ((D, cfg["actor_hidden"], B.N_ACTIONS), (Dc, cfg["critic_hidden"], 1)):
        if cfg.get("recurrent", 0):
            shapes = [(din, h), (h,), (h, 3 * h), (3 * h,), (h, 3 * h), (3 * h,), (h, dout), (dout,)]
        else:
            shapes = [(din, h), (h,), (h, h), (h,), (h, dout), (dout,)]
        for shp in shapes:
            t = torch.zeros(shp)
            if len(shp) == 2:
                torch.nn.init.orthogonal_(t, gain=math.sqrt(2.0), generator=g)
            blocks.append(t.reshape(-1))
    return torch.cat(blocks).float()


class Trainer:
    """Feed-forward IPPO / MAPPO on one GPU.  cfg: a dict with the fields of marl_config."""

    def __init__(self, cfg, seed=0, params=None):
        if cfg.get("recurrent", 0):
            raise B.MarlError("Trainer drives the feed-forward systems; the recurrent entry points are called directly")
        self.cfg = dict(cfg)
        sizes = B.query_sizes(self.cfg)
        self.state = B.EnvState(self.cfg)
        self.traj = B.Traj(self.cfg)
        p = init_params(self.cfg, seed) if params is None else torch.as_tensor(params, dtype=torch.float32)
        if p.numel() != sizes.n_params:
            raise B.MarlError(f"expected {sizes.n_params} parameters, got {p.numel()}")
        self.params = p.cuda().contiguous()
        self.adam_m = torch.zeros_like(self.params)
        self.adam_v = torch.zeros_like(self.params)
        self.counters = B.alloc_counters()
        E, Mb = self.cfg["n_epochs"], self.cfg["n_minibatches"]
        self.rows = self.cfg["rollout_len"] * self.cfg["n_envs"]
        self.perm = torch.zeros((E, self.rows), dtype=torch.int32, device="cuda")
        self.stats = torch.zeros((E * Mb, 8), dtype=torch.float32, device="cuda")
        self.ws_rollout = B.alloc_workspace(sizes.rollout_workspace_bytes)
        self.ws_update = B.alloc_workspace(sizes.update_workspace_bytes)
        self.ws_eval = B.alloc_workspace(sizes.eval_workspace_bytes)
        self.eval_state = B.EnvState(self.cfg)
        self.eval_out = B.EvalStats(self.cfg)
        self.gen = torch.Generator(device="cuda").manual_seed(int(seed) + 1)
        self.iterations = 0
        B.env_reset(self.cfg, self.state)

    def step(self):
        """One training iteration; returns nothing and does not synchronise."""
        for e in range(self.perm.shape[0]):
            self.perm[e].copy_(torch.randperm(self.rows, generator=self.gen, device="cuda"))
        B.train_step(self.cfg, self.state, self.params, self.traj, self.adam_m, self.adam_v, self.counters, self.perm,
                     self.stats, self.ws_rollout, self.ws_update)
        self.iterations += 1

    def train(self, iterations):
        for _ in range(int(iterations)):
            self.step()

    def last_stats(self):
        """Mean over the last iteration's minibatches: a dict of the eight columns of `stats`."""
        names = ("policy_loss", "value_loss", "entropy", "approx_kl", "clip_fraction", "grad_norm", "total_loss", "non_finite")
        m = self.stats.mean(dim=0).tolist()
        return dict(zip(names, m))

    def evaluate(self, episodes=4):
        """Greedy evaluation block on fresh environments: (mean episode return summed over agents, mean length)."""
        B.env_reset(self.cfg, self.eval_state)
        B.evaluate(self.cfg, self.eval_state, self.params, episodes, self.eval_out, self.ws_eval)
        n = float(self.eval_out.episodes.sum().item())
        return float(self.eval_out.ret_sum.sum().item()) / n, float(self.eval_out.len_sum.sum().item()) / n
