"""Whole-iteration sanity of the oracle: repeated rollout -> GAE -> PPO update (Fig. 2) makes the policy better.

No stage-by-stage pin can show that the stages fit together (an advantage with the wrong sign, a gradient
applied uphill or a reward credited to the wrong agent all pass shape checks), so this runs the loop on the
smallest workload and asks for what the method exists to deliver: the greedy policy's mean episode return
rises well above the untrained one's and episodes end sooner (food is collected before the step cap).
"""
import numpy as np

import workloads as W


def test_mean_return_rises_on_the_smallest_workload(orc):
    cfg = W.scaled(W.CONFIGS[0], n_envs=64)
    params = W.init_params(cfg, seed=1)
    state = orc.EnvState(cfg)
    orc.env_reset(cfg, state)
    traj = orc.Traj(cfg)
    m, v = np.zeros_like(params), np.zeros_like(params)
    T, EM = cfg["rollout_len"], cfg["n_epochs"] * cfg["n_minibatches"]

    def greedy():
        s = orc.EnvState(cfg)
        orc.env_reset(cfg, s)
        ret, length, episodes, _ = orc.evaluate(cfg, s, params, 8)
        return ret.sum() / episodes.sum(), length.sum() / episodes.sum()

    ret0, len0 = greedy()
    for it in range(250):
        orc.rollout(cfg, state, params, traj, it * T)
        orc.compute_gae(cfg, traj)
        orc.ppo_update(cfg, traj, params, m, v, it * EM, W.make_perm(cfg, seed=100 + it))
    ret1, len1 = greedy()
    assert ret0 < 0.05 and len0 > 24.0          # the untrained greedy policy almost never collects the food
    assert ret1 > 0.2 and ret1 > ret0 + 0.2     # after 250 iterations it does, in every fifth episode or more
    assert len1 < 22.0
    assert np.all(np.isfinite(params))
