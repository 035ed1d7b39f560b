"""Helpers shared by the GPU parity tests."""
import numpy as np
import torch

import workloads as W

REL_TOL = {0: 1e-4, 1: 2e-2}   # fp32 configs; bf16 GEMM configs
# Elements below FLOOR * max|reference| are measured against that floor.  fp32: see rel_err.  bf16: one
# rounding of an O(1) hidden activation to bf16 already moves it by up to 2^-9 = 2e-3, and the outputs are
# sums of such activations, so their absolute error is ~2e-3 of the output scale whatever their own size.
FLOOR = {0: 1e-2, 1: 0.25}


def err(got, ref, cfg):
    return rel_err(got, ref, FLOOR[cfg["precision"]])


def rel_err(got, ref, floor=1e-2):
    """max_i |g_i - o_i| / max(|o_i|, floor * max|o|).

    Relative error per element, except that elements smaller than `floor` times the tensor's
    largest magnitude are measured against that floor: an fp32 dot product of K terms carries an
    absolute error of about sqrt(K) * 2^-24 times the magnitude of its terms whatever the order of
    summation, so an element that is the small remainder of cancelling terms cannot be held to 1e-4
    of its own magnitude by any fp32 evaluation (1e-4 * 1e-2 = 1e-6 of the scale is ~16 ulp)."""
    got = np.asarray(got, np.float64).reshape(-1)
    ref = np.asarray(ref, np.float64).reshape(-1)
    scale = np.maximum(np.abs(ref), floor * max(np.abs(ref).max(), 1e-30))
    return float((np.abs(got - ref) / scale).max())


def small(k, **kw):
    """Config k (1-based) shrunk to a CPU-oracle-sized case that still spans several tiles and a ragged tail."""
    base = {1: dict(n_envs=70, rollout_len=9, n_minibatches=3),
            2: dict(n_envs=66, rollout_len=10, n_minibatches=4, n_epochs=2, episode_cap=8),
            3: dict(n_envs=45, rollout_len=8, n_minibatches=2, n_epochs=2, episode_cap=6),
            4: dict(n_envs=21, rollout_len=6, n_minibatches=2, n_epochs=1, episode_cap=5),
            5: dict(n_envs=150, rollout_len=6, n_minibatches=4)}[k]
    base.update(kw)
    return W.scaled(W.CONFIGS[k - 1], **base)


def dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


def load_traj(M, cfg, otr, debug=False):
    """Device trajectory filled from an oracle trajectory."""
    tr = M.Traj(cfg, debug=debug)
    for f in ("obs", "action", "logp", "value", "reward", "done", "last_value", "adv", "ret"):
        getattr(tr, f).copy_(dev(getattr(otr, f)))
    return tr
