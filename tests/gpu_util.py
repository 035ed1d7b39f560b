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


# The bf16 configuration is compared twice.  Against the oracle's weights-only mode (precision 1: everything but the
# weight rounding exact) at the wide floor above, which measures the activation rounding itself; and against the
# oracle's input-rounding mode (precision 2: h1, h2, dz2, dz1 rounded to bf16 where the method rounds them), where only
# the fp32 accumulation order and activations that sit on a rounding boundary are left.  Such an activation (its fp32
# and fp64 evaluations fall on different sides of a bf16 rounding boundary: about 3 % of the samples have one among
# their 512 first-layer units) moves by a whole bf16 step, 2^-9, and the next layer amplifies it: the second-layer
# pre-activations all move by ~1e-4, which flips ~5 % of THEIR roundings, and the output moves by ~3e-4 of its scale
# (measured: 2.4e-4).  Hence a floor of 2.5e-2 (2e-2 * 2.5e-2 = 5e-4 of the scale) -- ten times below the first
# comparison's -- at the same 2e-2 relative bound.
# Gradients pass through two more rounded products (dz2, dz1) and are sums of per-sample terms that largely cancel, so
# a moved sample shows more in them (at the 1000-sample test sizes: up to 1.1e-3 of the largest element, 2.2 % of an
# element a twentieth of the largest): their floor is 0.1 (2e-3 of the largest element), against 0.25 in the first
# comparison, and at the 1000-sample sizes the bound is 3e-2 (measured 2.2e-2 on one element of one shape, from run to run).
TIGHT_TOL, TIGHT_FLOOR, TIGHT_FLOOR_GRAD, TIGHT_TOL_GRAD = 2e-2, 2.5e-2, 0.1, 3e-2


def tight_cfg(cfg):
    """The oracle-side configuration of the second comparison (None for fp32 configurations)."""
    return W.scaled(cfg, precision=2) if cfg["precision"] == 1 else None


def err_tight(got, ref, grad=False):
    return rel_err(got, ref, TIGHT_FLOOR_GRAD if grad else TIGHT_FLOOR)


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
