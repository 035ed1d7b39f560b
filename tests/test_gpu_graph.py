"""The single-call training step, eagerly and as a replayed HIP graph, against the three separate calls.

Every replay starts from a snapshot of the run (environment state, parameters, optimiser moments) and is
checked against rollout + compute_gae + ppo_update called one by one from that same snapshot with the host-side
step offset and optimiser step count the device counters should hold.  The forward pass has no atomics, so the
whole trajectory (and the environment state after it) must come out bit for bit: a replay that sampled with a
stale step counter, or rolled out under stale parameters, would differ in its actions.  The update sums
gradients with fp32 atomics and takes Adam's bias corrections from a device-side pow, so parameters and moments
are compared to 1e-5 of their scale.  Between replays the program does ordinary eager work and synchronises.
"""
import numpy as np
import pytest
import torch

import workloads as W
from gpu_util import dev, rel_err, small

pytestmark = pytest.mark.gpu

TRAJ_FIELDS = ("obs", "action", "logp", "value", "reward", "done", "last_value", "adv", "ret")


@pytest.fixture(scope="module")
def M():
    import paper_2107_01460_amd as m
    return m


class Run:
    """All device buffers of one training run."""

    def __init__(self, M, cfg, params):
        self.cfg = cfg
        self.st = M.EnvState(cfg)
        M.env_reset(cfg, self.st)
        self.tr = M.Traj(cfg)
        self.params = dev(params).clone()
        self.m = torch.zeros_like(self.params)
        self.v = torch.zeros_like(self.params)
        sizes = M.query_sizes(cfg)
        self.ws_r = M.alloc_workspace(sizes.rollout_workspace_bytes)
        self.ws_u = M.alloc_workspace(sizes.update_workspace_bytes)
        self.stats = torch.zeros((cfg["n_epochs"] * cfg["n_minibatches"], 8), device="cuda")

    def load(self, other):
        for f in type(self.st).FIELDS:
            getattr(self.st, f).copy_(getattr(other.st, f))
        self.params.copy_(other.params)
        self.m.copy_(other.m)
        self.v.copy_(other.v)


def check_step(M, cfg, graph_run, ref_run, it, perm_dev):
    """ref_run (loaded with the snapshot taken before the step) takes the step by the three separate calls."""
    T, EM = cfg["rollout_len"], cfg["n_epochs"] * cfg["n_minibatches"]
    M.rollout(cfg, ref_run.st, ref_run.params, ref_run.tr, it * T, ref_run.ws_r)
    M.compute_gae(cfg, ref_run.tr)
    M.ppo_update(cfg, ref_run.tr, ref_run.params, ref_run.m, ref_run.v, it * EM, perm_dev, ref_run.stats, None, ref_run.ws_u)
    torch.cuda.synchronize()
    for f in TRAJ_FIELDS:
        assert torch.equal(getattr(graph_run.tr, f), getattr(ref_run.tr, f)), (it, f)
    for f in type(graph_run.st).FIELDS:
        assert torch.equal(getattr(graph_run.st, f), getattr(ref_run.st, f)), (it, f)
    tol = 1e-5 if cfg["precision"] == 0 else 2e-3   # bf16: a parameter near a rounding boundary of its bf16 copy
    assert rel_err(graph_run.params.cpu().numpy(), ref_run.params.cpu().numpy()) < tol, it
    assert rel_err(graph_run.m.cpu().numpy(), ref_run.m.cpu().numpy()) < 10 * tol, it
    assert rel_err(graph_run.v.cpu().numpy(), ref_run.v.cpu().numpy()) < 10 * tol, it
    assert rel_err(graph_run.stats[:, :4].cpu().numpy(), ref_run.stats[:, :4].cpu().numpy(), 0.05) < 100 * tol, it


@pytest.mark.parametrize("k", [1, 2, 3, 4])
def test_train_step_eager_and_graph_replays(M, k):
    cfg = small(k)
    print("case", cfg["name"], flush=True)
    T, EM = cfg["rollout_len"], cfg["n_epochs"] * cfg["n_minibatches"]
    params = W.init_params(cfg, bias_scale=0.1)
    run, ref = Run(M, cfg, params), Run(M, cfg, params)
    counters = M.alloc_counters()
    perm = dev(W.make_perm(cfg, seed=3))
    it = 0

    # ---- two ordinary calls (the first also sets the kernel attributes)
    for _ in range(2):
        ref.load(run)
        M.train_step(cfg, run.st, run.params, run.tr, run.m, run.v, counters, perm, run.stats, run.ws_r, run.ws_u)
        torch.cuda.synchronize()
        check_step(M, cfg, run, ref, it, perm)
        it += 1
        assert counters.tolist() == [it * T, it * EM]

    # ---- capture one call, replay it for the following iterations with a new row order each time
    g = torch.cuda.CUDAGraph()
    snap = Run(M, cfg, params)
    snap.load(run)
    saved = counters.clone()
    with torch.cuda.graph(g):
        M.train_step(cfg, run.st, run.params, run.tr, run.m, run.v, counters, perm, run.stats, run.ws_r, run.ws_u)
    torch.cuda.synchronize()
    # capturing runs nothing: the run and its counters are as before
    assert torch.equal(run.params, snap.params) and torch.equal(counters, saved)
    for r in range(4):
        perm.copy_(dev(W.make_perm(cfg, seed=10 + r)))
        ref.load(run)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        check_step(M, cfg, run, ref, it, perm)
        it += 1
        assert counters.tolist() == [it * T, it * EM]
        assert bool(torch.isfinite(run.params).all())
