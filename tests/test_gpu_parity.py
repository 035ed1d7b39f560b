"""HIP path vs CPU oracle, element by element, through the C ABI.  Needs a real MI355X."""
import numpy as np
import pytest
import torch

import workloads as W
from gpu_util import REL_TOL, TIGHT_TOL, TIGHT_TOL_GRAD, dev, err, err_tight, load_traj, rel_err, small, tight_cfg

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def M():
    import paper_2107_01460_amd as m
    assert torch.cuda.is_available()
    m.lib()
    return m


def assert_state_equal(M, gstate, ostate):
    host = gstate.to_host()
    for f in M.EnvState.FIELDS:
        assert np.array_equal(host[f], getattr(ostate, f)), f


@pytest.mark.parametrize("k", [1, 2, 3, 4, 5])
def test_env_reset_step_observe_bit_exact(M, orc, k):
    cfg = small(k, n_envs={1: 70, 2: 333, 3: 200, 4: 77, 5: 1000}[k], n_minibatches=1,
                episode_cap={1: 25, 2: 50, 3: 15, 4: 12, 5: 25}[k])
    N, A, D = cfg["n_envs"], cfg["n_agents"], W.obs_dim(cfg)
    print("case", cfg["name"], N, flush=True)
    os_ = orc.EnvState(cfg)
    orc.env_reset(cfg, os_)
    gs = M.EnvState(cfg)
    M.env_reset(cfg, gs)
    assert_state_equal(M, gs, os_)
    obs = torch.empty((N, A, D), device="cuda")
    M.observe(cfg, gs, obs)
    assert np.array_equal(obs.cpu().numpy(), orc.observe(cfg, os_))
    steps = 60
    acts = W.random_actions(cfg, steps, seed=k, p_load=0.35)
    reward = torch.empty((N, A), device="cuda")
    done = torch.empty((N,), dtype=torch.uint8, device="cuda")
    n_done = 0
    rsum = 0.0
    for t in range(steps):
        M.env_step(cfg, gs, dev(acts[t]), obs, reward, done)
        oobs, orew, odone = orc.env_step(cfg, os_, acts[t])
        assert np.array_equal(done.cpu().numpy(), odone), t
        assert np.array_equal(reward.cpu().numpy().view(np.uint32), orew.view(np.uint32)), t
        assert np.array_equal(obs.cpu().numpy(), oobs), t
        assert_state_equal(M, gs, os_)
        n_done += int(odone.sum())
        rsum += float(orew.sum())
    assert n_done > 0 and rsum > 0     # resets and loads were exercised
    # obs = NULL is allowed
    M.env_step(cfg, gs, dev(acts[0]), None, reward, done)
    orc.env_step(cfg, os_, acts[0], want_obs=False)
    assert_state_equal(M, gs, os_)


def test_env_single_env_and_large_grid(M, orc):
    cfg = W.scaled(W.CONFIGS[0], grid=40, n_agents=1, n_food=8, max_level=5, view=7, n_envs=1, episode_cap=7)
    os_, gs = orc.EnvState(cfg), M.EnvState(cfg)
    orc.env_reset(cfg, os_)
    M.env_reset(cfg, gs)
    obs = torch.empty((1, 1, W.obs_dim(cfg)), device="cuda")
    reward = torch.empty((1, 1), device="cuda")
    done = torch.empty((1,), dtype=torch.uint8, device="cuda")
    acts = W.random_actions(cfg, 30, seed=2)
    for t in range(30):
        M.env_step(cfg, gs, dev(acts[t]), obs, reward, done)
        oobs, orew, odone = orc.env_step(cfg, os_, acts[t])
        assert np.array_equal(obs.cpu().numpy(), oobs) and np.array_equal(done.cpu().numpy(), odone)
    assert_state_equal(M, gs, os_)


@pytest.mark.parametrize("k", [1, 2, 3, 4, 5])
def test_policy_forward(M, orc, k):
    check_policy_forward(M, orc, small(k), k)


def check_policy_forward(M, orc, cfg, k):
    A, D = cfg["n_agents"], W.obs_dim(cfg)
    rows = 333
    print("case", cfg["name"], rows, flush=True)
    params = W.init_params(cfg, bias_scale=0.2)
    rng = np.random.default_rng(k)
    obs = (rng.integers(0, 4, size=(rows, A, D)) * (rng.random((rows, A, D)) < 0.3)).astype(np.float32)
    ws = M.alloc_workspace(M.query_sizes(W.scaled(cfg, n_envs=rows, n_minibatches=1)).rollout_workspace_bytes)
    logits = torch.empty((rows, A, 6), device="cuda")
    value = torch.empty((rows, A), device="cuda")
    M.policy_forward(cfg, dev(params), dev(obs), rows, logits, value, ws)
    ol, ov = orc.policy_forward(cfg, params, obs)
    tol = REL_TOL[cfg["precision"]]
    assert err(logits.cpu().numpy(), ol, cfg) < tol
    assert err(value.cpu().numpy(), ov, cfg) < tol
    if tight_cfg(cfg):
        ol2, ov2 = orc.policy_forward(tight_cfg(cfg), params, obs)
        print("tight forward", err_tight(logits.cpu().numpy(), ol2), err_tight(value.cpu().numpy(), ov2), flush=True)
        assert err_tight(logits.cpu().numpy(), ol2) < TIGHT_TOL
        assert err_tight(value.cpu().numpy(), ov2) < TIGHT_TOL
    # either output alone
    l2 = torch.empty_like(logits)
    M.policy_forward(cfg, dev(params), dev(obs), rows, l2, None, ws)
    assert torch.equal(l2, logits)


def test_sampling_identical_logits_and_uniforms(M, orc):
    cfg = small(1)
    rng = np.random.default_rng(11)
    n = 50000
    logits = (rng.normal(size=(n, 6)) * 2).astype(np.float32)
    u = W.random_uniforms(W.scaled(cfg, n_envs=n // 2), 1, seed=5).reshape(n, 6)
    action = torch.empty(n, dtype=torch.int32, device="cuda")
    sampled = torch.empty_like(action)
    logp = torch.empty(n, device="cuda")
    M.sample_actions(cfg, dev(logits), dev(u), None, n, 0, action, sampled, logp)
    oa, osmp, olp, gap = orc.sample(logits, u)
    mism = action.cpu().numpy() != oa
    assert np.all(gap[mism] < 1e-5), (mism.sum(), gap[mism].max() if mism.any() else 0)
    assert mism.mean() < 1e-3
    ok = ~mism
    assert rel_err(logp.cpu().numpy()[ok], olp[ok]) < 1e-4
    assert torch.equal(action, sampled)
    # forced actions: logp follows the forced action, the draw is still reported
    forced = rng.integers(0, 6, size=n).astype(np.int32)
    M.sample_actions(cfg, dev(logits), dev(u), dev(forced), n, 0, action, sampled, logp)
    _, _, olp2, _ = orc.sample(logits, u, forced)
    assert np.array_equal(action.cpu().numpy(), forced)
    assert rel_err(logp.cpu().numpy(), olp2) < 1e-4
    # Philox uniforms: same key schedule as the oracle (step, sample = env*A + agent)
    n2, A = 600, cfg["n_agents"]
    step = (3 << 32) + 12345
    M.sample_actions(cfg, dev(logits[:n2]), None, None, n2, step, action[:n2], sampled[:n2], logp[:n2])
    uu = np.array([orc.sample_uniforms(cfg, step, i // A, i % A) for i in range(n2)])
    oa3, _, _, gap3 = orc.sample(logits[:n2], uu)
    mism3 = action[:n2].cpu().numpy() != oa3
    assert np.all(gap3[mism3] < 1e-5) and mism3.sum() <= 1


@pytest.mark.parametrize("k", [1, 2, 3, 4, 5])
def test_rollout_teacher_forced(M, orc, k):
    cfg = small(k)
    N, A, T = cfg["n_envs"], cfg["n_agents"], cfg["rollout_len"]
    print("case", cfg["name"], N, T, flush=True)
    params = W.init_params(cfg, bias_scale=0.1)
    os_ = orc.EnvState(cfg)
    orc.env_reset(cfg, os_)
    otr = orc.Traj(cfg)
    orc.rollout(cfg, os_, params, otr, step_offset=1000)
    gs = M.EnvState(cfg)
    M.env_reset(cfg, gs)
    gtr = M.Traj(cfg, debug=True)
    sizes = M.query_sizes(cfg)
    ws = M.alloc_workspace(sizes.rollout_workspace_bytes)
    M.rollout(cfg, gs, dev(params), gtr, 1000, ws, forced_actions=dev(otr.action))
    torch.cuda.synchronize()
    tol = REL_TOL[cfg["precision"]]
    assert np.array_equal(gtr.obs.cpu().numpy(), otr.obs)
    assert np.array_equal(gtr.reward.cpu().numpy().view(np.uint32), otr.reward.view(np.uint32))
    assert np.array_equal(gtr.done.cpu().numpy(), otr.done)
    assert np.array_equal(gtr.action.cpu().numpy(), otr.action)
    assert_state_equal(M, gs, os_)
    assert err(gtr.logits.cpu().numpy(), otr.logits, cfg) < tol
    assert err(gtr.value.cpu().numpy(), otr.value, cfg) < tol
    assert err(gtr.last_value.cpu().numpy(), otr.last_value, cfg) < tol
    assert err(gtr.logp.cpu().numpy(), otr.logp, cfg) < tol
    if tight_cfg(cfg):
        os2 = orc.EnvState(cfg)
        orc.env_reset(cfg, os2)
        otr2 = orc.Traj(cfg)
        orc.rollout(tight_cfg(cfg), os2, params, otr2, step_offset=1000, forced_actions=otr.action)
        for f in ("logits", "value", "last_value", "logp"):
            e = err_tight(getattr(gtr, f).cpu().numpy(), getattr(otr2, f))
            print("tight rollout", f, e, flush=True)
            assert e < TIGHT_TOL, f
    if cfg["precision"] == 0:
        # the sampler's own draw: equal to the oracle's except at near-ties of the perturbed logits
        mism = gtr.sampled.cpu().numpy() != otr.sampled
        lim = 1e-5 + 2e-4 * np.abs(otr.logits).max()   # logits themselves differ by up to tol
        assert np.all(otr.gap[mism] < lim), (mism.sum(), otr.gap[mism].max())
        assert mism.mean() < 5e-3
    # free-running (unforced) rollout with forced uniforms equal to the oracle's Philox stream must
    # reproduce the forced run wherever the draw agreed
    assert otr.done.sum() > 0


@pytest.mark.parametrize("k,kind,agents,food", [(2, 0, 3, 3), (2, 0, 3, 1), (5, 0, 1, 2), (2, 1, 3, 4), (4, 0, 5, 6), (3, 2, 2, 3)])
def test_long_rollout_through_many_resets(M, orc, k, kind, agents, food):
    """Many episodes per environment inside ONE rollout (the state of an environment stays on chip for the whole
    rollout), with agent and food counts below the unrolled capacities: the oracle, forced with the GPU's own actions,
    must reproduce every observation, reward, done flag and the final state bit for bit."""
    cfg = small(k, n_envs=53, rollout_len=96, n_minibatches=1, episode_cap=7, n_agents=agents, n_food=food,
                env_kind=kind, precision=0)
    if kind:
        cfg = W.scaled(cfg, max_level=min(cfg["max_level"], food))
    if cfg["actor_hidden"] > 256:
        cfg = W.scaled(cfg, actor_hidden=128, critic_hidden=128)
    print("case", cfg["name"], "kind", kind, "A", agents, "F", food, flush=True)
    params = W.init_params(cfg, bias_scale=0.1)
    gs = M.EnvState(cfg)
    M.env_reset(cfg, gs)
    gtr = M.Traj(cfg, debug=True)
    ws = M.alloc_workspace(M.query_sizes(cfg).rollout_workspace_bytes)
    M.rollout(cfg, gs, dev(params), gtr, 31, ws)
    torch.cuda.synchronize()
    os_ = orc.EnvState(cfg)
    orc.env_reset(cfg, os_)
    otr = orc.Traj(cfg)
    orc.rollout(cfg, os_, params, otr, step_offset=31, forced_actions=gtr.action.cpu().numpy())
    assert np.array_equal(gtr.obs.cpu().numpy(), otr.obs)
    assert np.array_equal(gtr.reward.cpu().numpy().view(np.uint32), otr.reward.view(np.uint32))
    assert np.array_equal(gtr.done.cpu().numpy(), otr.done)
    assert_state_equal(M, gs, os_)
    assert otr.done.sum() >= 10 * cfg["n_envs"]
    assert err(gtr.logits.cpu().numpy(), otr.logits, cfg) < REL_TOL[0]
    assert err(gtr.value.cpu().numpy(), otr.value, cfg) < REL_TOL[0]
    assert err(gtr.last_value.cpu().numpy(), otr.last_value, cfg) < REL_TOL[0]


@pytest.mark.parametrize("k", [1, 3, 5])
def test_gae(M, orc, k):
    cfg = small(k, n_envs=300, rollout_len=37, n_minibatches=1)
    rng = np.random.default_rng(k)
    otr = orc.Traj(cfg)
    otr.reward[:] = rng.random(otr.reward.shape) * (rng.random(otr.reward.shape) < 0.2)
    otr.value[:] = rng.normal(size=otr.value.shape)
    otr.last_value[:] = rng.normal(size=otr.last_value.shape)
    otr.done[:] = rng.random(otr.done.shape) < 0.1
    orc.compute_gae(cfg, otr)
    gtr = load_traj(M, cfg, otr)
    gtr.adv.zero_()
    gtr.ret.zero_()
    M.compute_gae(cfg, gtr)
    assert rel_err(gtr.adv.cpu().numpy(), otr.adv) < 1e-4
    assert rel_err(gtr.ret.cpu().numpy(), otr.ret) < 1e-4


def oracle_traj(orc, cfg, bias_scale=0.1):
    params = W.init_params(cfg, bias_scale=bias_scale)
    s = orc.EnvState(cfg)
    orc.env_reset(cfg, s)
    tr = orc.Traj(cfg)
    orc.rollout(cfg, s, params, tr, step_offset=5)
    orc.compute_gae(cfg, tr)
    return params, tr


@pytest.mark.parametrize("k,clipv,norm", [(1, 0, 1), (2, 0, 1), (3, 0, 1), (4, 0, 1), (5, 0, 1), (2, 1, 0), (3, 1, 1)])
def test_ppo_single_minibatch_gradient(M, orc, k, clipv, norm):
    """One minibatch over the whole (small) trajectory at perturbed parameters: loss terms and gradient."""
    cfg = small(k, n_epochs=1, n_minibatches=1, clip_value=clipv, normalize_adv=norm, max_grad_norm=0.0)
    check_single_minibatch_gradient(M, orc, cfg, k)


@pytest.mark.parametrize("ha,hc,view", [(128, 64, 7), (256, 256, 5), (512, 256, 5), (256, 512, 7)])
def test_bf16_other_widths(M, orc, ha, hc, view):
    """bf16 networks of other widths than config 4's 147-512-512.  Which GEMM kernel a product takes depends on
    them: output widths that are no multiple of 256 take the 128 x 128 tile kernel, the others the kernel with
    the weights resident in registers, in a different instantiation for every contraction length (padded input
    width 128 or 192, hidden width 256 or 512); dz1 at width 256 takes the tile kernel again."""
    kw = dict(actor_hidden=ha, critic_hidden=hc, view=view)
    check_policy_forward(M, orc, small(4, **kw), 40 + view)
    check_single_minibatch_gradient(M, orc, small(4, n_epochs=1, n_minibatches=1, max_grad_norm=0.0, **kw), 4)


@pytest.mark.parametrize("ha,hc", [(96, 512), (32, 160), (224, 192)])
def test_fp32_other_widths(M, orc, ha, hc):
    """fp32 networks of hidden widths that none of the workloads uses (any multiple of 32 up to 512 is accepted): they
    take the generic tile GEMMs with the separate output-layer / loss / dz2 kernels instead of the fused ones."""
    kw = dict(actor_hidden=ha, critic_hidden=hc)
    check_policy_forward(M, orc, small(2, **kw), 60 + ha // 32)
    check_single_minibatch_gradient(M, orc, small(2, n_epochs=1, n_minibatches=1, max_grad_norm=0.0, **kw), 2)


def test_bf16_odd_chunk_count(M, orc):
    """816 samples (17 environments): the weight-gradient kernel's k ranges hold 8 and 5 chunks of 64 samples, so
    the chunk-pair loop ends on a single chunk, and the last 64-row tile of the other kernels is ragged."""
    check_single_minibatch_gradient(M, orc, small(4, n_envs=17, n_epochs=1, n_minibatches=1, max_grad_norm=0.0), 4)


def test_wide_central_critic(M, orc):
    """A centralised critic whose input (8 agents x 147 = 1176 values) is wider than the fused forward kernel
    keeps in LDS: its forward pass, loss and gradient take the layer-by-layer kernels."""
    kw = dict(n_agents=8, view=7, n_food=5)
    check_policy_forward(M, orc, small(3, **kw), 31)
    check_single_minibatch_gradient(M, orc, small(3, n_epochs=1, n_minibatches=1, max_grad_norm=0.0, **kw), 3)


def check_single_minibatch_gradient(M, orc, cfg, k):
    print("case", cfg["name"], flush=True)
    params0, otr = oracle_traj(orc, cfg)
    rng = np.random.default_rng(100 + k)
    params = (params0 + 0.1 * np.abs(params0).mean() * rng.normal(size=params0.size)).astype(np.float32)
    otr.value[:] += (0.2 * rng.normal(size=otr.value.shape)).astype(np.float32)
    # ratios on both sides of the clip range, but well away from its edges: the branch of the min is a
    # discrete decision that a rounding error must not flip (in bf16 the ratio carries ~1% noise)
    otr.logp[:] += rng.choice([-0.4, 0.0, 0.0, 0.4], size=otr.logp.shape).astype(np.float32)
    R = cfg["rollout_len"] * cfg["n_envs"]
    perm = W.make_perm(cfg, seed=3)
    po, mo, vo = params.copy(), np.zeros_like(params), np.zeros_like(params)
    ostats, ograd = orc.ppo_update(cfg, otr, po, mo, vo, adam_step0=0, perm=perm)
    gtr = load_traj(M, cfg, otr)
    sizes = M.query_sizes(cfg)
    ws = M.alloc_workspace(sizes.update_workspace_bytes)
    gp, gm, gv = dev(params), torch.zeros(params.size, device="cuda"), torch.zeros(params.size, device="cuda")
    stats = torch.zeros((1, 8), device="cuda")
    gdump = torch.zeros(params.size, device="cuda")
    M.ppo_update(cfg, gtr, gp, gm, gv, 0, dev(perm), stats, gdump, ws)
    torch.cuda.synchronize()
    tol = REL_TOL[cfg["precision"]]
    g = gdump.cpu().numpy()
    Pa = orc.actor_param_count(cfg)
    assert err(g[:Pa], ograd[:Pa], cfg) < tol, "actor gradient"
    assert err(g[Pa:], ograd[Pa:], cfg) < tol, "critic gradient"
    if tight_cfg(cfg):
        p2, m2, v2 = params.copy(), np.zeros_like(params), np.zeros_like(params)
        ostats2, ograd2 = orc.ppo_update(tight_cfg(cfg), otr, p2, m2, v2, adam_step0=0, perm=perm)
        print("tight gradient", err_tight(g[:Pa], ograd2[:Pa], True), err_tight(g[Pa:], ograd2[Pa:], True), flush=True)
        assert err_tight(g[:Pa], ograd2[:Pa], True) < TIGHT_TOL_GRAD, "actor gradient against the input-rounding oracle mode"
        assert err_tight(g[Pa:], ograd2[Pa:], True) < TIGHT_TOL_GRAD, "critic gradient against the input-rounding oracle mode"
    st = stats.cpu().numpy()[0]
    assert 0.0 < ostats[0, 4] < 1.0           # clip fraction: both branches of the min are exercised
    for i in (0, 1, 2, 3, 5, 6):
        assert abs(st[i] - ostats[0, i]) < tol * max(abs(ostats[0, i]), 1e-2), (i, st[i], ostats[0, i])
    assert abs(st[4] - ostats[0, 4]) < 3.0 / (R * cfg["n_agents"])   # a ratio sitting on the clip edge may flip
    assert st[7] == 0
    # Adam: the oracle's optimiser step applied to the GPU's own gradient must land on the GPU's parameters
    # (the step normalises by |g|, so feeding it two gradients that differ by 1e-4 of their scale would not)
    pa, ma, va = params.copy(), np.zeros_like(params), np.zeros_like(params)
    orc.adam_step(cfg, pa, ma, va, g.astype(np.float64), 1)
    assert rel_err(gm.cpu().numpy(), ma) < 1e-5 and rel_err(gv.cpu().numpy(), va) < 1e-5
    assert rel_err(gp.cpu().numpy() - params, pa - params) < 1e-3   # fp32 rounding of p - delta
    assert np.abs(pa - params).max() > 0.5 * cfg["lr"]


@pytest.mark.parametrize("k", [1, 2, 3, 4, 5])
def test_ppo_update_epochs_and_minibatches(M, orc, k):
    cfg = small(k)
    print("case", cfg["name"], flush=True)
    params, otr = oracle_traj(orc, cfg)
    perm = W.make_perm(cfg, seed=9)
    E, Mb = cfg["n_epochs"], cfg["n_minibatches"]
    po, mo, vo = params.copy(), np.zeros_like(params), np.zeros_like(params)
    ostats, ograd = orc.ppo_update(cfg, otr, po, mo, vo, adam_step0=3, perm=perm)
    gtr = load_traj(M, cfg, otr)
    ws = M.alloc_workspace(M.query_sizes(cfg).update_workspace_bytes)
    gp, gm, gv = dev(params), torch.zeros(params.size, device="cuda"), torch.zeros(params.size, device="cuda")
    stats = torch.zeros((E * Mb, 8), device="cuda")
    gdump = torch.zeros(params.size, device="cuda")
    M.ppo_update(cfg, gtr, gp, gm, gv, 3, dev(perm), stats, gdump, ws)
    torch.cuda.synchronize()
    tol = REL_TOL[cfg["precision"]]
    st = stats.cpu().numpy()
    for i in (0, 1, 2, 5, 6):
        assert np.all(np.abs(st[:, i] - ostats[:, i]) < 20 * tol * np.maximum(np.abs(ostats[:, i]), 1e-2)), (i, st[:, i], ostats[:, i])
    assert np.all(st[:, 7] == 0)
    # after E*M optimiser steps the two parameter vectors have moved the same way.  Adam divides by |g|,
    # which magnifies the 1e-4 gradient differences of near-zero elements, so the bound is on the scale of
    # the largest move; the per-step statistics above are the tight check of the loop itself.
    # (bf16: the sign of a near-zero gradient element decides a full +-lr step, so only the gradient is compared)
    if cfg["precision"] == 0:
        assert rel_err(gp.cpu().numpy() - params, po - params, floor=1.0) < 0.05
    assert err(gdump.cpu().numpy(), ograd, cfg) < (100 * tol if cfg["precision"] == 0 else 5 * tol)
    # identity order when perm is NULL
    gp2, gm2, gv2 = dev(params), torch.zeros_like(gm), torch.zeros_like(gm)
    M.ppo_update(cfg, gtr, gp2, gm2, gv2, 3, None, stats, None, ws)
    R = cfg["rollout_len"] * cfg["n_envs"]
    po2, mo2, vo2 = params.copy(), np.zeros_like(params), np.zeros_like(params)
    orc.ppo_update(cfg, otr, po2, mo2, vo2, adam_step0=3, perm=None)
    if cfg["precision"] == 0:
        assert rel_err(gp2.cpu().numpy() - params, po2 - params, floor=1.0) < 0.05


@pytest.mark.parametrize("k", [1, 2, 3, 4, 5])
def test_greedy_evaluation_block(M, orc, k):
    """Per-environment return / length / episode counts of the greedy evaluation block, bit for bit, for every
    environment whose run stayed clear of a near-tie between its two largest logits (an fp32 evaluation may break
    such a tie the other way, after which the two runs are different episodes)."""
    n_envs = {1: 200, 2: 130, 3: 90, 4: 80, 5: 300}[k]
    cfg = small(k, n_envs=n_envs, n_minibatches=1, episode_cap={1: 12, 2: 10, 3: 9, 4: 6, 5: 12}[k])
    E = {1: 3, 2: 3, 3: 2, 4: 2, 5: 3}[k]
    print("case", cfg["name"], n_envs, E, flush=True)
    params = W.init_params(cfg, bias_scale=0.3)
    off = 0
    for name, shape in W.param_layout(cfg):   # a bias towards "load", so that food is lifted and episodes end early
        if name == "actor.b3":
            params[off + 5] += 1.0
        off += int(np.prod(shape))
    os_ = orc.EnvState(cfg)
    orc.env_reset(cfg, os_)
    # (bf16 configuration: the oracle in its input-rounding mode, so that the two sides' logits differ by the
    # accumulation order only and most environments stay clear of a tie that the difference could break)
    oret, olen, oeps, gap = orc.evaluate(tight_cfg(cfg) or cfg, os_, params, E)
    gs = M.EnvState(cfg)
    M.env_reset(cfg, gs)
    out = M.EvalStats(cfg)
    out.ret_sum.fill_(7.0)      # the call clears its outputs
    out.episodes.fill_(5)
    ws = M.alloc_workspace(M.query_sizes(cfg).eval_workspace_bytes)
    M.evaluate(cfg, gs, dev(params), E, out, ws)
    torch.cuda.synchronize()
    gret, glen, geps = out.ret_sum.cpu().numpy(), out.len_sum.cpu().numpy(), out.episodes.cpu().numpy()
    assert np.all(geps == E) and np.all(oeps == E)
    scale = float(np.abs(params).max())
    # logits differ between the two sides by up to the tolerance times their scale (a few units here)
    lim = (2e-4 if cfg["precision"] == 0 else 4e-3) * max(1.0, scale) * 4
    clear = gap > lim
    print("clear environments", clear.mean(), flush=True)
    assert clear.mean() > (0.9 if cfg["precision"] == 0 else 0.6), clear.mean()
    assert np.array_equal(gret[clear].view(np.uint32), oret[clear].view(np.uint32))
    assert np.array_equal(glen[clear], olen[clear])
    assert np.all(glen >= E) and np.all(glen <= E * cfg["episode_cap"])
    assert oret[clear].sum() > 0
    # final state of the clear environments
    host = gs.to_host()
    for f in M.EnvState.FIELDS:
        assert np.array_equal(host[f][..., clear], getattr(os_, f)[..., clear]), f
