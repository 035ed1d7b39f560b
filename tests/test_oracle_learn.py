"""Pins for the oracle's networks, sampler, GAE, PPO loss/gradient and Adam: float64 autograd
and library routines of torch (CPU) as special cases, central finite differences, brute-force
sums and closed forms."""
import sys

import numpy as np
import pytest
import torch

import workloads as W

torch.set_num_threads(2)


def small_cfg(central=0, **kw):
    base = dict(grid=6, n_agents=3, n_food=2, max_level=3, episode_cap=12, view=3, n_envs=6, rollout_len=10,
                actor_hidden=16, critic_hidden=24, central_critic=central, n_epochs=2, n_minibatches=3, seed=1234)
    base.update(kw)
    return W.scaled(W.CONFIGS[0], **base)


def split_params(cfg, p):
    out, o = {}, 0
    for name, shape in W.param_layout(cfg):
        n = int(np.prod(shape))
        out[name] = p[o:o + n].reshape(shape)
        o += n
    return out


def torch_mlp(P, prefix, x):
    h1 = torch.tanh(x @ P[prefix + ".W1"] + P[prefix + ".b1"])
    h2 = torch.tanh(h1 @ P[prefix + ".W2"] + P[prefix + ".b2"])
    return h2 @ P[prefix + ".W3"] + P[prefix + ".b3"]


def make_traj(orc, cfg, seed=0, bias_scale=0.1):
    params = W.init_params(cfg, bias_scale=bias_scale)
    s = orc.EnvState(cfg)
    orc.env_reset(cfg, s)
    tr = orc.Traj(cfg)
    orc.rollout(cfg, s, params, tr, step_offset=17)
    orc.compute_gae(cfg, tr)
    return params, tr, s


def torch_minibatch_loss(cfg, tr, P, rows):
    """The minibatch objective written with torch library pieces (Categorical, clamp), float64."""
    A, D = cfg["n_agents"], W.obs_dim(cfg)
    rows = torch.as_tensor(np.asarray(rows), dtype=torch.long)
    obs = torch.tensor(tr.obs[:-1].reshape(-1, A, D), dtype=torch.float64)[rows]          # [r][A][D]
    flat = lambda x: torch.tensor(x.reshape(-1, A), dtype=torch.float64)[rows].reshape(-1)
    action = torch.tensor(tr.action.reshape(-1, A))[rows].reshape(-1).long()
    logp_old, adv, ret, v_old = flat(tr.logp), flat(tr.adv), flat(tr.ret), flat(tr.value)
    if cfg["normalize_adv"]:
        adv = (adv - adv.mean()) / (adv.std(unbiased=False) + 1e-8)
    dist = torch.distributions.Categorical(logits=torch_mlp(P, "actor", obs.reshape(-1, D)))
    ratio = torch.exp(dist.log_prob(action) - logp_old)
    f32 = lambda k: float(np.float32(cfg[k]))     # the configuration struct carries fp32 fields
    eps = f32("clip_eps")
    l_pi = -torch.minimum(ratio * adv, torch.clamp(ratio, 1 - eps, 1 + eps) * adv).mean()
    ent = dist.entropy().mean()
    if cfg["central_critic"]:
        v = torch_mlp(P, "critic", obs.reshape(-1, A * D)).expand(-1, A).reshape(-1)
    else:
        v = torch_mlp(P, "critic", obs.reshape(-1, D)).reshape(-1)
    lv = 0.5 * (v - ret) ** 2
    if cfg["clip_value"]:
        vc = v_old + torch.clamp(v - v_old, -eps, eps)
        lv = torch.maximum(lv, 0.5 * (vc - ret) ** 2)
    l_v = lv.mean()
    return l_pi - f32("ent_coef") * ent + f32("vf_coef") * l_v, (l_pi, l_v, ent)


def test_policy_forward_matches_torch_float64(orc):
    for central in (0, 1):
        cfg = small_cfg(central)
        params = W.init_params(cfg, bias_scale=0.3)
        rng = np.random.default_rng(0)
        obs = rng.integers(0, 4, size=(50, cfg["n_agents"], W.obs_dim(cfg))).astype(np.float32)
        logits, value = orc.policy_forward(cfg, params, obs)
        P = {k: torch.tensor(v, dtype=torch.float64) for k, v in split_params(cfg, params).items()}
        x = torch.tensor(obs, dtype=torch.float64)
        ref_l = torch_mlp(P, "actor", x.reshape(-1, W.obs_dim(cfg))).reshape(50, -1, 6).numpy()
        if central:
            ref_v = torch_mlp(P, "critic", x.reshape(50, -1)).expand(-1, cfg["n_agents"]).numpy()
        else:
            ref_v = torch_mlp(P, "critic", x.reshape(-1, W.obs_dim(cfg))).reshape(50, -1).numpy()
        assert np.allclose(logits, ref_l, rtol=0, atol=2e-7 * np.abs(ref_l).max())
        assert np.allclose(value, ref_v, rtol=0, atol=2e-7 * np.abs(ref_v).max())
        assert np.abs(ref_l).max() > 0.1


def test_bf16_config_uses_rounded_weights(orc):
    cfg = small_cfg(0, precision=1)
    params = W.init_params(cfg, bias_scale=0.3)
    rounded = torch.tensor(params).to(torch.bfloat16).to(torch.float32).numpy()   # library RNE rounding
    assert np.array_equal(rounded, np.array([orc.round_bf16(x) for x in params], np.float32))
    obs = np.random.default_rng(1).integers(0, 4, size=(9, 3, 27)).astype(np.float32)
    l16, v16 = orc.policy_forward(cfg, params, obs)
    l32, v32 = orc.policy_forward(W.scaled(cfg, precision=0), rounded, obs)
    assert np.array_equal(l16, l32) and np.array_equal(v16, v32)
    lraw, _ = orc.policy_forward(W.scaled(cfg, precision=0), params, obs)
    assert not np.array_equal(lraw, l32)


class _TanhBf16(torch.autograd.Function):
    """tanh whose output, and whose gradient with respect to its input, are rounded to bf16 (torch's own casts);
    the derivative is taken from the rounded output."""

    @staticmethod
    def forward(ctx, z):
        h = torch.tanh(z).float().bfloat16().double()
        ctx.save_for_backward(h)
        return h

    @staticmethod
    def backward(ctx, g):
        (h,) = ctx.saved_tensors
        return (g * (1 - h * h)).float().bfloat16().double()


def _mlp_bf16_inputs(P, prefix, x):
    h1 = _TanhBf16.apply(x @ P[prefix + ".W1"] + P[prefix + ".b1"])
    h2 = _TanhBf16.apply(h1 @ P[prefix + ".W2"] + P[prefix + ".b2"])
    return h2 @ P[prefix + ".W3"] + P[prefix + ".b3"]


@pytest.mark.parametrize("central", [0, 1])
def test_bf16_input_rounding_mode_against_torch_casts(orc, central, monkeypatch):
    """precision 2 (weights AND the inputs of every matrix product in bf16): the forward pass and the gradient must
    equal a float64 torch evaluation with bfloat16 casts at the same points (library rounding, library autograd for
    the products), and the mode must really differ from the weights-only mode by about one bf16 rounding."""
    cfg1 = small_cfg(central, precision=1, ent_coef=0.05)
    cfg2 = W.scaled(cfg1, precision=2)
    params, tr, _ = make_traj(orc, cfg1)
    rng = np.random.default_rng(11)
    moved = (params.astype(np.float64) + 0.15 * rng.normal(size=params.size) * np.abs(params).mean()).astype(np.float32)
    p64 = torch.tensor(moved).to(torch.bfloat16).double().numpy()        # the weights as the networks see them
    rows = rng.permutation(cfg1["rollout_len"] * cfg1["n_envs"])[:24].astype(np.int32)
    stats2, grad2 = orc.minibatch_loss_grad(cfg2, tr, p64, rows)
    stats1, grad1 = orc.minibatch_loss_grad(cfg1, tr, p64, rows)
    P = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in split_params(cfg1, p64).items()}
    monkeypatch.setattr(sys.modules[__name__], "torch_mlp", _mlp_bf16_inputs)
    loss, _ = torch_minibatch_loss(cfg2, tr, P, rows)
    loss.backward()
    ref = np.concatenate([P[n].grad.reshape(-1).numpy() for n, _ in W.param_layout(cfg1)])
    assert abs(stats2[5] - loss.item()) < 1e-12 * max(1, abs(loss.item()))
    assert np.abs(grad2 - ref).max() < 1e-10 * max(1.0, np.abs(ref).max())
    # the mode is switched on and is a perturbation (one bf16 rounding, 2^-9 relative, per input of a product; the
    # value gradient is proportional to v - ret, a difference that a small change of v can move by much more)
    d = np.linalg.norm(grad2 - grad1) / np.linalg.norm(grad1)
    assert 1e-5 < d < 0.5, d
    # forward pass through the public entry point: logits and values against the same torch evaluation
    obs = rng.integers(0, 4, size=(40, cfg1["n_agents"], W.obs_dim(cfg1))).astype(np.float32)
    l2, v2 = orc.policy_forward(cfg2, moved, obs)
    with torch.no_grad():
        x = torch.tensor(obs, dtype=torch.float64)
        ref_l = _mlp_bf16_inputs(P, "actor", x.reshape(-1, W.obs_dim(cfg1))).reshape(40, -1, 6).numpy()
        ref_v = (_mlp_bf16_inputs(P, "critic", x.reshape(40, -1)).expand(-1, cfg1["n_agents"]) if central else
                 _mlp_bf16_inputs(P, "critic", x.reshape(-1, W.obs_dim(cfg1))).reshape(40, -1)).numpy()
    assert np.allclose(l2, ref_l, rtol=0, atol=2e-7 * np.abs(ref_l).max())
    assert np.allclose(v2, ref_v, rtol=0, atol=2e-7 * np.abs(ref_v).max())


def test_bf16_input_rounding_mode_is_the_weights_only_mode_on_representable_activations(orc):
    """With saturated hidden units (|pre-activation| > 20: tanh is exactly +-1 in float64, which bf16 holds) the two
    bf16 modes are the same function, bit for bit."""
    cfg1 = small_cfg(0, precision=1)
    params = W.init_params(cfg1, bias_scale=0.3)
    P = split_params(cfg1, params)
    for net in ("actor", "critic"):
        P[net + ".W1"] *= 0.0
        P[net + ".b1"][:] = np.where(np.arange(P[net + ".b1"].size) % 2 == 0, 30.0, -30.0)
        P[net + ".W2"] *= 0.0
        P[net + ".b2"][:] = np.where(np.arange(P[net + ".b2"].size) % 3 == 0, -25.0, 25.0)
    sat = np.concatenate([P[n].reshape(-1) for n, _ in W.param_layout(cfg1)]).astype(np.float32)
    obs = np.random.default_rng(2).integers(0, 4, size=(12, cfg1["n_agents"], W.obs_dim(cfg1))).astype(np.float32)
    l1, v1 = orc.policy_forward(cfg1, sat, obs)
    l2, v2 = orc.policy_forward(W.scaled(cfg1, precision=2), sat, obs)
    assert np.array_equal(l1, l2) and np.array_equal(v1, v2) and np.abs(l1).max() > 0
    # and on ordinary activations they differ
    plain = W.init_params(cfg1, bias_scale=0.3)          # (split_params hands out views: `params` is saturated now)
    l1, _ = orc.policy_forward(cfg1, plain, obs)
    l2, _ = orc.policy_forward(W.scaled(cfg1, precision=2), plain, obs)
    assert not np.array_equal(l1, l2)


def test_sampler_logp_argmax_and_frequencies(orc):
    rng = np.random.default_rng(2)
    logits = rng.normal(size=(4000, 6)).astype(np.float32) * 2
    u = rng.random((4000, 6), dtype=np.float32).clip(1e-7, 1 - 1e-7)
    action, sampled, logp, gap = orc.sample(logits, u)
    z = logits.astype(np.float64) - np.log(-np.log(u.astype(np.float64)))
    assert np.array_equal(action, z.argmax(1)) and np.array_equal(action, sampled)
    srt = np.sort(z, 1)
    assert np.allclose(gap, srt[:, -1] - srt[:, -2], rtol=1e-6, atol=1e-7)
    ref = torch.distributions.Categorical(logits=torch.tensor(logits, dtype=torch.float64)).log_prob(
        torch.tensor(action).long()).numpy()
    assert np.allclose(logp, ref, rtol=0, atol=1e-6)
    # forced actions replace the draw but the draw is still reported
    forced = rng.integers(0, 6, size=4000).astype(np.int32)
    a2, s2, lp2, _ = orc.sample(logits, u, forced)
    assert np.array_equal(a2, forced) and np.array_equal(s2, sampled)
    ref2 = torch.log_softmax(torch.tensor(logits, dtype=torch.float64), 1).numpy()[np.arange(4000), forced]
    assert np.allclose(lp2, ref2, rtol=0, atol=1e-6)
    # exact tie -> lowest index
    a3, _, _, g3 = orc.sample(np.zeros((1, 6), np.float32), np.full((1, 6), 0.5, np.float32))
    assert a3[0] == 0 and g3[0] == 0
    # Gumbel-max identity: frequencies follow softmax(logits)
    one = np.array([0.5, -1.0, 2.0, 0.0, 1.0, -3.0], np.float32)
    n = 60000
    uu = rng.random((n, 6), dtype=np.float32).clip(1e-7, 1 - 1e-7)
    aa, _, _, _ = orc.sample(np.tile(one, (n, 1)), uu)
    p = np.exp(one - one.max()); p /= p.sum()
    freq = np.bincount(aa, minlength=6) / n
    assert np.all(np.abs(freq - p) < 5 * np.sqrt(p * (1 - p) / n) + 1e-4)


def brute_gae(reward, value, done, last_value, gamma, lam):
    T, N, A = reward.shape
    v_ext = np.concatenate([value, last_value[None]], 0).astype(np.float64)
    adv = np.zeros((T, N, A))
    for t in range(T):
        for n in range(N):
            for a in range(A):
                tot, alive = 0.0, 1.0
                for l in range(T - t):
                    nd = 1.0 - done[t + l, n]
                    delta = reward[t + l, n, a] + gamma * nd * v_ext[t + l + 1, n, a] - v_ext[t + l, n, a]
                    tot += (gamma * lam) ** l * alive * delta
                    alive *= nd
                adv[t, n, a] = tot
    return adv


def fill_random_traj(orc, cfg, seed):
    rng = np.random.default_rng(seed)
    tr = orc.Traj(cfg)
    tr.reward[:] = rng.random(tr.reward.shape) * (rng.random(tr.reward.shape) < 0.3)
    tr.value[:] = rng.normal(size=tr.value.shape)
    tr.last_value[:] = rng.normal(size=tr.last_value.shape)
    tr.done[:] = rng.random(tr.done.shape) < 0.15
    return tr


def test_gae_brute_force_and_special_cases(orc):
    cfg = small_cfg(0, n_envs=5, rollout_len=12)
    tr = fill_random_traj(orc, cfg, 3)
    orc.compute_gae(cfg, tr)
    ref = brute_gae(tr.reward, tr.value, tr.done, tr.last_value, np.float32(0.99), np.float32(0.95))
    assert np.allclose(tr.adv, ref, rtol=1e-6, atol=1e-6)
    assert np.allclose(tr.ret, ref + tr.value, rtol=1e-6, atol=1e-6)
    assert tr.done.sum() > 3
    # lambda = 1: ret_t is the discounted return, cut at done, bootstrapped with last_value at the end
    c1 = W.scaled(cfg, **{"lambda": 1.0})
    orc.compute_gae(c1, tr)
    T, N, A = tr.reward.shape
    g = np.float64(np.float32(0.99))
    for n in range(N):
        for a in range(A):
            for t in range(T):
                G, disc, cut = 0.0, 1.0, False
                for k in range(t, T):
                    G += disc * tr.reward[k, n, a]
                    disc *= g
                    if tr.done[k, n]:
                        cut = True
                        break
                if not cut:
                    G += disc * tr.last_value[n, a]
                assert abs(tr.ret[t, n, a] - G) < 1e-5
    # lambda = 0: one-step TD error;  gamma = 0: reward minus value
    c0 = W.scaled(cfg, **{"lambda": 0.0})
    orc.compute_gae(c0, tr)
    v_next = np.concatenate([tr.value[1:], tr.last_value[None]], 0)
    delta = tr.reward + g * (1 - tr.done[:, :, None]) * v_next - tr.value
    assert np.allclose(tr.adv, delta, atol=1e-6)
    cg = W.scaled(cfg, gamma=0.0)
    orc.compute_gae(cg, tr)
    assert np.allclose(tr.adv, tr.reward - tr.value, atol=1e-7)


@pytest.mark.parametrize("central,norm,clipv", [(0, 1, 0), (1, 1, 0), (0, 0, 1), (1, 0, 1)])
def test_minibatch_gradient_autograd_and_finite_differences(orc, central, norm, clipv):
    cfg = small_cfg(central, normalize_adv=norm, clip_value=clipv, ent_coef=0.05)
    params, tr, _ = make_traj(orc, cfg)
    rng = np.random.default_rng(4)
    # move the parameters so that ratios leave 1 and some samples are clipped
    p64 = params.astype(np.float64) + 0.15 * rng.normal(size=params.size) * np.abs(params).mean()
    tr.value[:] += 0.3 * rng.normal(size=tr.value.shape).astype(np.float32)   # v_old differs from v_new
    rows = rng.permutation(cfg["rollout_len"] * cfg["n_envs"])[:20].astype(np.int32)
    stats, grad = orc.minibatch_loss_grad(cfg, tr, p64, rows)
    assert 0.02 < stats[4] < 0.98, stats     # clip fraction: both branches are exercised
    # library special case: float64 autograd of the same objective
    P = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in split_params(cfg, p64).items()}
    loss, (l_pi, l_v, ent) = torch_minibatch_loss(cfg, tr, P, rows)
    loss.backward()
    ref = np.concatenate([P[n].grad.reshape(-1).numpy() for n, _ in W.param_layout(cfg)])
    assert abs(stats[5] - loss.item()) < 1e-12 * max(1, abs(loss.item()))
    assert abs(stats[0] - l_pi.item()) < 1e-12 and abs(stats[1] - l_v.item()) < 1e-12
    assert abs(stats[2] - ent.item()) < 1e-12
    assert np.abs(grad - ref).max() < 1e-10 * max(1.0, np.abs(ref).max())
    assert np.abs(ref).max() > 1e-4
    # central finite differences of the oracle's own loss on a sample of coordinates
    idx = np.concatenate([rng.choice(params.size, 60, replace=False), [0, params.size - 1]])
    h = 1e-6
    for i in idx:
        pp, pm = p64.copy(), p64.copy()
        pp[i] += h
        pm[i] -= h
        lp = orc.minibatch_loss_grad(cfg, tr, pp, rows, want_grad=False)[0][5]
        lm = orc.minibatch_loss_grad(cfg, tr, pm, rows, want_grad=False)[0][5]
        fd = (lp - lm) / (2 * h)
        assert abs(fd - grad[i]) < 1e-6 * max(1.0, np.abs(grad).max()), (i, fd, grad[i])


def test_first_minibatch_is_plain_policy_gradient(orc):
    cfg = small_cfg(0, ent_coef=0.0, vf_coef=0.0)
    params, tr, _ = make_traj(orc, cfg)
    rows = np.arange(30, dtype=np.int32)
    stats, grad = orc.minibatch_loss_grad(cfg, tr, params.astype(np.float64), rows)
    assert stats[4] == 0.0 and abs(stats[3]) < 1e-12          # ratio == 1: nothing clipped, KL 0
    # at ratio 1 the gradient is -mean(A' grad logp)
    P = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in split_params(cfg, params.astype(np.float64)).items()}
    A, D = cfg["n_agents"], W.obs_dim(cfg)
    obs = torch.tensor(tr.obs[:-1].reshape(-1, A, D)[rows].reshape(-1, D), dtype=torch.float64)
    act = torch.tensor(tr.action.reshape(-1, A)[rows].reshape(-1)).long()
    adv = torch.tensor(tr.adv.reshape(-1, A)[rows].reshape(-1), dtype=torch.float64)
    adv = (adv - adv.mean()) / (adv.std(unbiased=False) + 1e-8)
    lp = torch.log_softmax(torch_mlp(P, "actor", obs), 1)[torch.arange(len(act)), act]
    (-(adv * lp).mean()).backward()
    Pa = orc.actor_param_count(cfg)
    ref = np.concatenate([P[n].grad.reshape(-1).numpy() for n, _ in W.param_layout(cfg)[:6]])
    assert np.abs(grad[:Pa] - ref).max() < 1e-6 * np.abs(ref).max()   # logp_old is stored in fp32
    assert np.all(grad[Pa:] == 0)


def test_adam_matches_torch_and_closed_form(orc):
    cfg = small_cfg(0)
    rng = np.random.default_rng(5)
    n = 300
    p0 = rng.normal(size=n).astype(np.float32)
    p, m, v = p0.copy(), np.zeros(n, np.float32), np.zeros(n, np.float32)
    tp = torch.tensor(p0.astype(np.float64), requires_grad=True)
    opt = torch.optim.Adam([tp], lr=cfg["lr"], betas=(cfg["beta1"], cfg["beta2"]), eps=cfg["adam_eps"])
    for k in range(1, 8):
        g = rng.normal(size=n) * 10.0 ** rng.integers(-6, 1, size=n)
        if k == 1:
            first = g.copy()
        orc.adam_step(cfg, p, m, v, g, k)
        tp.grad = torch.tensor(g)
        opt.step()
        if k == 1:
            lr, eps = np.float32(cfg["lr"]).astype(np.float64), np.float32(cfg["adam_eps"]).astype(np.float64)
            closed = p0 - lr * first / (np.abs(first) + eps)
            assert np.allclose(p, closed, rtol=0, atol=3e-7)   # fp32 storage of parameters
    assert np.allclose(p, tp.detach().numpy(), rtol=0, atol=1.5e-6)
    assert np.abs(p - p0).max() > 1e-3


@pytest.mark.parametrize("central,precision", [(0, 0), (1, 0), (0, 1)])
def test_ppo_update_whole_loop_against_torch(orc, central, precision):
    cfg = small_cfg(central, precision=precision, max_grad_norm=0.05)
    params, tr, _ = make_traj(orc, cfg)
    perm = W.make_perm(cfg, seed=77)
    R, E, M = cfg["rollout_len"] * cfg["n_envs"], cfg["n_epochs"], cfg["n_minibatches"]
    p = params.copy()
    m, v = np.zeros_like(p), np.zeros_like(p)
    stats, gdump = orc.ppo_update(cfg, tr, p, m, v, adam_step0=0, perm=perm)
    # reference loop: float64 autograd + library Adam on float64 master weights
    master = torch.tensor(params.astype(np.float64), requires_grad=True)
    opt = torch.optim.Adam([master], lr=cfg["lr"], betas=(cfg["beta1"], cfg["beta2"]), eps=cfg["adam_eps"])
    shapes = W.param_layout(cfg)
    it = 0
    for e in range(E):
        for mb in range(M):
            eff = master
            if precision == 1:
                eff = master + (master.detach().float().bfloat16().double() - master.detach())  # straight-through
            P, o = {}, 0
            for name, shape in shapes:
                k = int(np.prod(shape))
                P[name] = eff[o:o + k].reshape(shape)
                o += k
            rows = perm[e, mb * (R // M):(mb + 1) * (R // M)]
            opt.zero_grad()
            loss, (l_pi, l_v, ent) = torch_minibatch_loss(cfg, tr, P, rows)
            loss.backward()
            norm = master.grad.norm().item()
            master.grad.mul_(cfg["max_grad_norm"] / max(norm, cfg["max_grad_norm"]))
            assert abs(stats[it, 5] - norm) < 2e-4 * norm
            assert abs(stats[it, 6] - loss.item()) < 2e-4 * max(1, abs(loss.item()))
            assert stats[it, 7] == 0
            last_grad = master.grad.clone().numpy()
            opt.step()
            it += 1
    # fp32 storage of parameters / moments after each of the E*M steps: ~1e-7 relative drift per step
    assert np.abs(p - master.detach().numpy()).max() < 2e-5 * cfg["lr"] / 3e-4
    assert np.abs(p - params).max() > 0.5 * cfg["lr"]
    assert np.abs(gdump - last_grad).max() < 1e-3 * np.abs(last_grad).max()
    assert stats[:, 5].min() > cfg["max_grad_norm"]   # clipping active in every step
    # identity order when perm is None
    p2, m2, v2 = params.copy(), np.zeros_like(p), np.zeros_like(p)
    ident = np.tile(np.arange(R, dtype=np.int32), (E, 1))
    orc.ppo_update(cfg, tr, p2, m2, v2, perm=None)
    p3, m3, v3 = params.copy(), np.zeros_like(p), np.zeros_like(p)
    orc.ppo_update(cfg, tr, p3, m3, v3, perm=ident)
    assert np.array_equal(p2, p3)


def test_rollout_is_consistent_with_its_parts(orc):
    cfg = small_cfg(1)
    params, tr, s_after = make_traj(orc, cfg)
    T, N, A = cfg["rollout_len"], cfg["n_envs"], cfg["n_agents"]
    s = orc.EnvState(cfg)
    orc.env_reset(cfg, s)
    for t in range(T):
        assert np.array_equal(tr.obs[t], orc.observe(cfg, s))
        logits, value = orc.policy_forward(cfg, params, tr.obs[t])
        assert np.array_equal(logits, tr.logits[t]) and np.array_equal(value, tr.value[t])
        u = np.array([[orc.sample_uniforms(cfg, 17 + t, n, a) for a in range(A)] for n in range(N)])
        act, smp, logp, gap = orc.sample(logits, u)
        assert np.array_equal(act.reshape(N, A), tr.action[t]) and np.array_equal(gap.reshape(N, A), tr.gap[t])
        assert np.allclose(logp.reshape(N, A), tr.logp[t], atol=1e-6)
        _, r, d = orc.env_step(cfg, s, tr.action[t], want_obs=False)
        assert np.array_equal(r, tr.reward[t]) and np.array_equal(d, tr.done[t])
    assert np.array_equal(tr.obs[T], orc.observe(cfg, s))
    assert np.array_equal(orc.policy_forward(cfg, params, tr.obs[T])[1], tr.last_value)
    for f in orc.EnvState.FIELDS:
        assert np.array_equal(getattr(s, f), getattr(s_after, f))
    # centralised critic: one value per env
    assert np.all(tr.value == tr.value[:, :, :1])
    # forced actions and forced uniforms are honoured
    forced = W.random_actions(cfg, T, seed=9)
    fu = W.random_uniforms(cfg, T, seed=10)
    s2 = orc.EnvState(cfg)
    orc.env_reset(cfg, s2)
    tr2 = orc.Traj(cfg)
    orc.rollout(cfg, s2, params, tr2, forced_actions=forced, forced_uniforms=fu)
    assert np.array_equal(tr2.action, forced)
    a0, smp0, _, _ = orc.sample(tr2.logits[0], fu[0])
    assert np.array_equal(smp0.reshape(N, A), tr2.sampled[0])
