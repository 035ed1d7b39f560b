"""Pins of the oracle's recurrent (GRU) networks and their sequence PPO update.

(i) one step against torch.nn.GRUCell in float64 (a library routine of the same published cell);
(ii) the feed-forward special case: with the update gate shut and no hidden-to-hidden weights the cell is a
     second tanh layer, so the recurrent oracle must reproduce the (separately pinned) feed-forward oracle;
(iii) loss and back-propagation through time against float64 autograd over the same sequences, episode
      boundaries included, and against central finite differences;
(iv) reset semantics: nothing after an episode boundary depends on the hidden state before it;
(v) the optimiser loop against the separately pinned Adam step.
"""
import numpy as np
import pytest
import torch

import workloads as W


def blocks(cfg, params):
    out, off = {}, 0
    for name, shape in W.param_layout(cfg):
        n = int(np.prod(shape))
        out[name] = params[off:off + n].reshape(shape)
        off += n
    return out


def small_rec(central, **kw):
    base = dict(n_envs=5, rollout_len=7, actor_hidden=32, critic_hidden=32, central_critic=central, recurrent=1,
                n_minibatches=1, n_epochs=1, episode_cap=3, grid=5, n_agents=2, n_food=1, view=3, max_level=2,
                precision=0)
    base.update(kw)
    return W.scaled(W.CONFIGS[0], **base)


def torch_cell(b, prefix, x, h):
    f = lambda k: torch.tensor(b[prefix + "." + k], dtype=torch.float64)
    H = b[prefix + ".be"].shape[0]
    cell = torch.nn.GRUCell(H, H).double()
    with torch.no_grad():
        cell.weight_ih.copy_(f("Wi").t())
        cell.weight_hh.copy_(f("Wh").t())
        cell.bias_ih.copy_(f("bi"))
        cell.bias_hh.copy_(f("bh"))
    e = torch.tanh(x @ f("We") + f("be"))
    h2 = cell(e, h)
    return h2 @ f("W3") + f("b3"), h2


@pytest.mark.parametrize("central", [0, 1])
def test_one_step_matches_torch_grucell(orc, central):
    cfg = small_rec(central)
    rng = np.random.default_rng(3)
    params = W.init_params(cfg, bias_scale=0.3)
    A, D, Ha, Hc = cfg["n_agents"], W.obs_dim(cfg), cfg["actor_hidden"], cfg["critic_hidden"]
    rows = 6
    obs = rng.integers(0, 3, size=(rows, A, D)).astype(np.float32)
    ha = rng.normal(size=(rows, A, Ha)).astype(np.float32) * 0.5
    hc = rng.normal(size=(rows, Hc) if central else (rows, A, Hc)).astype(np.float32) * 0.5
    logits, value, ha2, hc2 = orc.rec_policy_step(cfg, params, obs, ha, hc)
    b = blocks(cfg, params)
    tl, th = torch_cell(b, "actor", torch.tensor(obs.reshape(rows * A, D), dtype=torch.float64),
                        torch.tensor(ha.reshape(rows * A, Ha), dtype=torch.float64))
    assert np.allclose(logits.reshape(rows * A, -1), tl.detach().numpy(), atol=2e-6)
    assert np.allclose(ha2.reshape(rows * A, Ha), th.detach().numpy(), atol=2e-6)
    xc = obs.reshape(rows, A * D) if central else obs.reshape(rows * A, D)
    tv, tch = torch_cell(b, "critic", torch.tensor(xc, dtype=torch.float64),
                         torch.tensor(hc.reshape(-1, Hc), dtype=torch.float64))
    v = tv.detach().numpy()[:, 0]
    assert np.allclose(value, np.repeat(v, A).reshape(rows, A) if central else v.reshape(rows, A), atol=2e-6)
    assert np.allclose(hc2.reshape(-1, Hc), tch.detach().numpy(), atol=2e-6)


def test_shut_update_gate_reduces_to_the_feed_forward_network(orc):
    cfg_r = small_rec(0)
    cfg_f = W.scaled(cfg_r, recurrent=0)
    pf = W.init_params(cfg_f, bias_scale=0.2)
    bf = blocks(cfg_f, pf)
    parts = []
    for net in ("actor", "critic"):
        H = bf[net + ".b1"].shape[0]
        Wi = np.zeros((H, 3 * H), np.float32)
        Wi[:, 2 * H:] = bf[net + ".W2"]
        bi = np.zeros(3 * H, np.float32)
        bi[H:2 * H] = -60.0                      # update gate z = sigma(-60): the old state is dropped
        bi[2 * H:] = bf[net + ".b2"]
        parts += [bf[net + ".W1"].ravel(), bf[net + ".b1"], Wi.ravel(), bi, np.zeros(H * 3 * H, np.float32),
                  np.zeros(3 * H, np.float32), bf[net + ".W3"].ravel(), bf[net + ".b3"]]
    pr = np.concatenate(parts).astype(np.float32)
    assert pr.size == W.param_count(cfg_r)
    rng = np.random.default_rng(5)
    A, D = cfg_r["n_agents"], W.obs_dim(cfg_r)
    obs = rng.integers(0, 3, size=(9, A, D)).astype(np.float32)
    ha = rng.normal(size=(9, A, cfg_r["actor_hidden"])).astype(np.float32)
    hc = rng.normal(size=(9, A, cfg_r["critic_hidden"])).astype(np.float32)
    lr, vr, _, _ = orc.rec_policy_step(cfg_r, pr, obs, ha, hc)
    lf, vf = orc.policy_forward(cfg_f, pf, obs)
    assert np.allclose(lr, lf, atol=1e-6) and np.allclose(vr, vf, atol=1e-6)


def rec_traj(orc, cfg, seed=0):
    params = W.init_params(cfg, bias_scale=0.2)
    s = orc.EnvState(cfg)
    orc.env_reset(cfg, s)
    tr, rec = orc.Traj(cfg), orc.RecState(cfg)
    rng = np.random.default_rng(seed)
    rec.ha0[:] = 0.3 * rng.normal(size=rec.ha0.shape)
    rec.hc0[:] = 0.3 * rng.normal(size=rec.hc0.shape)
    orc.rec_rollout(cfg, s, params, tr, rec, step_offset=11)
    orc.compute_gae(cfg, tr)
    return params, tr, rec


def torch_sequence_loss(cfg, tr, rec, params64, envs):
    """The same loss written with torch float64 ops; returns (stats dict, gradient)."""
    b = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in blocks(cfg, params64).items()}
    T, A, D = cfg["rollout_len"], cfg["n_agents"], W.obs_dim(cfg)
    central = cfg["central_critic"]
    t64 = lambda x: torch.tensor(np.asarray(x), dtype=torch.float64)
    obs, adv = t64(tr.obs[:, envs]), t64(tr.adv[:, envs])
    ret, v_old, logp_old = t64(tr.ret[:, envs]), t64(tr.value[:, envs]), t64(tr.logp[:, envs])
    act = torch.tensor(tr.action[:, envs].astype(np.int64))
    done = t64(tr.done[:, envs])
    if cfg["normalize_adv"]:
        adv = (adv - adv.mean()) / (adv.std(unbiased=False) + 1e-8)

    def cell(prefix, x, h):
        H = h.shape[-1]
        e = torch.tanh(x @ b[prefix + ".We"] + b[prefix + ".be"])
        gi = e @ b[prefix + ".Wi"] + b[prefix + ".bi"]
        gh = h @ b[prefix + ".Wh"] + b[prefix + ".bh"]
        r = torch.sigmoid(gi[..., :H] + gh[..., :H])
        z = torch.sigmoid(gi[..., H:2 * H] + gh[..., H:2 * H])
        n = torch.tanh(gi[..., 2 * H:] + r * gh[..., 2 * H:])
        h2 = (1 - z) * n + z * h
        return h2 @ b[prefix + ".W3"] + b[prefix + ".b3"], h2

    ha, hc = t64(rec.ha0[envs]), t64(rec.hc0[envs])
    f32 = lambda k: float(np.float32(cfg[k]))   # the configuration struct carries fp32 constants
    eps = f32("clip_eps")
    pi, vl, ent, kl, cf = 0, 0, 0, 0, 0
    B = len(envs) * T * A
    for t in range(T):
        if t > 0:
            keep = 1 - done[t - 1]
            ha = ha * keep[:, None, None]
            hc = hc * (keep[:, None] if central else keep[:, None, None])
        logits, ha = cell("actor", obs[t], ha)
        xc = obs[t].reshape(len(envs), A * D) if central else obs[t]
        v, hc = cell("critic", xc, hc)
        v = v[..., 0]
        if central:
            v = v[:, None].expand(-1, A)
        lp = torch.log_softmax(logits, -1)
        p = lp.exp()
        H = -(p * lp).sum(-1)
        lpa = torch.gather(lp, -1, act[t][..., None])[..., 0]
        log_ratio = lpa - logp_old[t]
        ratio = log_ratio.exp()
        s1, s2 = ratio * adv[t], ratio.clamp(1 - eps, 1 + eps) * adv[t]
        pi = pi - torch.minimum(s1, s2).sum() / B
        ent = ent + H.sum() / B
        kl = kl + ((ratio - 1) - log_ratio).sum() / B
        cf = cf + ((ratio - 1).abs() > eps).double().sum() / B
        vl = vl + (0.5 * (v - ret[t]) ** 2).sum() / B
    total = pi - f32("ent_coef") * ent + f32("vf_coef") * vl
    total.backward()
    grad = np.concatenate([b[name].grad.numpy().ravel() for name, _ in W.param_layout(cfg)])
    return dict(pi=pi.item(), v=vl.item(), ent=ent.item(), kl=kl.item(), cf=cf.item(), total=total.item()), grad


@pytest.mark.parametrize("central", [0, 1])
def test_sequence_loss_and_bptt_match_autograd(orc, central):
    cfg = small_rec(central)
    params, tr, rec = rec_traj(orc, cfg)
    assert tr.done.sum() > 3 and tr.done[:-1].sum() > 0          # episode boundaries inside the sequences
    rng = np.random.default_rng(8)
    p64 = params.astype(np.float64) + 0.05 * rng.normal(size=params.size)
    tr.logp[:] += rng.choice([-0.4, 0.0, 0.0, 0.4], size=tr.logp.shape).astype(np.float32)
    envs = np.array([3, 0, 4], np.int32)
    stats, grad = orc.rec_minibatch_loss_grad(cfg, tr, rec, p64, envs)
    ts, tg = torch_sequence_loss(cfg, tr, rec, p64, envs)
    for i, k in enumerate(("pi", "v", "ent", "kl", "cf", "total")):
        assert abs(stats[i] - ts[k]) < 1e-10 * max(1.0, abs(ts[k])), k
    assert 0 < stats[4] < 1
    assert np.abs(grad - tg).max() < 1e-10 * max(1.0, np.abs(tg).max())
    assert np.abs(tg).max() > 1e-4
    # central finite differences on a few parameters of every block
    off = 0
    for name, shape in W.param_layout(cfg):
        n = int(np.prod(shape))
        for i in rng.choice(n, size=min(2, n), replace=False) + off:
            h = 1e-6
            pp, pm = p64.copy(), p64.copy()
            pp[i] += h
            pm[i] -= h
            fp, _ = orc.rec_minibatch_loss_grad(cfg, tr, rec, pp, envs, want_grad=False)
            fm, _ = orc.rec_minibatch_loss_grad(cfg, tr, rec, pm, envs, want_grad=False)
            assert abs((fp[5] - fm[5]) / (2 * h) - grad[i]) < 1e-6 * max(1.0, abs(grad[i])), name
        off += n


def two_rollouts(orc, cfg):
    params = W.init_params(cfg, bias_scale=0.2)
    runs = []
    for scale in (0.0, 1.0):
        s = orc.EnvState(cfg)
        orc.env_reset(cfg, s)
        tr, rec = orc.Traj(cfg), orc.RecState(cfg)
        rec.ha0[:] = scale
        rec.hc0[:] = -scale
        forced = W.random_actions(cfg, cfg["rollout_len"], seed=4, p_load=0.4)
        orc.rec_rollout(cfg, s, params, tr, rec, step_offset=0, forced_actions=forced)
        runs.append((tr, rec))
    return runs


def test_nothing_after_an_episode_boundary_depends_on_the_state_before_it(orc):
    (t0, r0), (t1, r1) = two_rollouts(orc, small_rec(0, n_envs=16, rollout_len=9, episode_cap=12))
    assert np.array_equal(t0.done, t1.done)                      # forced actions: identical environment histories
    after = np.cumsum(t0.done, axis=0) - t0.done > 0             # [T][N]: steps after the first boundary of the env
    assert after.any() and (~after).any()
    assert np.array_equal(t0.logits[after], t1.logits[after]) and np.array_equal(t0.value[after], t1.value[after])
    assert not np.array_equal(t0.logits[~after], t1.logits[~after])
    ended = t0.done.any(axis=0)
    assert ended.any() and (~ended).any()
    assert np.array_equal(r0.ha1[ended], r1.ha1[ended]) and np.array_equal(r0.hc1[ended], r1.hc1[ended])
    assert not np.array_equal(r0.ha1[~ended], r1.ha1[~ended])
    # a boundary at the last step: the next rollout starts from the zero state
    (t0, r0), _ = two_rollouts(orc, small_rec(1, n_envs=6, rollout_len=9, episode_cap=9))
    last = t0.done[-1].astype(bool)
    assert last.any() and np.all(r0.ha1[last] == 0) and np.all(r0.hc1[last] == 0)
    assert np.all(np.abs(r0.ha1[~last]).max(axis=(1, 2)) > 0) if (~last).any() else True


def test_update_loop_is_the_pinned_adam_step_on_the_sequence_gradient(orc):
    cfg = small_rec(1, n_envs=6, n_minibatches=3, n_epochs=2)
    params, tr, rec = rec_traj(orc, cfg)
    perm = W.make_env_perm(cfg, seed=2)
    p, m, v = params.copy(), np.zeros_like(params), np.zeros_like(params)
    stats, last_grad = orc.rec_ppo_update(cfg, tr, rec, p, m, v, adam_step0=5, perm=perm)
    q, qm, qv = params.copy(), np.zeros_like(params), np.zeros_like(params)
    k = 5
    for e in range(2):
        for mb in range(3):
            envs = perm[e, mb * 2:(mb + 1) * 2]
            st, g = orc.rec_minibatch_loss_grad(cfg, tr, rec, q.astype(np.float64), envs)
            norm = np.sqrt((g * g).sum())
            g = g * (cfg["max_grad_norm"] / max(norm, cfg["max_grad_norm"]))
            k += 1
            orc.adam_step(cfg, q, qm, qv, g, k)
            row = stats[e * 3 + mb]
            assert abs(row[0] - st[0]) < 1e-6 and abs(row[5] - norm) < 1e-6 * max(1, norm) and row[7] == 0
    assert np.array_equal(p, q) and np.array_equal(m, qm) and np.array_equal(v, qv)
    assert np.allclose(last_grad, g, atol=1e-7)
