"""Pins of the oracle's greedy evaluation block.

The loop is pinned by (i) closed forms for policies whose greedy action is known in advance, (ii) a step-by-step
re-statement in Python that uses only the separately pinned single-step functions (observe / policy_forward /
env_step) and keeps its own books, and (iii) invariants of the bookkeeping.
"""
import numpy as np

import workloads as W


def fresh_state(orc, cfg):
    s = orc.EnvState(cfg)
    orc.env_reset(cfg, s)
    return s


def constant_policy(cfg, action):
    """Parameters whose logits do not depend on the observation: zero weights, output bias favouring `action`."""
    P = W.param_count(cfg)
    p = np.zeros(P, np.float32)
    off = 0
    for name, shape in W.param_layout(cfg):
        if name == "actor.b3":
            p[off + action] = 1.0
        off += int(np.prod(shape))
    return p


def test_noop_policy_runs_every_episode_to_the_cap(orc):
    cfg = W.scaled(W.CONFIGS[1], n_envs=17, n_minibatches=1, episode_cap=9)
    E = 3
    ret, length, eps, gap = orc.evaluate(cfg, fresh_state(orc, cfg), constant_policy(cfg, 0), E)
    assert np.all(eps == E) and np.all(length == E * 9) and np.all(ret == 0.0)
    assert np.allclose(gap, 1.0)          # bias 1 against 0: the two largest logits differ by exactly 1


def test_all_zero_parameters_tie_to_the_lowest_index(orc):
    cfg = W.scaled(W.CONFIGS[0], n_envs=5, n_minibatches=1, episode_cap=7)
    p = np.zeros(W.param_count(cfg), np.float32)
    ret, length, eps, gap = orc.evaluate(cfg, fresh_state(orc, cfg), p, 2)
    assert np.all(length == 14) and np.all(ret == 0.0) and np.all(gap == 0.0)   # exact ties -> action 0 (stay)


def test_always_load_collects_only_adjacent_food(orc):
    """Everybody always loads and nobody moves: the return of an environment is the total level of the foods its
    initial layout lets the adjacent agents lift, summed over the episodes; every episode runs to the cap unless
    all food goes in the first step."""
    cfg = W.scaled(W.CONFIGS[1], n_envs=64, n_minibatches=1, episode_cap=6, grid=5)
    E = 4
    s = fresh_state(orc, cfg)
    ret, length, eps, _ = orc.evaluate(cfg, s.copy(), constant_policy(cfg, 5), E)
    A, F, N = cfg["n_agents"], cfg["n_food"], cfg["n_envs"]
    # independent bookkeeping on fresh layouts episode by episode: layouts depend on (seed, env, episode) only
    exp_ret, exp_len = np.zeros(N), np.zeros(N, np.int64)
    cur = s.copy()
    act = np.full((N, A), 5, np.int32)
    done_eps = np.zeros(N, np.int64)
    for t in range(E * cfg["episode_cap"]):
        ar, ac, al = cur.agent_row.copy(), cur.agent_col.copy(), cur.agent_lvl.copy()
        fr, fc, fl = cur.food_row.copy(), cur.food_col.copy(), cur.food_lvl.copy()
        _, reward, done = orc.env_step(cfg, cur, act, want_obs=False)
        for n in range(N):
            if done_eps[n] >= E:
                continue
            lifted = 0
            for f in range(F):
                if fl[f, n] == 0:
                    continue
                adj = [a for a in range(A) if abs(int(ar[a, n]) - int(fr[f, n])) + abs(int(ac[a, n]) - int(fc[f, n])) == 1]
                if adj and sum(int(al[a, n]) for a in adj) >= fl[f, n]:
                    lifted += int(fl[f, n])
            assert abs(float(reward[n].sum()) - lifted) < 1e-5      # loaders share exactly the food level
            exp_ret[n] += lifted
            exp_len[n] += 1
            done_eps[n] += int(done[n])
    assert np.allclose(ret, exp_ret, atol=1e-4)
    assert np.array_equal(length, exp_len) and np.all(eps == E)
    assert ret.sum() > 0


def test_evaluate_matches_a_step_by_step_restatement(orc):
    for k, E in ((0, 3), (2, 2)):
        cfg = W.scaled(W.CONFIGS[k], n_envs=12, n_minibatches=1, episode_cap=8)
        params = W.init_params(cfg, bias_scale=0.3)
        s = fresh_state(orc, cfg)
        ret, length, eps, gap = orc.evaluate(cfg, s.copy(), params, E)
        N, A = cfg["n_envs"], cfg["n_agents"]
        cur = s.copy()
        r_sum, l_sum, e_cnt = np.zeros(N, np.float32), np.zeros(N, np.int32), np.zeros(N, np.int32)
        g_min = np.full(N, np.inf, np.float32)
        for t in range(E * cfg["episode_cap"]):
            obs = orc.observe(cfg, cur)
            logits, _ = orc.policy_forward(cfg, params, obs)
            act = np.argmax(logits, axis=-1).astype(np.int32)          # numpy: first index on ties
            srt = np.sort(logits, axis=-1)
            step_gap = (srt[..., -1] - srt[..., -2]).min(axis=-1)
            _, reward, done = orc.env_step(cfg, cur, act, want_obs=False)
            on = e_cnt < E
            team = np.zeros(N, np.float32)
            for a in range(A):
                team = (team + reward[:, a]).astype(np.float32)
            r_sum = np.where(on, (r_sum + team).astype(np.float32), r_sum)
            l_sum = np.where(on, l_sum + 1, l_sum)
            g_min = np.where(on, np.minimum(g_min, step_gap), g_min)
            e_cnt = np.where(on, e_cnt + done.astype(np.int32), e_cnt)
        assert np.array_equal(ret.view(np.uint32), r_sum.view(np.uint32))
        assert np.array_equal(length, l_sum) and np.array_equal(eps, e_cnt) and np.all(eps == E)
        assert np.array_equal(gap, g_min)
        assert np.all(length >= E) and np.all(length <= E * cfg["episode_cap"])
