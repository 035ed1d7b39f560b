"""Pins for the oracle's environment: hand-built grids with hand-computed outcomes for every
rule, a declarative exhaustive check over all joint actions on tiny grids, reset invariants
and uniformity, and observation layout."""
import itertools

import numpy as np
import pytest

import workloads as W

NOOP, NORTH, SOUTH, WEST, EAST, LOAD = range(6)


def tiny(G=4, A=2, F=1, L=2, cap=25, V=3, N=1, seed=7):
    return W.scaled(W.CONFIGS[0], grid=G, n_agents=A, n_food=F, max_level=L, episode_cap=cap, view=V,
                    n_envs=N, seed=seed)


def build(orc, cfg, agents, food, t=0, env=0, state=None):
    s = state or orc.EnvState(cfg)
    for a, (r, c, l) in enumerate(agents):
        s.agent_row[a, env], s.agent_col[a, env], s.agent_lvl[a, env] = r, c, l
    for f, (r, c, l) in enumerate(food):
        s.food_row[f, env], s.food_col[f, env], s.food_lvl[f, env] = r, c, l
    s.t_in_ep[env] = t
    return s


def agents_of(s, env=0):
    return [(int(s.agent_row[a, env]), int(s.agent_col[a, env])) for a in range(s.agent_row.shape[0])]


def test_moves_and_walls(orc):
    cfg = tiny(G=4, A=2, F=1)
    s = build(orc, cfg, [(0, 0, 1), (3, 3, 2)], [(2, 0, 4)])
    _, r, d = orc.env_step(cfg, s, [[NORTH, SOUTH]])       # both into walls
    assert agents_of(s) == [(0, 0), (3, 3)] and not d[0] and np.all(r == 0)
    _, r, d = orc.env_step(cfg, s, [[EAST, WEST]])         # plain moves: east = col+1, west = col-1
    assert agents_of(s) == [(0, 1), (3, 2)]
    _, r, d = orc.env_step(cfg, s, [[SOUTH, NORTH]])       # south = row+1, north = row-1
    assert agents_of(s) == [(1, 1), (2, 2)]
    assert s.t_in_ep[0] == 3


def test_move_into_food_or_agent_blocked(orc):
    cfg = tiny(G=4, A=2, F=1)
    s = build(orc, cfg, [(1, 0, 1), (1, 1, 1)], [(2, 0, 4)])
    orc.env_step(cfg, s, [[SOUTH, WEST]])   # agent0 into food, agent1 into agent0's cell
    assert agents_of(s) == [(1, 0), (1, 1)]
    # following into a cell that is being vacated is also refused (start-of-step occupancy)
    orc.env_step(cfg, s, [[NORTH, WEST]])
    assert agents_of(s) == [(0, 0), (1, 1)]
    # a swap is refused for both
    s = build(orc, cfg, [(1, 0, 1), (1, 1, 1)], [(3, 3, 4)])
    orc.env_step(cfg, s, [[EAST, WEST]])
    assert agents_of(s) == [(1, 0), (1, 1)]


def test_head_on_collision_both_stay(orc):
    cfg = tiny(G=4, A=2, F=1)
    s = build(orc, cfg, [(1, 0, 1), (1, 2, 1)], [(3, 3, 4)])
    orc.env_step(cfg, s, [[EAST, WEST]])    # both target (1,1)
    assert agents_of(s) == [(1, 0), (1, 2)]
    # only one of them moves there: fine
    orc.env_step(cfg, s, [[EAST, NOOP]])
    assert agents_of(s) == [(1, 1), (1, 2)]


def test_three_agents_one_cell(orc):
    cfg = tiny(G=4, A=3, F=1, L=3)
    s = build(orc, cfg, [(1, 0, 1), (1, 2, 1), (0, 1, 1)], [(3, 3, 9)])
    orc.env_step(cfg, s, [[EAST, WEST, SOUTH]])
    assert agents_of(s) == [(1, 0), (1, 2), (0, 1)]


def test_load_rules_and_reward_split(orc):
    cfg = tiny(G=5, A=3, F=2, L=3)
    # food0 (lvl 3) at (2,2); agents: a0 lvl1 at (2,1), a1 lvl2 at (1,2), a2 lvl3 at (2,3); food1 far away
    s = build(orc, cfg, [(2, 1, 1), (1, 2, 2), (2, 3, 3)], [(2, 2, 3), (4, 4, 2)])
    # insufficient: only a0 (lvl 1) loads -> nothing
    _, r, d = orc.env_step(cfg, s, [[LOAD, NOOP, NOOP]])
    assert np.all(r == 0) and s.food_lvl[0, 0] == 3 and not d[0]
    # exact level: a0 + a1 = 3 -> rewards 3*1/3 and 3*2/3, non-loader adjacent a2 gets 0
    _, r, d = orc.env_step(cfg, s, [[LOAD, LOAD, NOOP]])
    assert r[0, 0] == np.float32(3 * 1) / np.float32(3)
    assert r[0, 1] == np.float32(3 * 2) / np.float32(3)
    assert r[0, 2] == 0 and s.food_lvl[0, 0] == 0 and not d[0]
    assert abs(float(r.sum()) - 3.0) < 1e-6
    # the collected food's cell is now free to walk on
    orc.env_step(cfg, s, [[EAST, NOOP, NOOP]])
    assert agents_of(s)[0] == (2, 2)


def test_overshoot_load_shares_food_level(orc):
    cfg = tiny(G=5, A=3, F=2, L=3)
    s = build(orc, cfg, [(2, 1, 1), (1, 2, 2), (2, 3, 3)], [(2, 2, 3), (4, 4, 2)])
    _, r, _ = orc.env_step(cfg, s, [[LOAD, LOAD, LOAD]])   # summed level 6 >= 3
    exp = [np.float32(3 * l) / np.float32(6) for l in (1, 2, 3)]
    assert list(r[0]) == exp


def test_diagonal_is_not_adjacent_and_load_far_is_noop(orc):
    cfg = tiny(G=5, A=2, F=1, L=3)
    s = build(orc, cfg, [(1, 1, 3), (4, 4, 3)], [(2, 2, 1)])
    _, r, d = orc.env_step(cfg, s, [[LOAD, LOAD]])
    assert np.all(r == 0) and s.food_lvl[0, 0] == 1 and agents_of(s) == [(1, 1), (4, 4)]


def test_agent_adjacent_to_two_foods_loads_both(orc):
    cfg = tiny(G=5, A=2, F=3, L=3)
    # a0 lvl 3 at (2,2) between food0 (2,1) lvl 2 and food1 (2,3) lvl 3; food2 far (keeps episode alive)
    s = build(orc, cfg, [(2, 2, 3), (0, 0, 1)], [(2, 1, 2), (2, 3, 3), (4, 4, 6)])
    _, r, d = orc.env_step(cfg, s, [[LOAD, NOOP]])
    assert r[0, 0] == np.float32(2.0) + np.float32(3.0) and r[0, 1] == 0
    assert list(s.food_lvl[:, 0]) == [0, 0, 6] and not d[0]


def test_last_food_collected_done_and_reset(orc):
    cfg = tiny(G=4, A=2, F=1, L=2, seed=11)
    s = build(orc, cfg, [(1, 1, 2), (3, 3, 1)], [(1, 2, 2)], t=4)
    s.episode_id[0] = 5
    obs, r, d = orc.env_step(cfg, s, [[LOAD, NOOP]])
    assert d[0] == 1 and r[0, 0] == 2.0 and r[0, 1] == 0.0
    assert s.episode_id[0] == 6 and s.t_in_ep[0] == 0
    # the new layout is that of (seed, env 0, episode 6), whatever happened before
    fresh = orc.EnvState(cfg)
    orc.env_reset(cfg, fresh)
    fresh.episode_id[0] = 5
    fresh2 = build(orc, cfg, [(0, 0, 1), (0, 1, 1)], [(0, 2, 1)], state=fresh)
    orc.env_step(cfg, fresh2, [[NOOP, LOAD]])   # agent1 lvl1 adjacent to food lvl1 -> done
    for f in orc.EnvState.FIELDS:
        assert np.array_equal(getattr(s, f), getattr(fresh2, f)), f
    # the observation returned is the new episode's first
    assert np.array_equal(obs, orc.observe(cfg, s))


def test_cap_reached_done_and_reset(orc):
    cfg = tiny(G=4, A=2, F=1, cap=3)
    s = build(orc, cfg, [(0, 0, 1), (3, 3, 1)], [(1, 2, 4)])
    for t in range(2):
        _, _, d = orc.env_step(cfg, s, [[NOOP, NOOP]])
        assert d[0] == 0 and s.t_in_ep[0] == t + 1
    _, _, d = orc.env_step(cfg, s, [[NOOP, NOOP]])
    assert d[0] == 1 and s.t_in_ep[0] == 0 and s.episode_id[0] == 1


def _declarative_check(cfg, before, actions, after, reward, done):
    """Checks one transition against the rules stated as predicates over sets (no stepping)."""
    G, A, F = cfg["grid"], cfg["n_agents"], cfg["n_food"]
    pos = [(int(before.agent_row[a, 0]), int(before.agent_col[a, 0])) for a in range(A)]
    lvl = [int(before.agent_lvl[a, 0]) for a in range(A)]
    food = {(int(before.food_row[f, 0]), int(before.food_col[f, 0])): (f, int(before.food_lvl[f, 0]))
            for f in range(F) if before.food_lvl[f, 0]}
    delta = {NOOP: (0, 0), NORTH: (-1, 0), SOUTH: (1, 0), WEST: (0, -1), EAST: (0, 1), LOAD: (0, 0)}
    want = [(p[0] + delta[a][0], p[1] + delta[a][1]) for p, a in zip(pos, actions)]
    occupied = set(pos) | set(food)
    valid = [w != p and 0 <= w[0] < G and 0 <= w[1] < G and w not in occupied for w, p in zip(want, pos)]
    contested = {w for i, w in enumerate(want) if valid[i] and sum(1 for j in range(A) if valid[j] and want[j] == w) > 1}
    exp_pos = [want[i] if valid[i] and want[i] not in contested else pos[i] for i in range(A)]
    exp_rew = [np.float32(0)] * A
    eaten = set()
    for cell, (f, fl) in sorted(food.items(), key=lambda kv: kv[1][0]):
        loaders = [i for i in range(A) if actions[i] == LOAD and abs(pos[i][0] - cell[0]) + abs(pos[i][1] - cell[1]) == 1]
        tot = sum(lvl[i] for i in loaders)
        if tot >= fl:
            eaten.add(f)
            for i in loaders:
                exp_rew[i] = np.float32(exp_rew[i] + np.float32(fl * lvl[i]) / np.float32(tot))
    exp_done = (len(eaten) == len(food)) or (before.t_in_ep[0] + 1 == cfg["episode_cap"])
    assert bool(done[0]) == exp_done
    assert [np.float32(x) for x in reward[0]] == exp_rew
    if not exp_done:
        assert agents_of(after) == exp_pos
        assert len(set(exp_pos)) == A
        for f in range(F):
            assert after.food_lvl[f, 0] == (0 if f in eaten else before.food_lvl[f, 0])
        assert after.t_in_ep[0] == before.t_in_ep[0] + 1


@pytest.mark.parametrize("G,A,F,L", [(3, 2, 1, 2), (3, 3, 2, 2), (4, 3, 2, 3)])
def test_all_joint_actions_on_tiny_grids(orc, G, A, F, L):
    cfg = tiny(G=G, A=A, F=F, L=L, cap=1000, seed=100 + G * 10 + A)
    base = orc.EnvState(cfg)
    orc.env_reset(cfg, base)
    rng = np.random.default_rng(5)
    for layout in range(12):
        # diversify the layout: a few more random moves (never 'load') from the previous one
        for _ in range(layout):
            orc.env_step(cfg, base, rng.integers(0, 5, size=(1, A)))
        for joint in itertools.product(range(6), repeat=A):
            s = base.copy()
            _, r, d = orc.env_step(cfg, s, [list(joint)])
            _declarative_check(cfg, base, joint, s, r, d)


def test_no_overlap_invariant_random_walk(orc):
    cfg = W.scaled(W.CONFIGS[1], n_envs=256)
    s = orc.EnvState(cfg)
    orc.env_reset(cfg, s)
    acts = W.random_actions(cfg, 400, seed=3)
    G = cfg["grid"]
    total_done = 0
    for t in range(400):
        _, r, d = orc.env_step(cfg, s, acts[t], want_obs=False)
        cells = s.agent_row.astype(int) * G + s.agent_col
        fcells = np.where(s.food_lvl > 0, s.food_row.astype(int) * G + s.food_col, -1 - np.arange(3)[:, None])
        allc = np.concatenate([cells, fcells], 0)
        srt = np.sort(allc, 0)
        assert np.all(srt[1:] != srt[:-1])
        assert s.agent_row.max() < G and s.agent_col.max() < G
        assert np.all((r >= 0))
        total_done += int(d.sum())
    assert total_done > 0


def test_reset_invariants_and_key_independence(orc):
    cfg = W.scaled(W.CONFIGS[3], n_envs=512)   # 8 agents: food level bounded by the four strongest
    s = orc.EnvState(cfg)
    orc.env_reset(cfg, s)
    G = cfg["grid"]
    cells = np.concatenate([s.agent_row.astype(int) * G + s.agent_col, s.food_row.astype(int) * G + s.food_col])
    srt = np.sort(cells, 0)
    assert np.all(srt[1:] != srt[:-1]) and cells.max() < G * G
    assert s.agent_lvl.min() >= 1 and s.agent_lvl.max() <= cfg["max_level"]
    top4 = np.sort(s.agent_lvl.astype(int), 0)[-4:].sum(0)
    assert np.all(s.food_lvl >= 1) and np.all(s.food_lvl <= top4[None, :])
    assert np.any(s.food_lvl == top4[None, :])
    assert np.all(s.t_in_ep == 0) and np.all(s.episode_id == 0)
    # layout of env n does not depend on how many envs there are
    small = W.scaled(cfg, n_envs=16)
    s2 = orc.EnvState(small)
    orc.env_reset(small, s2)
    for f in ("agent_row", "agent_col", "agent_lvl", "food_row", "food_col", "food_lvl"):
        assert np.array_equal(getattr(s, f)[:, :16], getattr(s2, f))
    # another seed gives another layout
    s3 = orc.EnvState(small)
    orc.env_reset(W.scaled(small, seed=cfg["seed"] + 1), s3)
    assert not np.array_equal(s3.agent_row, s2.agent_row)


def test_reset_cells_uniform(orc):
    cfg = tiny(G=4, A=2, F=1, N=6000, seed=99)
    s = orc.EnvState(cfg)
    orc.env_reset(cfg, s)
    N = cfg["n_envs"]
    for arr_r, arr_c in ((s.agent_row[0], s.agent_col[0]), (s.agent_row[1], s.agent_col[1]), (s.food_row[0], s.food_col[0])):
        hist = np.bincount(arr_r.astype(int) * 4 + arr_c, minlength=16)
        chi2 = ((hist - N / 16) ** 2 / (N / 16)).sum()
        assert chi2 < 45, hist   # 15 dof
    # ordered pairs (agent0 cell, agent1 cell) uniform over the 240 distinct pairs
    pair = (s.agent_row[0].astype(int) * 4 + s.agent_col[0]) * 16 + s.agent_row[1].astype(int) * 4 + s.agent_col[1]
    hist = np.bincount(pair, minlength=256)
    diag = hist.reshape(16, 16).diagonal()
    assert diag.sum() == 0
    off = hist.reshape(16, 16)[~np.eye(16, dtype=bool)]
    chi2 = ((off - N / 240) ** 2 / (N / 240)).sum()
    assert chi2 < 330   # 239 dof, p ~ 1e-4
    lv = np.bincount(s.agent_lvl.reshape(-1), minlength=3)
    assert lv[0] == 0 and abs(lv[1] - N) < 5 * np.sqrt(2 * N * 0.25)


def test_observation_hand_built(orc):
    cfg = tiny(G=4, A=2, F=1, L=3, V=3)
    s = build(orc, cfg, [(0, 0, 2), (1, 1, 3)], [(0, 1, 5)])
    obs = orc.observe(cfg, s)[0]          # [A][27], index ((dy+1)*3 + (dx+1))*3 + ch
    o0 = obs[0].reshape(3, 3, 3)
    # agent 0 at the corner: row above and column left are wall
    assert np.array_equal(o0[:, :, 2], [[1, 1, 1], [1, 0, 0], [1, 0, 0]])
    assert o0[1, 1, 0] == 2                       # own level at the centre
    assert o0[1, 2, 1] == 5 and o0[1, 2, 0] == 0  # food to the east
    assert o0[2, 2, 0] == 3                       # other agent to the south-east
    assert o0[:, :, 0].sum() == 5 and o0[:, :, 1].sum() == 5
    o1 = obs[1].reshape(3, 3, 3)
    assert np.all(o1[:, :, 2] == 0)
    assert o1[1, 1, 0] == 3 and o1[0, 0, 0] == 2 and o1[0, 1, 1] == 5
    # eaten food disappears
    s.food_lvl[0, 0] = 0
    assert orc.observe(cfg, s)[0][:, 1::3].sum() == 0


@pytest.mark.parametrize("k", [1, 2, 3])
def test_observation_wall_count_closed_form(orc, k):
    cfg = W.scaled(W.CONFIGS[k], n_envs=200)
    s = orc.EnvState(cfg)
    orc.env_reset(cfg, s)
    obs = orc.observe(cfg, s)
    G, V = cfg["grid"], cfg["view"]
    h = (V - 1) // 2
    r = s.agent_row.T.astype(int)
    c = s.agent_col.T.astype(int)
    inside_r = np.minimum(r + h, G - 1) - np.maximum(r - h, 0) + 1
    inside_c = np.minimum(c + h, G - 1) - np.maximum(c - h, 0) + 1
    walls = obs[:, :, 2::3].sum(-1)
    assert np.array_equal(walls, V * V - inside_r * inside_c)
    centre = (h * V + h) * 3
    assert np.array_equal(obs[:, :, centre], s.agent_lvl.T.astype(np.float32))
    assert set(np.unique(obs)) <= {0.0, 1.0, 2.0, 3.0, 4.0, 5.0, 6.0, 7.0, 8.0, 9.0, 10.0, 11.0, 12.0}
