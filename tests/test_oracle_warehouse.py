"""Pins of the oracle's warehouse world: hand-built situations for every rule, invariants over long random runs,
and an independent set-based re-statement of the step in Python compared state for state."""
import numpy as np
import pytest

import workloads as W


def wh_cfg(kind=1, **kw):
    base = dict(W.CONFIGS[0], grid=6, n_agents=2, n_food=3, max_level=2, episode_cap=50, view=3, n_envs=1,
                n_minibatches=1, rollout_len=4, env_kind=kind)
    base.update(kw)
    return base


def set_state(orc, cfg, robots, shelves, env=0, state=None):
    """robots: [(row, col, carried shelf index or None)], shelves: [(row, col, requested)]"""
    s = state or orc.EnvState(cfg)
    for a, (r, c, carry) in enumerate(robots):
        s.agent_row[a, env], s.agent_col[a, env] = r, c
        s.agent_lvl[a, env] = 0 if carry is None else carry + 1
    for f, (r, c, req) in enumerate(shelves):
        s.food_row[f, env], s.food_col[f, env] = r, c
        s.food_lvl[f, env] = 2 if req else 1
    return s


def step(orc, cfg, s, actions):
    obs, rew, done = orc.env_step(cfg, s, np.array([actions], np.int32))
    return obs[0], rew[0], int(done[0])


def test_unloaded_robot_passes_under_a_shelf_and_loaded_one_is_blocked_by_it(orc):
    cfg = wh_cfg()
    s = set_state(orc, cfg, [(2, 2, None), (4, 4, 0)], [(4, 4, False), (2, 3, False), (4, 5, True)])
    _, rew, done = step(orc, cfg, s, [4, 4])      # both east: robot 0 under shelf 1, robot 1 (loaded) into shelf 2
    assert (s.agent_row[0, 0], s.agent_col[0, 0]) == (2, 3)
    assert (s.agent_row[1, 0], s.agent_col[1, 0]) == (4, 4) and (s.food_row[0, 0], s.food_col[0, 0]) == (4, 4)
    assert np.all(rew == 0) and done == 0


def test_carried_shelf_travels_with_its_robot_and_walls_stop_moves(orc):
    cfg = wh_cfg()
    s = set_state(orc, cfg, [(0, 0, 1), (3, 3, None)], [(5, 5, False), (0, 0, True), (1, 5, False)])
    step(orc, cfg, s, [1, 0])                     # north into the wall: stays, no collision
    assert (s.agent_row[0, 0], s.agent_col[0, 0]) == (0, 0)
    step(orc, cfg, s, [2, 0])
    assert (s.agent_row[0, 0], s.agent_col[0, 0]) == (1, 0) and (s.food_row[1, 0], s.food_col[1, 0]) == (1, 0)
    assert s.agent_lvl[0, 0] == 2 and s.food_lvl[1, 0] == 2


@pytest.mark.parametrize("kind", [1, 2])
def test_contested_and_occupied_cells_are_collisions(orc, kind):
    cfg = wh_cfg(kind)
    # two robots into the same empty cell: both stay; kind 2 ends the episode
    s = set_state(orc, cfg, [(2, 1, None), (2, 3, None)], [(0, 0, False), (0, 1, True), (0, 2, True)])
    s.episode_id[0] = 7
    _, rew, done = step(orc, cfg, s, [4, 3])
    assert done == (1 if kind == 2 else 0)
    if kind == 1:
        assert (s.agent_col[0, 0], s.agent_col[1, 0]) == (1, 3)
    else:
        assert s.episode_id[0] == 8 and s.t_in_ep[0] == 0
    # into an occupied cell (the occupant stays put): refused, a collision
    s = set_state(orc, cfg, [(2, 1, None), (2, 2, None)], [(0, 0, False), (0, 1, True), (0, 2, True)])
    _, rew, done = step(orc, cfg, s, [4, 0])
    assert done == (1 if kind == 2 else 0)
    # the occupant moves away in the same step: still refused (start-of-step occupancy)
    s = set_state(orc, cfg, [(2, 1, None), (2, 2, None)], [(0, 0, False), (0, 1, True), (0, 2, True)])
    step(orc, wh_cfg(1), s, [4, 4])
    assert (s.agent_col[0, 0], s.agent_col[1, 0]) == (1, 3)
    # walls and shelves are not collisions
    s = set_state(orc, cfg, [(0, 0, 0), (5, 5, None)], [(0, 0, False), (0, 1, True), (3, 3, True)])
    _, _, done = step(orc, cfg, s, [4, 2])        # loaded robot into a shelf, other robot into the wall
    assert done == 0


def test_toggle_picks_up_and_puts_down(orc):
    cfg = wh_cfg()
    s = set_state(orc, cfg, [(2, 2, None), (3, 3, 1)], [(2, 2, True), (3, 3, False), (0, 0, True)])
    step(orc, cfg, s, [5, 5])
    assert s.agent_lvl[0, 0] == 1 and s.agent_lvl[1, 0] == 0          # robot 0 now carries shelf 0, robot 1 nothing
    assert (s.food_row[1, 0], s.food_col[1, 0]) == (3, 3)
    step(orc, cfg, s, [0, 5])                                          # robot 1 picks its shelf up again
    assert s.agent_lvl[1, 0] == 2
    s = set_state(orc, cfg, [(1, 1, None), (3, 3, None)], [(2, 2, True), (4, 4, False), (0, 0, True)])
    step(orc, cfg, s, [5, 0])                                          # nothing to pick up
    assert s.agent_lvl[0, 0] == 0


def test_delivery_pays_one_and_moves_the_request(orc):
    cfg = wh_cfg(grid=6)                                               # goals (5, 2) and (5, 3)
    s = set_state(orc, cfg, [(4, 2, 0), (0, 0, None)], [(4, 2, True), (1, 1, True), (2, 4, False)])
    _, rew, done = step(orc, cfg, s, [2, 0])
    assert rew[0] == 1.0 and rew[1] == 0.0 and done == 0
    assert s.food_lvl[0, 0] == 1 and s.food_lvl[2, 0] == 2 and s.food_lvl[1, 0] == 2   # the only other idle shelf
    assert s.agent_lvl[0, 0] == 1                                      # still carried
    # an idle shelf on a goal earns nothing
    _, rew, _ = step(orc, cfg, s, [0, 0])
    assert np.all(rew == 0)
    # no other idle shelf: the delivered one is requested again
    cfg1 = wh_cfg(n_food=2, max_level=2)
    s = set_state(orc, cfg1, [(4, 3, 1), (0, 0, None)], [(1, 1, True), (4, 3, True)])
    _, rew, _ = step(orc, cfg1, s, [2, 0])
    assert rew[0] == 1.0 and s.food_lvl[1, 0] == 2 and s.food_lvl[0, 0] == 2
    # the choice among several idle shelves is the keyed Philox draw
    cfg2 = wh_cfg(n_food=6, max_level=1, grid=8)                       # goals (7, 3) and (7, 4)
    picks = []
    for ep in range(40):
        s = set_state(orc, cfg2, [(6, 4, 2), (0, 0, None)],
                      [(1, 1, False), (1, 3, False), (6, 4, True), (2, 2, False), (3, 5, False), (4, 1, False)])
        s.episode_id[0], s.t_in_ep[0] = ep, 3
        step(orc, cfg2, s, [2, 0])
        new = [f for f in range(6) if s.food_lvl[f, 0] == 2]
        assert len(new) == 1 and new[0] != 2
        word = orc.philox4x32_10([0, ep, 3 * 2, 3], [cfg2["seed"] & 0xffffffff, cfg2["seed"] >> 32])[0]
        cands = [0, 1, 3, 4, 5]
        assert new[0] == cands[orc.rand_below(word, 5)]
        picks.append(new[0])
    assert len(set(picks)) >= 4


def test_cap_ends_the_episode_and_reset_is_keyed(orc):
    cfg = wh_cfg(episode_cap=3, n_envs=5)
    s = orc.EnvState(cfg)
    orc.env_reset(cfg, s)
    first = s.copy()
    dones = []
    for t in range(7):
        _, _, d = orc.env_step(cfg, s, np.zeros((5, 2), np.int32))
        dones.append(d.copy())
    assert [int(d[0]) for d in dones] == [0, 0, 1, 0, 0, 1, 0]
    assert np.all(s.episode_id == 2)
    s2 = orc.EnvState(wh_cfg(episode_cap=3, n_envs=2))
    orc.env_reset(wh_cfg(episode_cap=3, n_envs=2), s2)                 # a layout depends on (seed, env, episode) only
    for f in ("agent_row", "agent_col", "food_row", "food_col", "food_lvl"):
        assert np.array_equal(getattr(first, f)[:, :2], getattr(s2, f))


def test_reset_layouts(orc):
    cfg = wh_cfg(n_envs=4000, n_food=5, max_level=2, n_agents=3)
    s = orc.EnvState(cfg)
    orc.env_reset(cfg, s)
    G = cfg["grid"]
    cells = np.concatenate([s.agent_row.astype(int) * G + s.agent_col, s.food_row.astype(int) * G + s.food_col])
    srt = np.sort(cells, axis=0)
    assert np.all(srt[1:] != srt[:-1]) and cells.max() < G * G
    assert np.all(s.agent_lvl == 0) and np.all((s.food_lvl == 1) | (s.food_lvl == 2))
    assert np.all((s.food_lvl == 2).sum(axis=0) == 2)
    freq = (s.food_lvl == 2).mean(axis=1)                               # every shelf requested 2/5 of the time
    assert np.all(np.abs(freq - 0.4) < 4 * np.sqrt(0.4 * 0.6 / 4000))
    occ = np.bincount(cells.reshape(-1), minlength=G * G) / (8 * 4000)  # cells uniform
    assert np.all(np.abs(occ - 1 / 36) < 5 * np.sqrt((1 / 36) / (8 * 4000)))


def test_observation_channels(orc):
    cfg = wh_cfg(view=5, grid=6)
    s = set_state(orc, cfg, [(4, 2, 0), (4, 3, None)], [(4, 2, True), (3, 2, False), (5, 5, True)])
    obs = orc.observe(cfg, s)[0]
    o = obs[0].reshape(5, 5, 3)                                        # robot 0 at (4, 2): window rows 2..6, cols 0..4
    assert o[2, 2, 0] == 2.0 and o[2, 3, 0] == 1.0                     # itself loaded, its neighbour unloaded
    assert o[2, 2, 1] == 2.0 and o[1, 2, 1] == 1.0                     # its requested shelf, the idle one north of it
    assert np.all(o[4, :, 2] == 1.0) and np.all(o[:4, :, 2] != 1.0)    # row 6 is outside
    assert o[3, 2, 2] == 0.5 and o[3, 3, 2] == 0.5 and o[3, 1, 2] == 0.0   # goals (5, 2), (5, 3)
    assert o.sum() == 2 + 1 + 2 + 1 + 5 + 1.0


def python_step(cfg, st, actions, philox, rand_below):
    """Independent re-statement with sets and dicts; st = dict of python lists for one environment."""
    G, A, F = cfg["grid"], cfg["n_agents"], cfg["n_food"]
    pos = [tuple(p) for p in st["robots"]]
    carry = list(st["carry"])                                          # shelf index or None
    shelf = [tuple(p) for p in st["shelves"]]
    req = list(st["requested"])
    delta = {1: (-1, 0), 2: (1, 0), 3: (0, -1), 4: (0, 1)}
    want = {}
    hit_robot = set()
    for a in range(A):
        if actions[a] in delta:
            t = (pos[a][0] + delta[actions[a]][0], pos[a][1] + delta[actions[a]][1])
            if not (0 <= t[0] < G and 0 <= t[1] < G):
                continue
            if t in pos:
                hit_robot.add(a)
                continue
            if carry[a] is not None and t in shelf:
                continue
            want[a] = t
    targets = list(want.values())
    contested = {a for a, t in want.items() if targets.count(t) > 1}
    collided = bool(hit_robot or contested)
    new_pos = list(pos)
    for a, t in want.items():
        if a not in contested:
            new_pos[a] = t
            if carry[a] is not None:
                shelf[carry[a]] = t
    new_carry = list(carry)
    for a in range(A):
        if actions[a] == 5:
            if carry[a] is not None:
                new_carry[a] = None
            else:
                for f in range(F):
                    if shelf[f] == pos[a] and f not in carry:
                        new_carry[a] = f
    reward = [0.0] * A
    goals = {(G - 1, G // 2 - 1), (G - 1, G // 2)}
    ordinal = 0
    for a in range(A):
        f = new_carry[a]
        if f is None or not req[f] or new_pos[a] not in goals:
            continue
        reward[a] = 1.0
        req[f] = False
        cands = [g for g in range(F) if g != f and not req[g]]
        if not cands:
            req[f] = True
        else:
            words = philox([st["env"], st["episode"], st["t"] * 2 + ordinal // 4, 3],
                           [cfg["seed"] & 0xffffffff, cfg["seed"] >> 32])
            req[cands[rand_below(words[ordinal % 4], len(cands))]] = True
        ordinal += 1
    t = st["t"] + 1
    done = t == cfg["episode_cap"] or (cfg["env_kind"] == 2 and collided)
    return dict(robots=new_pos, carry=new_carry, shelves=shelf, requested=req, t=t), reward, done


@pytest.mark.parametrize("kind,A,F,R,G", [(1, 2, 3, 2, 4), (2, 3, 4, 1, 5), (1, 4, 6, 3, 5), (1, 8, 8, 8, 6)])
def test_step_matches_the_set_based_restatement(orc, kind, A, F, R, G):
    cfg = wh_cfg(kind, n_agents=A, n_food=F, max_level=R, grid=G, n_envs=24, episode_cap=9)
    N = cfg["n_envs"]
    s = orc.EnvState(cfg)
    orc.env_reset(cfg, s)
    rng = np.random.default_rng(kind * 10 + A)
    n_deliveries = n_done = n_carry = 0
    for it in range(220):
        before = s.copy()
        actions = rng.integers(0, 6, size=(N, A)).astype(np.int32)
        actions = np.where(rng.random((N, A)) < 0.25, 2, actions).astype(np.int32)   # drift south, towards the goals
        _, rew, done = orc.env_step(cfg, s, actions)
        for n in range(N):
            st = dict(robots=[(int(before.agent_row[a, n]), int(before.agent_col[a, n])) for a in range(A)],
                      carry=[None if before.agent_lvl[a, n] == 0 else int(before.agent_lvl[a, n]) - 1 for a in range(A)],
                      shelves=[(int(before.food_row[f, n]), int(before.food_col[f, n])) for f in range(F)],
                      requested=[before.food_lvl[f, n] == 2 for f in range(F)],
                      t=int(before.t_in_ep[n]), env=n, episode=int(before.episode_id[n]))
            nxt, r, d = python_step(cfg, st, [int(x) for x in actions[n]], orc.philox4x32_10, orc.rand_below)
            assert list(rew[n]) == r and int(done[n]) == int(d), (it, n)
            n_deliveries += int(sum(r))
            n_done += int(d)
            if d:
                assert s.episode_id[n] == before.episode_id[n] + 1 and s.t_in_ep[n] == 0
                continue
            assert [(int(s.agent_row[a, n]), int(s.agent_col[a, n])) for a in range(A)] == nxt["robots"]
            assert [None if s.agent_lvl[a, n] == 0 else int(s.agent_lvl[a, n]) - 1 for a in range(A)] == nxt["carry"]
            assert [(int(s.food_row[f, n]), int(s.food_col[f, n])) for f in range(F)] == nxt["shelves"]
            assert [s.food_lvl[f, n] == 2 for f in range(F)] == nxt["requested"]
        # invariants of the rules
        cells = s.agent_row.astype(int) * G + s.agent_col
        srt = np.sort(cells, axis=0)
        assert np.all(srt[1:] != srt[:-1])                               # robots never share a cell
        assert np.all((s.food_lvl == 2).sum(axis=0) == R)                # always R requests
        for a in range(A):
            cy = s.agent_lvl[a]
            on = cy > 0
            n_carry += int(on.sum())
            f = cy[on].astype(int) - 1
            cols = np.nonzero(on)[0]
            assert np.array_equal(s.food_row[f, cols], s.agent_row[a, cols]) and np.array_equal(s.food_col[f, cols], s.agent_col[a, cols])
        carried = np.zeros((F, N), bool)
        for a in range(A):
            on = s.agent_lvl[a] > 0
            idx = s.agent_lvl[a][on].astype(int) - 1
            assert not carried[idx, np.nonzero(on)[0]].any()             # a shelf has one carrier at most
            carried[idx, np.nonzero(on)[0]] = True
        scell = np.where(carried, -1 - np.arange(F)[:, None], s.food_row.astype(int) * G + s.food_col)
        ss = np.sort(scell, axis=0)
        assert np.all(ss[1:] != ss[:-1])                                 # shelves on the floor never share a cell
    assert n_done > 0 and n_carry > 0
    if (kind, A) != (2, 3):
        assert n_deliveries > 0
