"""The C-ABI library loads without a GPU, exports every symbol the header declares, and rejects bad
arguments on the host before anything is launched."""
import ctypes as C
import os
import re

import pytest

import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def M():
    import paper_2107_01460_amd as m
    if not os.path.exists(m.binding._LIB_PATH):
        from paper_2107_01460_amd import build
        build.build(verbose=False)
    m.lib()
    return m


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "marl.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(marl_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(M):
    names = declared_symbols()
    assert len(names) >= 12
    for n in names:
        assert hasattr(M.lib(), n), n
    assert set(M.binding.EXPORTS) == set(names)


def test_query_sizes_and_parameter_counts(M):
    for cfg in W.CONFIGS:
        s = M.query_sizes(cfg)
        assert s.n_params == W.param_count(cfg)
        assert s.obs_dim == W.obs_dim(cfg) and s.critic_in_dim == W.critic_in_dim(cfg)
        T, N, A = cfg["rollout_len"], cfg["n_envs"], cfg["n_agents"]
        assert s.obs_bytes == 4 * (T + 1) * N * A * s.obs_dim
        assert s.step_scalar_bytes == 4 * T * N * A and s.done_bytes == T * N
        assert s.rollout_workspace_bytes > 0 and s.update_workspace_bytes > s.n_params * 8


@pytest.mark.parametrize("field,value", [
    ("grid", 1), ("grid", 65), ("n_agents", 9), ("n_food", 0), ("view", 4), ("actor_hidden", 100),
    ("critic_hidden", 1024), ("n_minibatches", 7), ("precision", 2), ("clip_eps", 0.0), ("gamma", 1.5),
    ("max_level", 0), ("max_level", 16), ("central_critic", 2), ("lr", 0.0), ("n_minibatches", 0), ("n_epochs", 0)])
def test_bad_config_rejected(M, field, value):
    cfg = W.scaled(W.CONFIGS[1], **{field: value})
    s = M.binding.Sizes()
    rc = M.lib().marl_query_sizes(C.byref(M.make_config(cfg)), C.byref(s))
    assert rc == -3, (field, rc)
    st = M.binding.EnvStateC(*([0x1000] * 8))
    assert M.lib().marl_env_reset(C.byref(M.make_config(cfg)), st, None) == -3


def test_zero_minibatches_rejected_for_recurrent_networks(M):
    """n_minibatches is a divisor in the checks of the recurrent configuration: zero must be an error, not a trap."""
    s = M.binding.Sizes()
    for nm in (0, -1):
        cfg = W.scaled(W.CONFIGS[0], recurrent=1, n_minibatches=nm)
        assert M.lib().marl_query_sizes(C.byref(M.make_config(cfg)), C.byref(s)) == -3


def test_recurrent_sizes(M):
    cfg = W.scaled(W.CONFIGS[2], recurrent=1)
    sz = M.query_sizes(cfg)
    assert sz.n_params == W.param_count(cfg)
    assert sz.hidden_actor_bytes == 4 * cfg["n_envs"] * cfg["n_agents"] * cfg["actor_hidden"]
    assert sz.hidden_critic_bytes == 4 * cfg["n_envs"] * cfg["critic_hidden"]
    assert sz.rollout_workspace_bytes > 0 and sz.update_workspace_bytes > 0
    assert M.query_sizes(W.CONFIGS[2]).hidden_actor_bytes == 0


def test_warehouse_config_checks(M):
    L = M.lib()
    sz = M.binding.Sizes()
    ok = M.make_config(W.scaled(W.CONFIGS[1], env_kind=2, max_level=3))
    assert L.marl_query_sizes(C.byref(ok), C.byref(sz)) == 0
    assert L.marl_query_sizes(C.byref(M.make_config(W.scaled(W.CONFIGS[1], env_kind=3))), C.byref(sz)) == -3
    # more requested shelves than shelves
    assert L.marl_query_sizes(C.byref(M.make_config(W.scaled(W.CONFIGS[0], env_kind=1, max_level=2))), C.byref(sz)) == -3


def test_too_many_entities_rejected(M):
    cfg = W.scaled(W.CONFIGS[0], grid=2, n_agents=3, n_food=2)
    s = M.binding.Sizes()
    assert M.lib().marl_query_sizes(C.byref(M.make_config(cfg)), C.byref(s)) == -3


def test_null_and_misaligned_pointers_rejected_before_launch(M):
    cfg = M.make_config(W.CONFIGS[0])
    L = M.lib()
    good = 0x10000
    null_state = M.binding.EnvStateC(*([good] * 7 + [None]))
    assert L.marl_env_reset(C.byref(cfg), null_state, None) == -1
    odd_state = M.binding.EnvStateC(*([good] * 7 + [good + 4]))
    assert L.marl_env_reset(C.byref(cfg), odd_state, None) == -2
    ok_state = M.binding.EnvStateC(*([good] * 8))
    assert L.marl_observe(C.byref(cfg), ok_state, None, None) == -1
    assert L.marl_env_step(C.byref(cfg), ok_state, good, good + 8, good, good, None) == -2
    traj = M.binding.TrajC(*([good] * 9 + [None, None]))
    assert L.marl_rollout(C.byref(cfg), ok_state, None, traj, 0, None, None, good, None) == -1
    assert L.marl_compute_gae(C.byref(cfg), M.binding.TrajC(*([good] * 7 + [None, good, None, None])), None) == -1
    assert L.marl_ppo_update(C.byref(cfg), traj, good, good, good, -1, None, good, None, good, None) == -5
    assert L.marl_ppo_update(C.byref(cfg), traj, good, good, good, 0, good + 2, good, None, good, None) == -2
    assert L.marl_policy_forward(C.byref(cfg), good, good, -1, good, good, good, None) == -5
    assert L.marl_sample_actions(C.byref(cfg), good, None, None, 1 << 31, 0, good, None, good, None) == -5
    ev = M.binding.EvalStatsC(good, good, good)
    assert L.marl_evaluate(C.byref(cfg), ok_state, good, 0, ev, good, None) == -5
    assert L.marl_evaluate(C.byref(cfg), ok_state, good, 1 << 20, ev, good, None) == -5
    assert L.marl_evaluate(C.byref(cfg), ok_state, None, 1, ev, good, None) == -1
    assert L.marl_evaluate(C.byref(cfg), ok_state, good, 1, M.binding.EvalStatsC(good, None, good), good, None) == -1
    rs = M.binding.RecStateC(good, good, good, good)
    # the recurrent entry points take recurrent configurations only, and the feed-forward ones refuse them
    assert L.marl_rollout_recurrent(C.byref(cfg), ok_state, good, traj, rs, 0, None, None, good, None) == -3
    rcfg = M.make_config(W.scaled(W.CONFIGS[0], recurrent=1))
    assert L.marl_rollout(C.byref(rcfg), ok_state, good, traj, 0, None, None, good, None) == -3
    assert L.marl_ppo_update(C.byref(rcfg), traj, good, good, good, 0, None, good, None, good, None) == -3
    assert L.marl_rollout_recurrent(C.byref(rcfg), ok_state, good, traj, M.binding.RecStateC(good, None, good, good), 0,
                                    None, None, good, None) == -1
    assert L.marl_ppo_update_recurrent(C.byref(rcfg), traj, rs, good, good, good, -1, None, good, None, good, None) == -5
    assert L.marl_ppo_update_recurrent(C.byref(rcfg), traj, rs, good, good + 4, good, 0, None, good, None, good, None) == -2
    bad = M.make_config(W.scaled(W.CONFIGS[0], recurrent=1, n_minibatches=3))     # 64 environments do not split in 3
    assert L.marl_ppo_update_recurrent(C.byref(bad), traj, rs, good, good, good, 0, None, good, None, good, None) == -3
    # the single-call training step: counters and both workspaces are required, feed-forward networks only
    assert L.marl_train_step(C.byref(cfg), ok_state, good, traj, good, good, None, None, good, good, good, None) == -1
    assert L.marl_train_step(C.byref(cfg), ok_state, good, traj, good, good, good, None, good, good, None, None) == -1
    assert L.marl_train_step(C.byref(cfg), ok_state, good, traj, good, good, good + 8, None, good, good, good, None) == -2
    assert L.marl_train_step(C.byref(rcfg), ok_state, good, traj, good, good, good, None, good, good, good, None) == -3
    assert L.marl_query_sizes(None, None) == -1
    assert M.status_string(0) == "ok" and "null" in M.status_string(-1)
    d, n, w = C.c_double(), C.c_int64(), C.c_double()
    assert L.marl_timing_read(99, C.byref(d), C.byref(n), C.byref(w)) == -5
    assert L.marl_timing_read(0, None, None, None) == -1


def test_missing_library_fails_loudly(M, monkeypatch):
    monkeypatch.setattr(M.binding, "_lib", None)
    monkeypatch.setattr(M.binding, "_LIB_PATH", "/nonexistent/libmarl_gfx950.so")
    with pytest.raises(M.MarlError):
        M.binding.lib()
