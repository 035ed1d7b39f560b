"""ctypes front end of the CPU oracle (test infrastructure only).

Only tests, the smoke check and the benchmark's cpu_baseline leg import this package.  It
imports nothing from the product package and the product package imports nothing from here.

All arrays are numpy, host memory.  The oracle's own C structs are declared here; they are
filled from a plain ``dict`` configuration.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "marl_oracle.cpp")
_LIB = os.path.join(_HERE, "libmarl_oracle.so")

N_ACTIONS = 6


def build(force=False):
    """Compile the oracle with g++ -O2 (no fast-math, no OpenMP)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["g++", "-O2", "-std=c++17", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", _LIB, _SRC]
        )
    return _LIB


class Config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "grid", "n_agents", "n_food", "max_level", "episode_cap", "view", "n_envs", "rollout_len",
        "actor_hidden", "critic_hidden", "central_critic", "precision",
        "n_epochs", "n_minibatches", "normalize_adv", "clip_value")] + [(n, C.c_float) for n in (
        "gamma", "lambda_", "clip_eps", "ent_coef", "vf_coef", "max_grad_norm",
        "lr", "beta1", "beta2", "adam_eps")] + [("seed", C.c_uint64), ("recurrent", C.c_int32),
                                                   ("env_kind", C.c_int32)]


_U8P = C.POINTER(C.c_uint8)
_I32P = C.POINTER(C.c_int32)
_U32P = C.POINTER(C.c_uint32)
_F32P = C.POINTER(C.c_float)
_F64P = C.POINTER(C.c_double)


class EnvStateC(C.Structure):
    _fields_ = [("agent_row", _U8P), ("agent_col", _U8P), ("agent_lvl", _U8P),
                ("food_row", _U8P), ("food_col", _U8P), ("food_lvl", _U8P),
                ("t_in_ep", _I32P), ("episode_id", _U32P)]


class RecStateC(C.Structure):
    _fields_ = [("ha0", _F32P), ("hc0", _F32P), ("ha1", _F32P), ("hc1", _F32P)]


class TrajC(C.Structure):
    _fields_ = [("obs", _F32P), ("action", _I32P), ("logp", _F32P), ("value", _F32P),
                ("reward", _F32P), ("done", _U8P), ("last_value", _F32P), ("adv", _F32P),
                ("ret", _F32P), ("logits", _F32P), ("sampled", _I32P), ("gap", _F32P)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_rand_unit.restype = C.c_float
        _lib.orc_round_bf16.restype = C.c_float
        _lib.orc_rand_below.restype = C.c_uint32
        _lib.orc_round_bf16.argtypes = [C.c_float]
        _lib.orc_rand_unit.argtypes = [C.c_uint32]
        _lib.orc_rand_below.argtypes = [C.c_uint32, C.c_uint32]
        _lib.orc_param_count.restype = C.c_int32
        _lib.orc_actor_param_count.restype = C.c_int32
        _lib.orc_env_reset.argtypes = [C.POINTER(Config), EnvStateC]
        _lib.orc_observe.argtypes = [C.POINTER(Config), EnvStateC, _F32P]
        _lib.orc_env_step.argtypes = [C.POINTER(Config), EnvStateC, _I32P, _F32P, _F32P, _U8P]
        _lib.orc_policy_forward.argtypes = [C.POINTER(Config), _F32P, _F32P, C.c_int64, _F32P, _F32P]
        _lib.orc_sample.argtypes = [_F32P, _F32P, _I32P, C.c_int64, _I32P, _I32P, _F32P, _F32P]
        _lib.orc_sample_uniforms.argtypes = [C.POINTER(Config), C.c_uint64, C.c_int32, C.c_int32, _F32P]
        _lib.orc_rollout.argtypes = [C.POINTER(Config), EnvStateC, _F32P, TrajC, C.c_uint64, _I32P, _F32P]
        _lib.orc_compute_gae.argtypes = [C.POINTER(Config), TrajC]
        _lib.orc_rec_policy_step.argtypes = [C.POINTER(Config), _F32P, _F32P, _F32P, _F32P, C.c_int64, _F32P, _F32P,
                                             _F32P, _F32P]
        _lib.orc_rec_rollout.argtypes = [C.POINTER(Config), EnvStateC, _F32P, TrajC, RecStateC, C.c_uint64, _I32P,
                                         _F32P]
        _lib.orc_rec_minibatch_loss_grad_f64.argtypes = [C.POINTER(Config), TrajC, RecStateC, _F64P, _I32P, C.c_int32,
                                                         _F64P, _F64P]
        _lib.orc_rec_ppo_update.argtypes = [C.POINTER(Config), TrajC, RecStateC, _F32P, _F32P, _F32P, C.c_int64, _I32P,
                                            _F32P, _F32P]
        _lib.orc_evaluate.argtypes = [C.POINTER(Config), EnvStateC, _F32P, C.c_int32, _F32P, _I32P, _I32P, _F32P]
        _lib.orc_minibatch_loss_grad_f64.argtypes = [C.POINTER(Config), TrajC, _F64P, _I32P, C.c_int32,
                                                     _F64P, _F64P]
        _lib.orc_adam_step.argtypes = [C.POINTER(Config), _F32P, _F32P, _F32P, _F64P, C.c_int64, C.c_int64]
        _lib.orc_ppo_update.argtypes = [C.POINTER(Config), TrajC, _F32P, _F32P, _F32P, C.c_int64, _I32P,
                                        _F32P, _F32P]
    return _lib


def make_config(cfg: dict) -> Config:
    c = Config()
    for name, _ in Config._fields_:
        key = "lambda" if name == "lambda_" else name
        setattr(c, name, cfg.get(key, 0) if name in ("recurrent", "env_kind") else cfg[key])
    return c


def _p(arr, ty):
    if arr is None:
        return None
    assert arr.flags["C_CONTIGUOUS"]
    return arr.ctypes.data_as(ty)


_PTR_OF = {np.dtype(np.uint8): _U8P, np.dtype(np.int32): _I32P, np.dtype(np.uint32): _U32P,
           np.dtype(np.float32): _F32P, np.dtype(np.float64): _F64P}


def _ap(arr):
    return None if arr is None else _p(arr, _PTR_OF[arr.dtype])


def obs_dim(cfg):
    return 3 * cfg["view"] * cfg["view"]


def param_count(cfg):
    return lib().orc_param_count(C.byref(make_config(cfg)))


def actor_param_count(cfg):
    return lib().orc_actor_param_count(C.byref(make_config(cfg)))


class EnvState:
    """Host copy of the vectorised environment state (entity-major structure of arrays)."""
    FIELDS = ("agent_row", "agent_col", "agent_lvl", "food_row", "food_col", "food_lvl", "t_in_ep",
              "episode_id")

    def __init__(self, cfg):
        N, A, F = cfg["n_envs"], cfg["n_agents"], cfg["n_food"]
        self.agent_row = np.zeros((A, N), np.uint8)
        self.agent_col = np.zeros((A, N), np.uint8)
        self.agent_lvl = np.zeros((A, N), np.uint8)
        self.food_row = np.zeros((F, N), np.uint8)
        self.food_col = np.zeros((F, N), np.uint8)
        self.food_lvl = np.zeros((F, N), np.uint8)
        self.t_in_ep = np.zeros((N,), np.int32)
        self.episode_id = np.zeros((N,), np.uint32)

    def c(self):
        return EnvStateC(*[_ap(getattr(self, f)) for f in self.FIELDS])

    def copy(self):
        o = object.__new__(EnvState)
        for f in self.FIELDS:
            setattr(o, f, getattr(self, f).copy())
        return o


class Traj:
    FIELDS = ("obs", "action", "logp", "value", "reward", "done", "last_value", "adv", "ret", "logits",
              "sampled", "gap")

    def __init__(self, cfg):
        N, A, T, D = cfg["n_envs"], cfg["n_agents"], cfg["rollout_len"], obs_dim(cfg)
        self.obs = np.zeros((T + 1, N, A, D), np.float32)
        self.action = np.zeros((T, N, A), np.int32)
        self.logp = np.zeros((T, N, A), np.float32)
        self.value = np.zeros((T, N, A), np.float32)
        self.reward = np.zeros((T, N, A), np.float32)
        self.done = np.zeros((T, N), np.uint8)
        self.last_value = np.zeros((N, A), np.float32)
        self.adv = np.zeros((T, N, A), np.float32)
        self.ret = np.zeros((T, N, A), np.float32)
        self.logits = np.zeros((T, N, A, N_ACTIONS), np.float32)
        self.sampled = np.zeros((T, N, A), np.int32)
        self.gap = np.zeros((T, N, A), np.float32)

    def c(self):
        return TrajC(*[_ap(getattr(self, f)) for f in self.FIELDS])


def philox4x32_10(ctr, key):
    ctr = np.asarray(ctr, np.uint32)
    key = np.asarray(key, np.uint32)
    out = np.zeros(4, np.uint32)
    lib().orc_philox4x32_10(_ap(ctr), _ap(key), _ap(out))
    return out


def rand_below(x, n):
    return lib().orc_rand_below(int(x), int(n))


def rand_unit(x):
    return lib().orc_rand_unit(int(x))


def round_bf16(x):
    return lib().orc_round_bf16(float(x))


def env_reset(cfg, state):
    lib().orc_env_reset(C.byref(make_config(cfg)), state.c())


def observe(cfg, state):
    N, A = cfg["n_envs"], cfg["n_agents"]
    obs = np.zeros((N, A, obs_dim(cfg)), np.float32)
    lib().orc_observe(C.byref(make_config(cfg)), state.c(), _ap(obs))
    return obs


def env_step(cfg, state, actions, want_obs=True):
    N, A = cfg["n_envs"], cfg["n_agents"]
    actions = np.ascontiguousarray(actions, np.int32).reshape(N, A)
    obs = np.zeros((N, A, obs_dim(cfg)), np.float32) if want_obs else None
    reward = np.zeros((N, A), np.float32)
    done = np.zeros((N,), np.uint8)
    lib().orc_env_step(C.byref(make_config(cfg)), state.c(), _ap(actions), _ap(obs), _ap(reward), _ap(done))
    return obs, reward, done


def policy_forward(cfg, params, obs_rows):
    """obs_rows [rows][A][D] -> logits [rows][A][6], value [rows][A]."""
    A = cfg["n_agents"]
    obs_rows = np.ascontiguousarray(obs_rows, np.float32)
    rows = obs_rows.size // (A * obs_dim(cfg))
    logits = np.zeros((rows, A, N_ACTIONS), np.float32)
    value = np.zeros((rows, A), np.float32)
    params = np.ascontiguousarray(params, np.float32)
    lib().orc_policy_forward(C.byref(make_config(cfg)), _ap(params), _ap(obs_rows), rows, _ap(logits), _ap(value))
    return logits, value


def sample(logits, uniforms, forced=None):
    logits = np.ascontiguousarray(logits, np.float32).reshape(-1, N_ACTIONS)
    uniforms = np.ascontiguousarray(uniforms, np.float32).reshape(-1, N_ACTIONS)
    n = logits.shape[0]
    action = np.zeros(n, np.int32)
    sampled = np.zeros(n, np.int32)
    logp = np.zeros(n, np.float32)
    gap = np.zeros(n, np.float32)
    f = None if forced is None else np.ascontiguousarray(forced, np.int32).reshape(-1)
    lib().orc_sample(_ap(logits), _ap(uniforms), _ap(f), n, _ap(action), _ap(sampled), _ap(logp), _ap(gap))
    return action, sampled, logp, gap


def sample_uniforms(cfg, step, env, agent):
    u = np.zeros(N_ACTIONS, np.float32)
    lib().orc_sample_uniforms(C.byref(make_config(cfg)), int(step), int(env), int(agent), _ap(u))
    return u


def rollout(cfg, state, params, traj, step_offset=0, forced_actions=None, forced_uniforms=None):
    params = np.ascontiguousarray(params, np.float32)
    fa = None if forced_actions is None else np.ascontiguousarray(forced_actions, np.int32)
    fu = None if forced_uniforms is None else np.ascontiguousarray(forced_uniforms, np.float32)
    lib().orc_rollout(C.byref(make_config(cfg)), state.c(), _ap(params), traj.c(), int(step_offset), _ap(fa), _ap(fu))


def evaluate(cfg, state, params, n_episodes):
    """Greedy evaluation block: (ret_sum [N] f32, len_sum [N] i32, episodes [N] i32, min_gap [N] f32)."""
    N = cfg["n_envs"]
    ret_sum, min_gap = np.zeros(N, np.float32), np.zeros(N, np.float32)
    len_sum, episodes = np.zeros(N, np.int32), np.zeros(N, np.int32)
    params = np.ascontiguousarray(params, np.float32)
    lib().orc_evaluate(C.byref(make_config(cfg)), state.c(), _ap(params), int(n_episodes), _ap(ret_sum), _ap(len_sum),
                       _ap(episodes), _ap(min_gap))
    return ret_sum, len_sum, episodes, min_gap


def compute_gae(cfg, traj):
    lib().orc_compute_gae(C.byref(make_config(cfg)), traj.c())


def minibatch_loss_grad(cfg, traj, params_f64, rows, want_grad=True):
    params_f64 = np.ascontiguousarray(params_f64, np.float64)
    rows = np.ascontiguousarray(rows, np.int32)
    stats = np.zeros(6, np.float64)
    grad = np.zeros(params_f64.size, np.float64) if want_grad else None
    lib().orc_minibatch_loss_grad_f64(C.byref(make_config(cfg)), traj.c(), _ap(params_f64), _ap(rows), rows.size,
                                      _ap(stats), _ap(grad))
    return stats, grad


def adam_step(cfg, params, m, v, grad_f64, k):
    grad_f64 = np.ascontiguousarray(grad_f64, np.float64)
    lib().orc_adam_step(C.byref(make_config(cfg)), _ap(params), _ap(m), _ap(v), _ap(grad_f64), int(k), params.size)


def ppo_update(cfg, traj, params, adam_m, adam_v, adam_step0=0, perm=None):
    """In-place on params / adam_m / adam_v (fp32 numpy).  Returns (stats [E*M][8], grad of last minibatch)."""
    E, M = cfg["n_epochs"], cfg["n_minibatches"]
    stats = np.zeros((E * M, 8), np.float32)
    grad = np.zeros(params.size, np.float32)
    pm = None if perm is None else np.ascontiguousarray(perm, np.int32)
    lib().orc_ppo_update(C.byref(make_config(cfg)), traj.c(), _ap(params), _ap(adam_m), _ap(adam_v), int(adam_step0),
                         _ap(pm), _ap(stats), _ap(grad))
    return stats, grad


# ---- recurrent networks ----------------------------------------------------------------------------------

class RecState:
    """Hidden states around one rollout: h*0 = state the rollout starts from, h*1 = state it leaves."""

    def __init__(self, cfg):
        N, A, Ha, Hc = cfg["n_envs"], cfg["n_agents"], cfg["actor_hidden"], cfg["critic_hidden"]
        cshape = (N, Hc) if cfg["central_critic"] else (N, A, Hc)
        self.ha0, self.ha1 = np.zeros((N, A, Ha), np.float32), np.zeros((N, A, Ha), np.float32)
        self.hc0, self.hc1 = np.zeros(cshape, np.float32), np.zeros(cshape, np.float32)

    def c(self):
        return RecStateC(_ap(self.ha0), _ap(self.hc0), _ap(self.ha1), _ap(self.hc1))


def rec_policy_step(cfg, params, obs_rows, ha_in, hc_in):
    """(logits, value, ha_out, hc_out) of one step of both recurrent networks."""
    obs_rows = np.ascontiguousarray(obs_rows, np.float32)
    n = obs_rows.shape[0]
    A = cfg["n_agents"]
    ha_in, hc_in = np.ascontiguousarray(ha_in, np.float32), np.ascontiguousarray(hc_in, np.float32)
    logits, value = np.zeros((n, A, N_ACTIONS), np.float32), np.zeros((n, A), np.float32)
    ha_out, hc_out = np.zeros_like(ha_in), np.zeros_like(hc_in)
    params = np.ascontiguousarray(params, np.float32)
    lib().orc_rec_policy_step(C.byref(make_config(cfg)), _ap(params), _ap(obs_rows), _ap(ha_in), _ap(hc_in), n,
                              _ap(logits), _ap(value), _ap(ha_out), _ap(hc_out))
    return logits, value, ha_out, hc_out


def rec_rollout(cfg, state, params, traj, rec, step_offset=0, forced_actions=None, forced_uniforms=None):
    params = np.ascontiguousarray(params, np.float32)
    fa = None if forced_actions is None else np.ascontiguousarray(forced_actions, np.int32)
    fu = None if forced_uniforms is None else np.ascontiguousarray(forced_uniforms, np.float32)
    lib().orc_rec_rollout(C.byref(make_config(cfg)), state.c(), _ap(params), traj.c(), rec.c(), int(step_offset),
                          _ap(fa), _ap(fu))


def rec_minibatch_loss_grad(cfg, traj, rec, params_f64, envs, want_grad=True):
    params_f64 = np.ascontiguousarray(params_f64, np.float64)
    envs = np.ascontiguousarray(envs, np.int32)
    stats = np.zeros(6, np.float64)
    grad = np.zeros(params_f64.size, np.float64) if want_grad else None
    lib().orc_rec_minibatch_loss_grad_f64(C.byref(make_config(cfg)), traj.c(), rec.c(), _ap(params_f64), _ap(envs),
                                          envs.size, _ap(stats), _ap(grad))
    return stats, grad


def rec_ppo_update(cfg, traj, rec, params, adam_m, adam_v, adam_step0=0, perm=None):
    """In place on params / adam_m / adam_v (fp32).  perm [E][N] over environments.  Returns (stats, last gradient)."""
    E, M = cfg["n_epochs"], cfg["n_minibatches"]
    stats = np.zeros((E * M, 8), np.float32)
    grad = np.zeros(params.size, np.float32)
    pm = None if perm is None else np.ascontiguousarray(perm, np.int32)
    lib().orc_rec_ppo_update(C.byref(make_config(cfg)), traj.c(), rec.c(), _ap(params), _ap(adam_m), _ap(adam_v),
                             int(adam_step0), _ap(pm), _ap(stats), _ap(grad))
    return stats, grad

