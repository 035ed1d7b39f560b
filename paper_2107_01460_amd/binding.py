"""ctypes binding of libmarl_gfx950.so: same names as the C ABI, argument marshalling only."""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libmarl_gfx950.so")
N_ACTIONS = 6
N_STATS = 8


class MarlError(RuntimeError):
    pass


class Config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "grid", "n_agents", "n_food", "max_level", "episode_cap", "view", "n_envs", "rollout_len",
        "actor_hidden", "critic_hidden", "central_critic", "precision",
        "n_epochs", "n_minibatches", "normalize_adv", "clip_value")] + [(n, C.c_float) for n in (
        "gamma", "lambda_", "clip_eps", "ent_coef", "vf_coef", "max_grad_norm",
        "lr", "beta1", "beta2", "adam_eps")] + [("seed", C.c_uint64), ("recurrent", C.c_int32),
                                                   ("env_kind", C.c_int32)]


class EnvStateC(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("agent_row", "agent_col", "agent_lvl", "food_row", "food_col",
                                          "food_lvl", "t_in_ep", "episode_id")]


class TrajC(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("obs", "action", "logp", "value", "reward", "done", "last_value",
                                          "adv", "ret", "logits", "sampled")]


class Sizes(C.Structure):
    _fields_ = [(n, C.c_int64) for n in (
        "obs_dim", "critic_in_dim", "n_params", "n_actor_params",
        "state_entity_bytes_agents", "state_entity_bytes_food", "state_t_bytes", "state_episode_bytes",
        "obs_bytes", "step_scalar_bytes", "done_bytes", "last_value_bytes", "logits_bytes",
        "rollout_workspace_bytes", "update_workspace_bytes", "eval_workspace_bytes",
        "hidden_actor_bytes", "hidden_critic_bytes")]


class EvalStatsC(C.Structure):
    _fields_ = [("ret_sum", C.c_void_p), ("len_sum", C.c_void_p), ("episodes", C.c_void_p)]


class RecStateC(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("ha0", "hc0", "ha1", "hc1")]


EXPORTS = ("marl_query_sizes", "marl_env_reset", "marl_observe", "marl_env_step", "marl_policy_forward",
           "marl_sample_actions", "marl_rollout", "marl_rollout_static", "marl_compute_gae", "marl_ppo_update", "marl_train_step", "marl_evaluate", "marl_rollout_recurrent", "marl_ppo_update_recurrent",
           "marl_timing_enable",
           "marl_timing_read", "marl_status_string")

_lib = None


def lib():
    """The loaded library.  There is no fallback: a missing build is an error."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise MarlError(f"{_LIB_PATH} is missing: run `python -m paper_2107_01460_amd.build` first")
        L = C.CDLL(_LIB_PATH)
        cp = C.POINTER(Config)
        vp = C.c_void_p
        L.marl_query_sizes.argtypes = [cp, C.POINTER(Sizes)]
        L.marl_env_reset.argtypes = [cp, EnvStateC, vp]
        L.marl_observe.argtypes = [cp, EnvStateC, vp, vp]
        L.marl_env_step.argtypes = [cp, EnvStateC, vp, vp, vp, vp, vp]
        L.marl_policy_forward.argtypes = [cp, vp, vp, C.c_int64, vp, vp, vp, vp]
        L.marl_sample_actions.argtypes = [cp, vp, vp, vp, C.c_int64, C.c_uint64, vp, vp, vp, vp]
        L.marl_rollout.argtypes = [cp, EnvStateC, vp, TrajC, C.c_uint64, vp, vp, vp, vp]
        L.marl_rollout_static.argtypes = [cp, EnvStateC, vp, TrajC, C.c_uint64, vp, vp, vp]
        L.marl_compute_gae.argtypes = [cp, TrajC, vp]
        L.marl_ppo_update.argtypes = [cp, TrajC, vp, vp, vp, C.c_int64, vp, vp, vp, vp, vp]
        L.marl_train_step.argtypes = [cp, EnvStateC, vp, TrajC, vp, vp, vp, vp, vp, vp, vp, vp]
        L.marl_evaluate.argtypes = [cp, EnvStateC, vp, C.c_int32, EvalStatsC, vp, vp]
        L.marl_rollout_recurrent.argtypes = [cp, EnvStateC, vp, TrajC, RecStateC, C.c_uint64, vp, vp, vp, vp]
        L.marl_ppo_update_recurrent.argtypes = [cp, TrajC, RecStateC, vp, vp, vp, C.c_int64, vp, vp, vp, vp, vp]
        L.marl_timing_enable.argtypes = [C.c_int32]
        L.marl_timing_read.argtypes = [C.c_int32, C.POINTER(C.c_double), C.POINTER(C.c_int64), C.POINTER(C.c_double)]
        L.marl_status_string.argtypes = [C.c_int32]
        L.marl_status_string.restype = C.c_char_p
        for name in EXPORTS[:-1]:
            getattr(L, name).restype = C.c_int32
        _lib = L
    return _lib


def status_string(code):
    return lib().marl_status_string(int(code)).decode()


def _check(code):
    if code != 0:
        raise MarlError(f"marl error {code}: {status_string(code)}")


def make_config(cfg: dict) -> Config:
    c = Config()
    for name, _ in Config._fields_:
        setattr(c, name, cfg.get(name, 0) if name in ("recurrent", "env_kind") else cfg["lambda" if name == "lambda_" else name])
    return c


def _ptr(t):
    if t is None:
        return None
    assert t.is_contiguous()
    return C.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def query_sizes(cfg) -> Sizes:
    s = Sizes()
    _check(lib().marl_query_sizes(C.byref(make_config(cfg)), C.byref(s)))
    return s


def alloc_workspace(nbytes, device="cuda"):
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


class EnvState:
    """Caller-owned device buffers of the vectorised environment state."""
    FIELDS = ("agent_row", "agent_col", "agent_lvl", "food_row", "food_col", "food_lvl", "t_in_ep", "episode_id")

    def __init__(self, cfg, device="cuda"):
        N, A, F = cfg["n_envs"], cfg["n_agents"], cfg["n_food"]
        u8 = dict(dtype=torch.uint8, device=device)
        self.agent_row = torch.zeros((A, N), **u8)
        self.agent_col = torch.zeros((A, N), **u8)
        self.agent_lvl = torch.zeros((A, N), **u8)
        self.food_row = torch.zeros((F, N), **u8)
        self.food_col = torch.zeros((F, N), **u8)
        self.food_lvl = torch.zeros((F, N), **u8)
        self.t_in_ep = torch.zeros((N,), dtype=torch.int32, device=device)
        self.episode_id = torch.zeros((N,), dtype=torch.int32, device=device)  # bit pattern of uint32

    def c(self):
        return EnvStateC(*[getattr(self, f).data_ptr() for f in self.FIELDS])

    def load(self, host_state):
        """Copies a host state (numpy arrays with the same field names) to the device."""
        import numpy as np
        for f in self.FIELDS:
            src = getattr(host_state, f)
            if f == "episode_id":
                src = src.view(np.int32)
            getattr(self, f).copy_(torch.from_numpy(src.copy()))

    def to_host(self):
        import numpy as np
        out = {f: getattr(self, f).cpu().numpy() for f in self.FIELDS}
        out["episode_id"] = out["episode_id"].view(np.uint32)
        return out


class Traj:
    """Caller-owned device buffers of one rollout."""
    FIELDS = ("obs", "action", "logp", "value", "reward", "done", "last_value", "adv", "ret", "logits", "sampled")

    def __init__(self, cfg, device="cuda", debug=False):
        N, A, T, D = cfg["n_envs"], cfg["n_agents"], cfg["rollout_len"], 3 * cfg["view"] ** 2
        f32 = dict(dtype=torch.float32, device=device)
        i32 = dict(dtype=torch.int32, device=device)
        self.obs = torch.empty((T + 1, N, A, D), **f32)
        self.action = torch.zeros((T, N, A), **i32)
        self.logp = torch.zeros((T, N, A), **f32)
        self.value = torch.zeros((T, N, A), **f32)
        self.reward = torch.zeros((T, N, A), **f32)
        self.done = torch.zeros((T, N), dtype=torch.uint8, device=device)
        self.last_value = torch.zeros((N, A), **f32)
        self.adv = torch.zeros((T, N, A), **f32)
        self.ret = torch.zeros((T, N, A), **f32)
        self.logits = torch.zeros((T, N, A, N_ACTIONS), **f32) if debug else None
        self.sampled = torch.zeros((T, N, A), **i32) if debug else None

    def c(self):
        return TrajC(*[(getattr(self, f).data_ptr() if getattr(self, f) is not None else None) for f in self.FIELDS])


def env_reset(cfg, state, stream=None):
    _check(lib().marl_env_reset(C.byref(make_config(cfg)), state.c(), _stream(stream)))


def observe(cfg, state, obs, stream=None):
    _check(lib().marl_observe(C.byref(make_config(cfg)), state.c(), _ptr(obs), _stream(stream)))


def env_step(cfg, state, actions, obs, reward, done, stream=None):
    _check(lib().marl_env_step(C.byref(make_config(cfg)), state.c(), _ptr(actions), _ptr(obs), _ptr(reward),
                               _ptr(done), _stream(stream)))


def policy_forward(cfg, params, obs, n_rows, logits, value, workspace, stream=None):
    _check(lib().marl_policy_forward(C.byref(make_config(cfg)), _ptr(params), _ptr(obs), int(n_rows), _ptr(logits),
                                     _ptr(value), _ptr(workspace), _stream(stream)))


def sample_actions(cfg, logits, uniforms, forced, n, step, action, sampled, logp, stream=None):
    _check(lib().marl_sample_actions(C.byref(make_config(cfg)), _ptr(logits), _ptr(uniforms), _ptr(forced), int(n),
                                     int(step), _ptr(action), _ptr(sampled), _ptr(logp), _stream(stream)))


def rollout(cfg, state, params, traj, step_offset, workspace, forced_actions=None, forced_uniforms=None, stream=None):
    _check(lib().marl_rollout(C.byref(make_config(cfg)), state.c(), _ptr(params), traj.c(), int(step_offset),
                              _ptr(forced_actions), _ptr(forced_uniforms), _ptr(workspace), _stream(stream)))


def rollout_static(cfg, state, params, traj, step_offset, forced_actions=None, forced_uniforms=None, stream=None):
    """marl_rollout on the library's built-in scratch: no workspace argument, no allocation inside the call."""
    _check(lib().marl_rollout_static(C.byref(make_config(cfg)), state.c(), _ptr(params), traj.c(), int(step_offset),
                                     _ptr(forced_actions), _ptr(forced_uniforms), _stream(stream)))


def compute_gae(cfg, traj, stream=None):
    _check(lib().marl_compute_gae(C.byref(make_config(cfg)), traj.c(), _stream(stream)))


class EvalStats:
    """Caller-owned device buffers of an evaluation block's per-environment results."""

    def __init__(self, cfg, device="cuda"):
        N = cfg["n_envs"]
        self.ret_sum = torch.zeros((N,), dtype=torch.float32, device=device)
        self.len_sum = torch.zeros((N,), dtype=torch.int32, device=device)
        self.episodes = torch.zeros((N,), dtype=torch.int32, device=device)

    def c(self):
        return EvalStatsC(self.ret_sum.data_ptr(), self.len_sum.data_ptr(), self.episodes.data_ptr())


def evaluate(cfg, state, params, n_episodes, out, workspace, stream=None):
    _check(lib().marl_evaluate(C.byref(make_config(cfg)), state.c(), _ptr(params), int(n_episodes), out.c(),
                               _ptr(workspace), _stream(stream)))


class RecState:
    """Caller-owned hidden states of the recurrent networks around one rollout (h*0 in, h*1 out)."""

    def __init__(self, cfg, device="cuda"):
        N, A, Ha, Hc = cfg["n_envs"], cfg["n_agents"], cfg["actor_hidden"], cfg["critic_hidden"]
        cshape = (N, Hc) if cfg["central_critic"] else (N, A, Hc)
        f32 = dict(dtype=torch.float32, device=device)
        self.ha0, self.ha1 = torch.zeros((N, A, Ha), **f32), torch.zeros((N, A, Ha), **f32)
        self.hc0, self.hc1 = torch.zeros(cshape, **f32), torch.zeros(cshape, **f32)

    def c(self):
        return RecStateC(self.ha0.data_ptr(), self.hc0.data_ptr(), self.ha1.data_ptr(), self.hc1.data_ptr())

    def advance(self):
        """The state the last rollout left becomes the state the next one starts from."""
        self.ha0, self.ha1 = self.ha1, self.ha0
        self.hc0, self.hc1 = self.hc1, self.hc0


def rollout_recurrent(cfg, state, params, traj, rec, step_offset, workspace, forced_actions=None, forced_uniforms=None,
                      stream=None):
    _check(lib().marl_rollout_recurrent(C.byref(make_config(cfg)), state.c(), _ptr(params), traj.c(), rec.c(),
                                        int(step_offset), _ptr(forced_actions), _ptr(forced_uniforms), _ptr(workspace),
                                        _stream(stream)))


def ppo_update_recurrent(cfg, traj, rec, params, adam_m, adam_v, adam_step0, perm, stats, grad_dump, workspace, stream=None):
    _check(lib().marl_ppo_update_recurrent(C.byref(make_config(cfg)), traj.c(), rec.c(), _ptr(params), _ptr(adam_m),
                                           _ptr(adam_v), int(adam_step0), _ptr(perm), _ptr(stats), _ptr(grad_dump),
                                           _ptr(workspace), _stream(stream)))


def alloc_counters():
    """Device memory of one marl_counters (step, adam_step), zeroed: a [2] int64 tensor."""
    return torch.zeros(2, dtype=torch.int64, device="cuda")


def train_step(cfg, state, params, traj, adam_m, adam_v, counters, perm, stats, rollout_workspace, update_workspace,
               stream=None):
    _check(lib().marl_train_step(C.byref(make_config(cfg)), state.c(), _ptr(params), traj.c(), _ptr(adam_m),
                                 _ptr(adam_v), _ptr(counters), _ptr(perm), _ptr(stats), _ptr(rollout_workspace),
                                 _ptr(update_workspace), _stream(stream)))


KERNEL_CLASSES = {"gemm_nn": 0, "gemm_nt": 1, "gemm_tn": 2, "env_step": 3, "gae": 4, "fused_train": 5, "rollout": 6}


def timing_enable(on):
    _check(lib().marl_timing_enable(1 if on else 0))


def timing_read(kernel_class):
    """(total_ms, launches, work) of one kernel class since timing_enable(True)."""
    ms, n, w = C.c_double(), C.c_int64(), C.c_double()
    _check(lib().marl_timing_read(int(kernel_class), C.byref(ms), C.byref(n), C.byref(w)))
    return ms.value, n.value, w.value


def ppo_update(cfg, traj, params, adam_m, adam_v, adam_step0, perm, stats, grad_dump, workspace, stream=None):
    _check(lib().marl_ppo_update(C.byref(make_config(cfg)), traj.c(), _ptr(params), _ptr(adam_m), _ptr(adam_v),
                                 int(adam_step0), _ptr(perm), _ptr(stats), _ptr(grad_dump), _ptr(workspace),
                                 _stream(stream)))
