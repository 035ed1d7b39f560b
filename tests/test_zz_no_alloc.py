"""marl_rollout_static (the rollout on the library's built-in scratch, for callers that cannot allocate) against
marl_rollout on a caller-owned workspace: same kernels, so every output must be equal bit for bit.  Two calls in a row,
the second on a smaller input, so that whatever the first call left in the scratch is seen not to matter."""
import ctypes as C

import numpy as np
import pytest
import torch

import workloads as W
from gpu_util import small

pytestmark = pytest.mark.gpu

FIELDS = ("obs", "action", "logp", "value", "reward", "done", "last_value", "logits", "sampled")


def run(M, cfg, params, static, step_offset):
    st = M.EnvState(cfg)
    M.env_reset(cfg, st)
    tr = M.Traj(cfg, debug=True)
    for f in FIELDS:                       # stale contents must not survive
        getattr(tr, f).fill_(7)
    if static:
        M.rollout_static(cfg, st, params, tr, step_offset)
    else:
        ws = M.alloc_workspace(M.query_sizes(cfg).rollout_workspace_bytes)
        M.rollout(cfg, st, params, tr, step_offset, ws)
    torch.cuda.synchronize()
    out = {f: getattr(tr, f).cpu().numpy() for f in FIELDS}
    out.update({"state." + f: v for f, v in st.to_host().items()})
    return out


def test_rollout_static_equals_rollout_on_two_calls_in_a_row():
    import paper_2107_01460_amd as M
    assert torch.cuda.is_available()
    first = small(3, n_envs=300, rollout_len=12)                 # centralised critic, H = 128 / 256
    second = small(2, n_envs=37, rollout_len=11, n_minibatches=1)   # smaller: fewer envs, other shapes
    for i, cfg in enumerate((first, second)):
        print("case", cfg["name"], cfg["n_envs"], flush=True)
        params = torch.from_numpy(W.init_params(cfg, bias_scale=0.1)).cuda()
        got = run(M, cfg, params, True, 1000 * i)
        ref = run(M, cfg, params, False, 1000 * i)
        for k in ref:
            assert np.array_equal(got[k], ref[k]), (cfg["name"], k)
        assert ref["done"].sum() > 0 and np.abs(ref["reward"]).sum() > 0


def test_rollout_static_rejects_what_does_not_fit():
    import paper_2107_01460_amd as M
    cfg = W.CONFIGS[3]                                           # bf16: per-step activations go through the workspace
    assert M.query_sizes(cfg).rollout_workspace_bytes > 8 * 1024 * 1024
    good = 0x10000
    st = M.binding.EnvStateC(*([good] * 8))
    traj = M.binding.TrajC(*([good] * 9 + [None, None]))
    rc = M.lib().marl_rollout_static(C.byref(M.make_config(cfg)), st, good, traj, 0, None, None, None)
    assert rc == -5
