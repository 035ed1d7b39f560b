"""Run-to-run determinism on the GPU: the same rollout + GAE + update from the same buffers, twice.

The environment, the sampler and GAE have no reductions, so state and trajectory must be equal bit for bit.  The
gradient of the networks that take the whole-network training kernel is reduced in a fixed order (the shares inside a
workgroup added in turn through LDS, the per-workgroup copies added in a fixed grouping, the gradient norm as per-block
shares added by a fixed tree),
so their parameters must be equal bit for bit as well, and so are the layer-by-layer kernels of the 256-wide fp32
critic (k splits and per-workgroup copies added in a fixed order); the bf16 configuration still meets in fp32 atomics and
is held to 0.1 of the parameter change in its norm.  The reported loss statistics are summed with atomics in every configuration."""
import numpy as np
import pytest
import torch

import workloads as W
from gpu_util import dev, small

pytestmark = pytest.mark.gpu

TRAJ = ("obs", "action", "logp", "value", "reward", "done", "last_value", "adv", "ret")


def one_run(M, cfg, params0, perm):
    st = M.EnvState(cfg)
    M.env_reset(cfg, st)
    tr = M.Traj(cfg)
    sizes = M.query_sizes(cfg)
    ws_r, ws_u = M.alloc_workspace(sizes.rollout_workspace_bytes), M.alloc_workspace(sizes.update_workspace_bytes)
    p = dev(params0)
    m, v = torch.zeros_like(p), torch.zeros_like(p)
    stats = torch.zeros((cfg["n_epochs"] * cfg["n_minibatches"], 8), device="cuda")
    snaps = []
    for it in range(2):
        M.rollout(cfg, st, p, tr, it * cfg["rollout_len"], ws_r)
        M.compute_gae(cfg, tr)
        torch.cuda.synchronize()
        out = {f: getattr(tr, f).cpu().numpy() for f in TRAJ}
        out.update({"state." + f: x for f, x in st.to_host().items()})
        snaps.append(out)
        M.ppo_update(cfg, tr, p, m, v, it * cfg["n_epochs"] * cfg["n_minibatches"], dev(perm), stats, None, ws_u)
        torch.cuda.synchronize()
        snaps[-1]["stats"] = stats.cpu().numpy().copy()
    return snaps, p.cpu().numpy(), m.cpu().numpy(), v.cpu().numpy(), stats.cpu().numpy()


# (3, 8192): 65 536 critic rows per minibatch, the size from which the 256-wide critic takes its register-resident kernels
@pytest.mark.parametrize("k,exact,n_envs", [(2, True, 1024), (3, True, 512), (3, True, 8192), (4, False, 96), (1, True, 700),
                                            (5, True, 3000)])
def test_two_runs_agree(k, exact, n_envs):
    import paper_2107_01460_amd as M
    cfg = small(k, n_envs=n_envs, rollout_len=16, n_minibatches=2, n_epochs=2)
    print("case", cfg["name"], flush=True)
    params0 = W.init_params(cfg, bias_scale=0.1)
    perm = W.make_perm(cfg)
    a = one_run(M, cfg, params0, perm)
    b = one_run(M, cfg, params0, perm)
    for f in a[0][0]:
        if f != "stats":
            assert np.array_equal(a[0][0][f], b[0][0][f]), f
    if exact:
        for f in a[0][1]:                                  # the second rollout ran under the updated parameters
            if f != "stats":
                assert np.array_equal(a[0][1][f], b[0][1][f]), f
        for x, y, name in zip(a[1:4], b[1:4], ("params", "adam_m", "adam_v")):
            assert np.array_equal(x.view(np.uint32), y.view(np.uint32)), name
    else:
        scale = np.abs(a[1] - params0).max()
        assert scale > 0
        if cfg["precision"] == 0:
            # 1e-5 of the largest parameter change, plus the rounding of the parameters themselves (an fp32 parameter
            # of magnitude 0.3 moves in steps of 3e-8, more than 1e-5 of a 2e-3 change)
            assert np.abs(a[1] - b[1]).max() <= 1e-5 * scale + 2 * np.spacing(np.abs(a[1]).max())
        else:
            # bf16 configuration: a master weight that differs in its last bit can round to the other bf16 neighbour,
            # which moves the next minibatch's gradient by 2^-9 of that weight's contribution; Adam then turns a
            # near-zero gradient element of either sign into a full step of lr, so single parameters may differ by
            # whole steps between two runs.  The runs are compared in the norm of the parameter change.
            da, db = a[1].astype(np.float64) - params0, b[1].astype(np.float64) - params0
            assert np.linalg.norm(da - db) <= 0.1 * np.linalg.norm(da)
    if cfg["precision"] == 0:
        assert np.allclose(a[4], b[4], rtol=1e-5, atol=1e-6)
    else:   # the first minibatch of the first update runs on identical parameters; later ones on weights that may have
        # rounded differently
        assert np.allclose(a[0][0]["stats"][0], b[0][0]["stats"][0], rtol=1e-4, atol=1e-6)
        assert np.allclose(a[4], b[4], rtol=0.2, atol=2e-3)
