"""Whole training runs on the GPU: the loop of Fig. 2 with evaluation blocks in between (Section 3) learns.

The per-stage parity tests compare every kernel with the oracle on given inputs; this checks that the stages
fit together over thousands of iterations of the single-call training step: the greedy policy's mean episode
return rises from about zero and episodes end before the step cap.  The oracle shows the same rise on the same
workload (test_oracle_learning.py); the two runs are not comparable number by number (chaotic divergence after
the first near-tie), so each side has its own thresholds.
"""
import pytest
import torch

import workloads as W

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("k,n_envs,iterations,min_return", [(1, 64, 1500, 0.5), (2, 1024, 60, 1.5), (3, 256, 60, 1.0)])
def test_mean_return_rises(k, n_envs, iterations, min_return):
    from paper_2107_01460_amd.trainer import Trainer
    cfg = W.scaled(W.CONFIGS[k - 1], n_envs=n_envs)
    print("case", cfg["name"], "N", n_envs, flush=True)
    tr = Trainer(cfg, seed=1)
    ret0, len0 = tr.evaluate(8)
    tr.train(iterations)
    torch.cuda.synchronize()
    ret1, len1 = tr.evaluate(8)
    st = tr.last_stats()
    print("return", ret0, "->", ret1, "length", len0, "->", len1, st, flush=True)
    assert ret0 < 0.1
    assert ret1 > min_return
    assert len1 < len0 - 1.0
    assert st["non_finite"] == 0.0 and bool(torch.isfinite(tr.params).all())
    assert int(tr.counters[0]) == iterations * cfg["rollout_len"]
    assert int(tr.counters[1]) == iterations * cfg["n_epochs"] * cfg["n_minibatches"]
