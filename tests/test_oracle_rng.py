"""Pins for the oracle's random-number layer: published Philox known answers, exact integer
and float mappings, and statistical sanity of the derived draws."""
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))


def test_philox_known_answers(orc):
    n = 0
    for line in open(os.path.join(HERE, "golden", "philox4x32_10_kat.txt")):
        if line.startswith("#") or not line.strip():
            continue
        w = [int(x, 16) for x in line.split()]
        out = orc.philox4x32_10(w[0:4], w[4:6])
        assert [int(x) for x in out] == w[6:10]
        n += 1
    assert n == 3


def test_rand_below_is_multiply_high(orc):
    # exact values: floor(x * n / 2^32)
    for x, n in [(0, 7), (0xFFFFFFFF, 7), (0x80000000, 2), (0x7FFFFFFF, 2), (0x55555556, 3), (123456789, 64)]:
        assert orc.rand_below(x, n) == (x * n) >> 32
    assert orc.rand_below(0xFFFFFFFF, 100) == 99


def test_rand_unit_open_interval_and_exact(orc):
    assert orc.rand_unit(0) == 0.5 / 2 ** 23
    assert orc.rand_unit(0xFFFFFFFF) == 1.0 - 0.5 / 2 ** 23
    assert orc.rand_unit(0x80000000) == 0.5 + 0.5 / 2 ** 23
    assert 0.0 < orc.rand_unit(0) and orc.rand_unit(0xFFFFFFFF) < 1.0


def test_round_bf16_rne(orc):
    assert orc.round_bf16(1.0) == 1.0
    # 1 + 2^-8 is exactly halfway between bf16 neighbours 1 and 1 + 2^-7: ties to even -> 1
    assert orc.round_bf16(1.0 + 2 ** -8) == 1.0
    assert orc.round_bf16(1.0 + 2 ** -7 + 2 ** -8) == 1.0 + 2 ** -6
    assert orc.round_bf16(1.0 + 2 ** -8 + 2 ** -20) == 1.0 + 2 ** -7
    assert orc.round_bf16(-3.0) == -3.0


def test_sampling_uniforms_statistics(orc):
    import workloads as W

    cfg = W.scaled(W.CONFIGS[0], n_envs=64)
    u = np.array([orc.sample_uniforms(cfg, s, e, a) for s in range(40) for e in range(64) for a in range(2)])
    assert u.shape == (5120, 6)
    assert 0 < u.min() and u.max() < 1
    m = u.size
    assert abs(u.mean() - 0.5) < 5 * np.sqrt(1 / 12 / m)
    assert abs(u.var() - 1 / 12) < 5 * np.sqrt(1 / 180 / m)
    # chi-square over 16 buckets
    hist = np.histogram(u, bins=16, range=(0, 1))[0]
    chi2 = ((hist - m / 16) ** 2 / (m / 16)).sum()
    assert chi2 < 45  # 15 dof, p ~ 1e-4
    # distinct (step, env, agent) keys give distinct draws; the same key repeats exactly
    assert len(np.unique(u[:, 0])) > 0.99 * len(u)
    assert np.array_equal(orc.sample_uniforms(cfg, 3, 5, 1), orc.sample_uniforms(cfg, 3, 5, 1))
    big = orc.sample_uniforms(cfg, (1 << 32) + 3, 5, 1)
    assert not np.array_equal(big, orc.sample_uniforms(cfg, 3, 5, 1))
