"""The oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only): a sanitized build of the same
source runs an environment roll-out with resets, GAE and a PPO update in a child process, which must end without a
report.  The sanitized library is loaded with the sanitizer runtime preloaded, so it runs in its own interpreter."""
import os
import subprocess
import sys
import textwrap

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _runtime(name):
    out = subprocess.run(["g++", "-print-file-name=" + name], capture_output=True, text=True).stdout.strip()
    return out if os.path.isabs(out) and os.path.exists(out) else None


@pytest.mark.parametrize("recurrent,env_kind", [(0, 0), (1, 0), (0, 2)])
def test_oracle_runs_clean_under_asan_and_ubsan(tmp_path, recurrent, env_kind):
    asan = _runtime("libasan.so")
    if asan is None:
        pytest.skip("no libasan in this toolchain")
    lib = str(tmp_path / "libmarl_oracle_san.so")
    subprocess.check_call(["g++", "-O1", "-g", "-std=c++17", "-fPIC", "-shared", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-o", lib,
                           os.path.join(ROOT, "oracle", "marl_oracle.cpp")])
    code = textwrap.dedent(f"""
        import sys
        sys.path.insert(0, {ROOT!r})
        import numpy as np
        import oracle as orc
        import workloads as W
        orc._LIB = {lib!r}
        orc.build = lambda force=False: orc._LIB
        cfg = W.scaled(W.CONFIGS[1], n_envs=6, rollout_len=12, n_minibatches=2, n_epochs=2, episode_cap=5,
                       recurrent={recurrent}, env_kind={env_kind})
        if {env_kind}:
            cfg = W.scaled(cfg, max_level=2)
        params = W.init_params(cfg, bias_scale=0.1)
        s = orc.EnvState(cfg)
        orc.env_reset(cfg, s)
        tr = orc.Traj(cfg)
        m, v = np.zeros_like(params), np.zeros_like(params)
        if {recurrent}:
            rec = orc.RecState(cfg)
            orc.rec_rollout(cfg, s, params, tr, rec, 3)
            orc.compute_gae(cfg, tr)
            orc.rec_ppo_update(cfg, tr, rec, params, m, v, 0, W.make_env_perm(cfg))
        else:
            orc.rollout(cfg, s, params, tr, 3)
            orc.compute_gae(cfg, tr)
            orc.ppo_update(cfg, tr, params, m, v, 0, W.make_perm(cfg))
            orc.evaluate(cfg, s, params, 2)
        assert tr.done.sum() > 0 and np.isfinite(params).all()
        print("clean")
    """)
    preload = ":".join(x for x in (asan, os.environ.get("LD_PRELOAD", "")) if x)   # the sanitizer runtime first, the rest kept
    env = dict(os.environ, LD_PRELOAD=preload, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0:exitcode=23",
               UBSAN_OPTIONS="halt_on_error=1:exitcode=24")
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, env=env, timeout=600)
    assert r.returncode == 0, (r.returncode, r.stderr[-3000:])
    assert "clean" in r.stdout
    assert "ERROR: AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr
