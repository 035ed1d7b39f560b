"""Throughput of the fused multi-agent PPO training step on one MI355X.

A step = rollout (T env steps of N envs with policy inference and sampling) + GAE + PPO update
(E epochs x M minibatches) on synthetic, seeded inputs that are resident in HBM before the timed region.
Prints one JSON line: env-agent steps per second of the headline workload, the roofline figures of its dominant
kernel measured live with HIP events, short runs of the other four workloads of the list ("workloads"), and the
CPU oracle timed on a bounded sample of the headline workload (one core, and all host cores).
"""
import argparse
import json
import os
import re
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

# envs the CPU oracle is timed on per process: the same config with full T, A, networks, E and M
# (cost is linear in the number of envs; about 10 s of work on one core)
ORACLE_SAMPLE_ENVS = {1: 64, 2: 64, 3: 48, 4: 2, 5: 2048}
ORACLE_MAX_PROCS = 16          # the CPU share of a one-GPU machine, whatever the affinity mask shows
PEAK = {"mfma_f32": 157.3, "mfma_bf16": 2500.0, "hbm": 8000.0}   # TFLOP/s, TFLOP/s, GB/s
# (timed steps, warm-up steps) of the short runs of the other workloads in the default invocation
SIDE_RUNS = {1: (300, 30), 2: (30, 4), 3: (8, 2), 4: (4, 1), 5: (20, 3)}
# rocprofv3 PMC summaries (FETCH_SIZE / WRITE_SIZE per launch, scaled by a plain copy of known size) by workload, and
# the kernel-name prefix of each timed kernel class in them
PMC_PROFILE = {"c3_15x15_4ag_mappo": "profiles/bench_c3_pmc_hbm_traffic.txt",
               "c5_8x8_2ag_ippo_wide": "profiles/bench_c5_pmc_hbm_traffic.txt"}
CLASS_KERNEL = {"fused_train": "fused_train_kernel<", "env_step": "env_step_kernel<", "gae": "gae_kernel",
                "rollout": "rollout_fused_kernel<"}


def gemm_flops_per_step(cfg, W):
    """Algorithmic MLP flops of one training step (hidden-layer GEMMs only, forward and backward)."""
    D, A, T, N = W.obs_dim(cfg), cfg["n_agents"], cfg["rollout_len"], cfg["n_envs"]
    Ha, Hc, Dc = cfg["actor_hidden"], cfg["critic_hidden"], W.critic_in_dim(cfg)
    S = N * A * T
    Sc = N * T if cfg["central_critic"] else S
    if cfg.get("recurrent", 0):
        # cell forward: embedding D*H + input and hidden gate products 3*H*H each; backward: the four gate-side
        # products (dWi, dWh, dE, dh) 3*H*H each and dWe
        fa, fc = 2 * (D * Ha + 6 * Ha * Ha), 2 * (Dc * Hc + 6 * Hc * Hc)
        ba, bc = 2 * (D * Ha + 12 * Ha * Ha), 2 * (Dc * Hc + 12 * Hc * Hc)
        return S * fa + (Sc + Sc // T) * fc + cfg["n_epochs"] * (S * (fa + ba) + Sc * (fc + bc))
    fwd_a, fwd_c = 2 * (D * Ha + Ha * Ha), 2 * (Dc * Hc + Hc * Hc)
    roll = S * fwd_a + (Sc + Sc // T) * fwd_c
    # update: forward + (dW2, dZ1, dW1) backward GEMMs = 2DH + 2HH + 2HH + 2HH + 2DH per sample and epoch
    upd = cfg["n_epochs"] * (S * (2 * fwd_a + 2 * Ha * Ha) + Sc * (2 * fwd_c + 2 * Hc * Hc))
    return roll + upd


def pmc_traffic(cfg_name, kernel_class):
    """HBM bytes per launch (read + write) of a kernel class from the committed rocprofv3 PMC summary of the workload.
    None when the workload or the class has no summary; an error when the summary exists but does not list the kernel
    (the profile no longer describes the build)."""
    path, prefix = PMC_PROFILE.get(cfg_name), CLASS_KERNEL.get(kernel_class)
    if path is None or prefix is None:
        return None, None
    full = os.path.join(ROOT, path)
    if not os.path.exists(full):
        raise RuntimeError(f"{path} is missing: bench.py quotes its HBM traffic figures")
    best = None
    for ln in open(full):
        if ln.startswith(prefix):
            mb = re.findall(r"->\s+([0-9.]+) MB", ln)
            n = re.search(r"\bn=\s*(\d+)", ln)
            if len(mb) == 2 and n:
                cand = (int(n.group(1)), (float(mb[0]) + float(mb[1])) * 1e6)
                best = cand if best is None or cand[0] > best[0] else best   # the instantiation launched most often
    if best is None:
        raise RuntimeError(f"{path} lists no kernel named {prefix}...: refresh the profile for this build")
    return best[1], path


# ---- CPU oracle beside it ---------------------------------------------------------------------------------------------

def oracle_one_step(cfg_id, n_envs, slice_index, recurrent, env_kind=0):
    """One training step of the oracle on n_envs environments of workload cfg_id; returns (env-agent steps, seconds).
    Slices of different processes are made disjoint through the seed (environment layouts and sampling are keyed by
    (seed, environment index))."""
    import oracle as orc
    import workloads as W
    cfg = W.CONFIGS[cfg_id - 1]
    c = W.scaled(cfg, n_envs=n_envs, seed=cfg["seed"] + 7919 * slice_index, recurrent=1 if recurrent else 0)
    if env_kind:
        c = W.scaled(c, env_kind=env_kind, max_level=min(c["max_level"], c["n_food"]))
    params = W.init_params(c)
    s = orc.EnvState(c)
    orc.env_reset(c, s)
    tr = orc.Traj(c)
    m, v = np.zeros_like(params), np.zeros_like(params)
    perm = W.make_env_perm(c) if recurrent else W.make_perm(c)
    t0 = time.perf_counter()
    if recurrent:
        rec = orc.RecState(c)
        orc.rec_rollout(c, s, params, tr, rec, 0)
        orc.compute_gae(c, tr)
        orc.rec_ppo_update(c, tr, rec, params, m, v, 0, perm)
    else:
        orc.rollout(c, s, params, tr, 0)
        orc.compute_gae(c, tr)
        orc.ppo_update(c, tr, params, m, v, 0, perm)
    return n_envs * c["n_agents"] * c["rollout_len"], time.perf_counter() - t0


def oracle_envs(cfg_id, cfg, recurrent):
    n_o = min(cfg["n_envs"], ORACLE_SAMPLE_ENVS[cfg_id])
    if recurrent:   # sequence minibatches: whole environments per minibatch; the recurrent oracle is about 4x slower
        n_o = max(cfg["n_minibatches"], n_o // 4 // cfg["n_minibatches"] * cfg["n_minibatches"])
    while (n_o * cfg["rollout_len"]) % cfg["n_minibatches"]:
        n_o += 1
    return n_o


def run_cpu_baseline(cfg_id, cfg, recurrent, env_kind=0):
    """The oracle as it stands (g++ -O2, one thread per process), one training step on a bounded sample: first one
    process, then P independent processes at once on disjoint slices (P = host cores available to this process)."""
    n_o = oracle_envs(cfg_id, cfg, recurrent)
    steps1, dt1 = oracle_one_step(cfg_id, n_o, 0, recurrent, env_kind)
    avail = len(os.sched_getaffinity(0))
    P = max(1, min(avail, ORACLE_MAX_PROCS))
    cmd = [sys.executable, os.path.abspath(__file__), "--oracle-worker", "--config", str(cfg_id), "--oracle-envs", str(n_o),
           "--env-kind", str(env_kind)]
    if recurrent:
        cmd.append("--recurrent")
    t0 = time.perf_counter()
    procs = [subprocess.Popen(cmd + ["--oracle-slice", str(p + 1)], stdout=subprocess.PIPE, text=True) for p in range(P)]
    results = []
    for p in procs:
        out, _ = p.communicate()
        if p.returncode != 0:
            raise RuntimeError("an oracle worker failed")
        results.append(json.loads(out.strip().splitlines()[-1]))
    wall = time.perf_counter() - t0
    slowest = max(r["seconds"] for r in results)
    total = sum(r["steps"] for r in results)
    desc = (f"{n_o} of {cfg['n_envs']} envs per process, full T={cfg['rollout_len']}, A={cfg['n_agents']}, networks, "
            f"E={cfg['n_epochs']}, M={cfg['n_minibatches']}; one training step; g++ -O2, no OpenMP, one thread per process")
    return {"value": total / slowest, "unit": "env-agent steps/s", "cores": P, "kind": "oracle",
            "sample": f"{P} independent processes at once on disjoint slices ({desc}); slowest process {slowest:.1f} s, "
                      f"{wall:.1f} s with start-up; {avail} cores in the affinity mask, at most {ORACLE_MAX_PROCS} used",
            "single_core": {"value": steps1 / dt1, "unit": "env-agent steps/s", "cores": 1,
                            "sample": f"one process, {desc}, {dt1:.1f} s"}}


# ---- the GPU measurement ---------------------------------------------------------------------------------------------

def measure(M, W, torch, cfg, steps, warmup, recurrent=False, graph=False, calibration_copy=False):
    """Times `steps` training steps of one workload (after `warmup` untimed ones) and then the same steps once more with
    per-launch event timers on.  Returns the figures of the JSON line for that workload."""
    sizes = M.query_sizes(cfg)
    dev = lambda x: torch.from_numpy(np.ascontiguousarray(x)).cuda()
    state = M.EnvState(cfg)
    traj = M.Traj(cfg)
    params = dev(W.init_params(cfg))
    adam_m, adam_v = torch.zeros_like(params), torch.zeros_like(params)
    perm = dev(W.make_env_perm(cfg) if recurrent else W.make_perm(cfg))
    rec = M.RecState(cfg) if recurrent else None
    E, Mb, T = cfg["n_epochs"], cfg["n_minibatches"], cfg["rollout_len"]
    stats = torch.zeros((E * Mb, 8), device="cuda")
    ws_r = M.alloc_workspace(sizes.rollout_workspace_bytes)
    ws_u = M.alloc_workspace(sizes.update_workspace_bytes)
    M.env_reset(cfg, state)
    it = [0]

    def step():
        i = it[0]
        if rec is not None:
            M.rollout_recurrent(cfg, state, params, traj, rec, i * T, ws_r)
            M.compute_gae(cfg, traj)
            M.ppo_update_recurrent(cfg, traj, rec, params, adam_m, adam_v, i * E * Mb, perm, stats, None, ws_u)
            rec.advance()
        else:
            M.rollout(cfg, state, params, traj, i * T, ws_r)
            M.compute_gae(cfg, traj)
            M.ppo_update(cfg, traj, params, adam_m, adam_v, i * E * Mb, perm, stats, None, ws_u)
        it[0] += 1

    if calibration_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").fill_(1.0)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if graph:
        # one ordinary call (it also sets kernel attributes), then the same call captured once and replayed: the step
        # offset of the sampling keys and Adam's step count live in device memory and advance there
        counters = M.alloc_counters()
        one_call = lambda: M.train_step(cfg, state, params, traj, adam_m, adam_v, counters, perm, stats, ws_r, ws_u)
        one_call()
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            one_call()
        timed_step = g.replay
        it[0] = 1
    else:
        timed_step = step
    for _ in range(warmup):
        timed_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        timed_step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    if graph:
        it[0] += warmup + steps
    # the same K steps once more with per-launch event timers on, for the per-kernel figures (the events cost a
    # few microseconds per launch, so they stay out of the timing above)
    M.timing_enable(True)
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    classes = {name: M.timing_read(cls) for name, cls in M.KERNEL_CLASSES.items()}
    # the environment step alone (transition + observation under fixed random actions): inside the rollout it is part
    # of the fused rollout kernel, so its HBM figures come from a loop of marl_env_step calls on the same state
    acts = torch.randint(0, 6, (cfg["n_envs"], cfg["n_agents"]), dtype=torch.int32, device="cuda")
    M.timing_enable(True)
    for _ in range(100):
        M.env_step(cfg, state, acts, traj.obs[0], traj.reward[0], traj.done[0])
    torch.cuda.synchronize()
    classes["env_step"] = M.timing_read(M.KERNEL_CLASSES["env_step"])
    M.timing_enable(False)
    mfma_peak = PEAK["mfma_bf16"] if cfg["precision"] == 1 else PEAK["mfma_f32"]
    ms_step = 1e3 * dt / steps

    def line(name):
        ms, n, work = classes[name]
        if n == 0 or ms <= 0:
            return None
        mfma = name.startswith("gemm") or name in ("fused_train", "rollout")
        a = work / (ms * 1e-3) / (1e12 if mfma else 1e9)
        peak = mfma_peak if mfma else PEAK["hbm"]
        traffic, source = pmc_traffic(cfg["name"], name)
        # share_of_step: the class's event time per step against the un-instrumented step time
        out = {"kernel": name, "bound": "mfma" if mfma else "hbm", "achieved": a, "peak": peak,
               "unit": "TFLOP/s" if mfma else "GB/s", "frac": a / peak, "traffic": traffic, "launches": n,
               "avg_us": 1e3 * ms / n, "share_of_step": None if name == "env_step" else (ms / steps) / ms_step}
        if name == "env_step":
            out["note"] = "marl_env_step alone, 100 calls under fixed actions; in the rollout it is part of the fused kernel"
        if source:
            out["traffic_source"] = source
        return out

    lines = [l for l in (line(k) for k in M.KERNEL_CLASSES) if l]
    st = stats.cpu().numpy()
    assert np.all(np.isfinite(st)) and np.all(st[:, 7] == 0), "non-finite loss"
    S = cfg["n_envs"] * cfg["n_agents"] * T
    tf_step = gemm_flops_per_step(cfg, W) / 1e12
    res = {"value": S * steps / dt, "ms_per_step": ms_step, "steps": steps, "warmup": warmup,
           "dtype": "bf16" if cfg["precision"] == 1 else "f32", "env_agent_steps_per_step": S,
           "mlp_gemm_tflop_per_step": tf_step, "mlp_gemm_tflops_end_to_end": tf_step / (dt / steps),
           "mlp_frac_of_mfma_peak_end_to_end": tf_step / (dt / steps) / mfma_peak, "lines": lines,
           "launch": "hip_graph_replay" if graph else "per_kernel"}
    res["_keep"] = (state, traj, params, sizes)
    return res


def dominant(lines):
    mf = [l for l in lines if l["bound"] == "mfma"]
    return dict(max(mf, key=lambda l: l["share_of_step"] or 0.0)) if mf else None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=3, help="1-based workload index (default 3: MAPPO 15x15, 16384 envs)")
    ap.add_argument("--n-envs", type=int, default=0,
                    help="override the number of environments of the workload (scalability sweep); 0 = the workload's own")
    ap.add_argument("--env-kind", type=int, default=0,
                    help="0: the foraging world of the workload list; 1 / 2: the warehouse world at the same shape "
                         "(2: episodes also end on a collision)")
    ap.add_argument("--recurrent", action="store_true",
                    help="the workload with recurrent networks (a GRU cell in place of the second hidden layer)")
    ap.add_argument("--eval-episodes", type=int, default=0,
                    help="also time one greedy evaluation block of this many episodes per environment (reported as \"eval\")")
    ap.add_argument("--graph", action="store_true",
                    help="time replays of one HIP graph of the single-call training step (marl_train_step) instead of "
                         "the three calls launched kernel by kernel: for the small, launch-bound workloads")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--only", action="store_true", help="the named workload only: no short runs of the other four")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="run one plain 1 GiB device copy before the warm-up (a kernel of known traffic for scaling PMC counters)")
    ap.add_argument("--oracle-worker", action="store_true", help=argparse.SUPPRESS)   # one process of the all-cores CPU figure
    ap.add_argument("--oracle-envs", type=int, default=0, help=argparse.SUPPRESS)
    ap.add_argument("--oracle-slice", type=int, default=0, help=argparse.SUPPRESS)
    args = ap.parse_args()
    if args.oracle_worker:   # CPU only: touches neither torch.cuda nor the HIP library
        steps, seconds = oracle_one_step(args.config, args.oracle_envs, args.oracle_slice, args.recurrent, args.env_kind)
        print(json.dumps({"steps": steps, "seconds": seconds}))
        return
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2107_01460_amd as M
    import workloads as W

    torch.cuda.set_device(0)
    cfg = W.CONFIGS[args.config - 1]
    variant = bool(args.n_envs or args.env_kind or args.recurrent or args.graph)
    if args.n_envs:
        cfg = W.scaled(cfg, n_envs=args.n_envs, name="%s@N=%d" % (cfg["name"], args.n_envs))
    if args.env_kind:
        cfg = W.scaled(cfg, env_kind=args.env_kind, max_level=min(cfg["max_level"], cfg["n_food"]),
                       name=cfg["name"] + ("+warehouse" if args.env_kind == 1 else "+warehouse_collision_ends"))
    if args.recurrent:
        if cfg["precision"] != 0:
            print("the recurrent networks are fp32 only", file=sys.stderr)
            sys.exit(2)
        cfg = W.scaled(cfg, recurrent=1, name=cfg["name"] + "+gru")
    if args.graph and args.recurrent:
        print("--graph covers the feed-forward training step only", file=sys.stderr)
        sys.exit(2)

    head = measure(M, W, torch, cfg, args.steps, args.warmup, recurrent=args.recurrent, graph=args.graph,
                   calibration_copy=args.calibration_copy)
    state, traj, params, sizes = head.pop("_keep")
    lines = head.pop("lines")
    E, Mb, T = cfg["n_epochs"], cfg["n_minibatches"], cfg["rollout_len"]
    out = {
        "metric": "env-agent steps/sec (rollout+PPO update) on 1 MI355X",
        "value": head["value"], "unit": "env-agent steps/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": head["dtype"], "data": "synthetic",
        "config": {"workload": cfg["name"], "config_index": args.config, "n_envs": cfg["n_envs"],
                   "n_agents": cfg["n_agents"], "rollout_len": T, "epochs": E, "minibatches": Mb,
                   "env_agent_steps_per_step": head["env_agent_steps_per_step"], "launch": head["launch"],
                   "mlp_gemm_tflop_per_step": head["mlp_gemm_tflop_per_step"]},
        "roofline": dominant(lines),
        "roofline_all": lines,
        "mlp_gemm_tflops_end_to_end": head["mlp_gemm_tflops_end_to_end"],
    }
    if args.eval_episodes > 0 and not args.recurrent:
        ev_state, ev_out = M.EnvState(cfg), M.EvalStats(cfg)
        ws_e = M.alloc_workspace(sizes.eval_workspace_bytes)
        ev_ms = []
        for _ in range(2):  # the second call is the timed one
            M.env_reset(cfg, ev_state)
            torch.cuda.synchronize()
            t2 = time.perf_counter()
            M.evaluate(cfg, ev_state, params, args.eval_episodes, ev_out, ws_e)
            torch.cuda.synchronize()
            ev_ms.append(1e3 * (time.perf_counter() - t2))
        n_steps = args.eval_episodes * cfg["episode_cap"]
        counted = int(ev_out.len_sum.sum().item())
        out["eval"] = {"episodes_per_env": args.eval_episodes, "env_steps_taken": n_steps, "ms": ev_ms[-1],
                       "env_agent_steps_per_s": cfg["n_envs"] * cfg["n_agents"] * n_steps / (ev_ms[-1] * 1e-3),
                       "counted_env_steps": counted,
                       "mean_episode_return": float(ev_out.ret_sum.sum().item()) / float(ev_out.episodes.sum().item())}
    del state, traj, params
    torch.cuda.empty_cache()
    # short runs of the other workloads of the list, so that one invocation shows all five
    if not args.only and not variant:
        side = {}
        for k in range(1, 6):
            if k == args.config:
                continue
            c = W.CONFIGS[k - 1]
            r = measure(M, W, torch, c, *SIDE_RUNS[k])
            r.pop("_keep")
            ls = r.pop("lines")
            by = {l["kernel"]: l for l in ls}
            r["roofline"] = dominant(ls)
            r["env_step"], r["gae"], r["rollout"] = by.get("env_step"), by.get("gae"), by.get("rollout")
            side[c["name"]] = r
            torch.cuda.empty_cache()
        out["workloads"] = side
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = run_cpu_baseline(args.config, W.CONFIGS[args.config - 1], args.recurrent, args.env_kind)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
