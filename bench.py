"""Throughput of the fused multi-agent PPO training step on one MI355X.

A step = rollout (T env steps of N envs with policy inference and sampling) + GAE + PPO update
(E epochs x M minibatches) on synthetic, seeded inputs that are resident in HBM before the timed region.
Prints one JSON line: env-agent steps per second, the roofline figures of the dominant kernel measured
live with HIP events, and the CPU oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

# env-agent steps the CPU oracle is timed on: envs of the same config with full T, A, networks, E and M
ORACLE_SAMPLE_ENVS = {1: 64, 2: 64, 3: 64, 4: 2, 5: 2048}
PEAK = {"mfma_f32": 157.3, "mfma_bf16": 2500.0, "hbm": 8000.0}   # TFLOP/s, TFLOP/s, GB/s
# HBM bytes per launch (read + write) of the dominant kernel, from the rocprofv3 PMC runs summarised in
# profiles/bench_c3_pmc_hbm_traffic.txt (FETCH_SIZE x 2.000 and WRITE_SIZE x 1.000 after the 1 GiB copy calibration).
PMC_TRAFFIC_BYTES = {("c3_15x15_4ag_mappo", "fused_train"): 450.4e6 + 80.8e6}


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


def run_cpu_baseline(cfg_id, cfg, W):
    import oracle as orc
    n_o = min(cfg["n_envs"], ORACLE_SAMPLE_ENVS[cfg_id])
    c = W.scaled(cfg, n_envs=n_o)
    if c.get("recurrent", 0):
        n_o = max(c["n_minibatches"], n_o // 4 // c["n_minibatches"] * c["n_minibatches"])
        c = W.scaled(cfg, n_envs=n_o)
    params = W.init_params(c)
    s = orc.EnvState(c)
    orc.env_reset(c, s)
    tr = orc.Traj(c)
    m, v = np.zeros_like(params), np.zeros_like(params)
    t0 = time.perf_counter()
    if c.get("recurrent", 0):
        rec = orc.RecState(c)
        orc.rec_rollout(c, s, params, tr, rec, 0)
        orc.compute_gae(c, tr)
        orc.rec_ppo_update(c, tr, rec, params, m, v, 0, W.make_env_perm(c))
    else:
        orc.rollout(c, s, params, tr, 0)
        orc.compute_gae(c, tr)
        orc.ppo_update(c, tr, params, m, v, 0, W.make_perm(c))
    dt = time.perf_counter() - t0
    steps = n_o * c["n_agents"] * c["rollout_len"]
    return {"value": steps / dt, "unit": "env-agent steps/s", "cores": 1, "kind": "oracle",
            "sample": f"{n_o} of {cfg['n_envs']} envs, full T={c['rollout_len']}, A={c['n_agents']}, networks, "
                      f"E={c['n_epochs']}, M={c['n_minibatches']}; one training step, {dt:.1f} s, g++ -O2 single thread"}


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
    ap.add_argument("--calibration-copy", action="store_true",
                    help="run one plain 1 GiB device copy before the warm-up (a kernel of known traffic for scaling PMC counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2107_01460_amd as M
    import workloads as W

    torch.cuda.set_device(0)
    cfg = W.CONFIGS[args.config - 1]
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
    sizes = M.query_sizes(cfg)
    dev = lambda x: torch.from_numpy(np.ascontiguousarray(x)).cuda()
    state = M.EnvState(cfg)
    traj = M.Traj(cfg)
    params = dev(W.init_params(cfg))
    adam_m, adam_v = torch.zeros_like(params), torch.zeros_like(params)
    perm = dev(W.make_env_perm(cfg) if args.recurrent else W.make_perm(cfg))
    rec = M.RecState(cfg) if args.recurrent else None
    E, Mb = cfg["n_epochs"], cfg["n_minibatches"]
    stats = torch.zeros((E * Mb, 8), device="cuda")
    ws_r = M.alloc_workspace(sizes.rollout_workspace_bytes)
    ws_u = M.alloc_workspace(sizes.update_workspace_bytes)
    M.env_reset(cfg, state)
    T = cfg["rollout_len"]
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

    if args.calibration_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").fill_(1.0)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if args.graph:
        # one ordinary call (it also sets kernel attributes), then the same call captured once and replayed: the step
        # offset of the sampling keys and Adam's step count live in device memory and advance there
        counters = M.alloc_counters()
        one_call = lambda: M.train_step(cfg, state, params, traj, adam_m, adam_v, counters, perm, stats, ws_r, ws_u)
        one_call()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            one_call()
        timed_step = graph.replay
        it[0] = 1
    else:
        timed_step = step
    for _ in range(args.warmup):
        timed_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        timed_step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    if args.graph:
        it[0] += args.warmup + args.steps
    # the same K steps once more with per-launch event timers on, for the per-kernel figures (the events cost a
    # few microseconds per launch, so they stay out of the headline timing above)
    M.timing_enable(True)
    t1 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt_timed = time.perf_counter() - t1
    classes = {}
    for name, cls in M.KERNEL_CLASSES.items():
        ms, n, work = M.timing_read(cls)
        classes[name] = (ms, n, work)
    M.timing_enable(False)
    mfma_peak = PEAK["mfma_bf16"] if cfg["precision"] == 1 else PEAK["mfma_f32"]

    def line(name):
        ms, n, work = classes[name]
        if n == 0 or ms <= 0:
            return None
        if name.startswith("gemm") or name == "fused_train":
            a = work / (ms * 1e-3) / 1e12
            return {"kernel": name, "bound": "mfma", "achieved": a, "peak": mfma_peak, "unit": "TFLOP/s",
                    "frac": a / mfma_peak, "traffic": None, "launches": n, "avg_us": 1e3 * ms / n,
                    "share_of_step": ms / (1e3 * dt_timed)}
        a = work / (ms * 1e-3) / 1e9
        return {"kernel": name, "bound": "hbm", "achieved": a, "peak": PEAK["hbm"], "unit": "GB/s",
                "frac": a / PEAK["hbm"], "traffic": None, "launches": n, "avg_us": 1e3 * ms / n,
                "share_of_step": ms / (1e3 * dt_timed)}

    lines = [l for l in (line(k) for k in M.KERNEL_CLASSES) if l]
    roofline = dict(max((l for l in lines if l["bound"] == "mfma"), key=lambda l: l["share_of_step"]))
    roofline["traffic"] = PMC_TRAFFIC_BYTES.get((cfg["name"], roofline["kernel"]))
    st = stats.cpu().numpy()
    assert np.all(np.isfinite(st)) and np.all(st[:, 7] == 0), "non-finite loss"

    S = cfg["n_envs"] * cfg["n_agents"] * T
    out = {
        "metric": "env-agent steps/sec (rollout+PPO update) on 1 MI355X",
        "value": S * args.steps / dt, "unit": "env-agent steps/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": 1e3 * dt / args.steps, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if cfg["precision"] == 1 else "f32", "data": "synthetic",
        "config": {"workload": cfg["name"], "config_index": args.config, "n_envs": cfg["n_envs"],
                   "n_agents": cfg["n_agents"], "rollout_len": T, "epochs": E, "minibatches": Mb,
                   "env_agent_steps_per_step": S, "launch": "hip_graph_replay" if args.graph else "per_kernel",
                   "mlp_gemm_tflop_per_step": gemm_flops_per_step(cfg, W) / 1e12},
        "roofline": roofline,
        "roofline_all": lines,
    }
    out["mlp_gemm_tflops_end_to_end"] = out["config"]["mlp_gemm_tflop_per_step"] / (dt / args.steps)
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
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = run_cpu_baseline(args.config, cfg, W)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
