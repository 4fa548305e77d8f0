#!/usr/bin/env python3
"""Benchmark of the batched PCGRL environment step on one MI355X.

A "step" is one pcgrl_step over the whole batch: edit, metrics, reward, bookkeeping and the
observation of every level, one kernel launch.  Inputs (levels, pre-generated random actions) are
resident in HBM before the timed region starts.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--batch B]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth


def algorithmic_bytes_per_env_step(cfg) -> int:
    """What one step of one level must move: write the observation, reward and done flag, read the
    action and the level once (canonical int8 grid), write back one cell, the metric cache and the
    counters."""
    from paper_2408_12525_amd import workloads as wl
    M = wl.num_metrics(cfg["problem"])
    return wl.obs_bytes(cfg) + cfg["max_h"] * cfg["max_w"] + 4 + 4 + 1 + 1 + 4 * M + 16


def traffic_from_profiles(tag: str):
    """HBM bytes per launch measured with rocprofv3 counters, if a summary was committed."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        parts = line.split()
        if len(parts) >= 2 and parts[0] == tag:
            try:
                return float(parts[1])
            except ValueError:
                return None
    return None


def cpu_baseline(cfg, seed, aseed, budget_s=12.0):
    """The CPU oracle as it stands, on a bounded sample of the same workload, sharded over the
    host threads this process may use (environments are independent)."""
    import numpy as np
    from concurrent.futures import ThreadPoolExecutor
    import oracle
    from paper_2408_12525_amd import workloads as wl

    threads = max(1, min(16, len(os.sched_getaffinity(0))))
    envs = min(cfg["batch"], 32 * threads)
    steps = 100
    scfg = dict(cfg, batch=envs)
    env = oracle.Oracle(scfg)
    env.reset(seed, want_obs=False)
    acts = wl.random_actions(scfg, aseed, steps)
    obs = env.new_obs()
    rew = np.zeros(envs, np.float32)
    done = np.zeros(envs, np.uint8)
    bounds = [(i * envs // threads, (i + 1) * envs // threads) for i in range(threads)]

    def shard(lo_hi):
        lo, hi = lo_hi
        for t in range(steps):
            env.step_range(lo, hi, acts[t], obs, rew, done)

    # one core
    t0 = time.perf_counter()
    n1 = 0
    lo, hi = bounds[0]
    for t in range(steps):
        env.step_range(lo, hi, acts[t], obs, rew, done)
        n1 += hi - lo
        if time.perf_counter() - t0 > budget_s / 3:
            break
    one = n1 / (time.perf_counter() - t0)
    # all threads (fresh episode so that every shard does the same work)
    env.reset(seed, want_obs=False)
    t0 = time.perf_counter()
    with ThreadPoolExecutor(threads) as ex:
        list(ex.map(shard, bounds))
    dt = time.perf_counter() - t0
    return {
        "value": envs * steps / dt, "unit": "env-steps/s", "cores": threads, "kind": "oracle",
        "value_1core": one,
        "sample": f"{envs} envs x {steps} steps of the same workload from the same seed "
                  f"(observation written every step), {threads} threads; 1-core figure on "
                  f"{hi - lo} envs",
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="maze16")
    ap.add_argument("--batch", type=int, default=None)
    ap.add_argument("--reps", type=int, default=3, help="timed repetitions of the K steps; the median is reported")
    ap.add_argument("--regions", choices=["incremental", "recount"], default="incremental")
    ap.add_argument("--max-changes", type=int, default=None, metavar="N",
                    help="end an episode after N modifying edits as well (episodes then end, and "
                         "levels restart, at different steps; default: the workload's own setting)")
    ap.add_argument("--obs-store", choices=["auto", "cached", "stream", "through"], default="auto",
                    help="how observations are stored (default: the library's own rule)")
    ap.add_argument("--launch", choices=["graph", "eager"], default="graph",
                    help="replay a HIP graph of pcgrl_step launches (default) or call it from Python")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle leg")
    ap.add_argument("--no-rollout", action="store_true", help="skip the pcgrl_rollout leg")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MIB",
                    help="instead of the benchmark, run 20 plain device copies of MIB MiB (the known "
                         "traffic that scales rocprofv3's FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only; environments are independent, so more "
              "GPUs would each run this same kernel on their own share of the batch (run with --gpus 1)",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2408_12525_amd import binding, workloads as wl

    if args.copy_calibration:
        n = args.copy_calibration << 20
        src = torch.full((n,), 7, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(20):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes": n, "copies": 20}))
        return

    cfg = wl.workload(args.workload, batch=args.batch)
    cfg["regions_mode"] = wl.REGIONS_RECOUNT if args.regions == "recount" else wl.REGIONS_INCREMENTAL
    cfg["obs_store_mode"] = ["auto", "cached", "stream", "through"].index(args.obs_store)
    if args.max_changes is not None:
        cfg["max_changes"] = args.max_changes
    K = args.steps if args.steps is not None else cfg["max_steps"]
    W = args.warmup
    B = cfg["batch"]
    dev = torch.device("cuda", 0)
    torch.cuda.set_device(dev)

    env = binding.Pcgrl(cfg, 0)
    obs = env.new_obs()
    rew = torch.empty(B, dtype=torch.float32, device=dev)
    done = torch.empty(B, dtype=torch.uint8, device=dev)
    seed, aseed = 0, 1
    n_act = min(K, 1000)   # the action stream repeats after 1000 steps (keeps it small in HBM)
    acts = torch.from_numpy(wl.random_actions(cfg, aseed, n_act)).to(dev)
    warm = torch.from_numpy(wl.random_actions(cfg, aseed + 1, max(W, 1))).to(dev)

    # One HIP graph holds `chunk` consecutive pcgrl_step launches (each a kernel node with its own
    # slice of the action stream); replaying it is how a launch-bound loop is meant to be driven
    # on this hardware.  --launch eager calls pcgrl_step from Python instead (about 9 us of host
    # time per call, which then bounds small batches).
    chunk = min(n_act, K)
    while K % chunk:
        chunk -= 1
    graph = None
    if args.launch == "graph":
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            env.pcgrl_reset(seed, obs)
            with torch.cuda.graph(graph, stream=side):
                for t in range(chunk):
                    env.pcgrl_step(acts[t], obs, rew, done)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()

    times_ms, ev_ms = [], []
    for rep in range(args.reps):
        env.pcgrl_reset(seed, obs)
        for t in range(W):
            env.pcgrl_step(warm[t], obs, rew, done)
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        e0.record()                      # on the current stream, the one the steps run on
        if graph is not None:
            for _ in range(K // chunk):
                graph.replay()
        else:
            for t in range(K):
                env.pcgrl_step(acts[t % n_act], obs, rew, done)
        e1.record()
        torch.cuda.synchronize()
        times_ms.append((time.perf_counter() - t0) * 1e3)
        ev_ms.append(e0.elapsed_time(e1))
    order = sorted(range(args.reps), key=lambda i: times_ms[i])
    mid = order[len(order) // 2]
    wall_ms, kern_ms = times_ms[mid], ev_ms[mid]
    ms_per_step = wall_ms / K
    value = B * K / (wall_ms * 1e-3)

    abytes = algorithmic_bytes_per_env_step(cfg)
    per_launch = abytes * B
    launch_s = kern_ms * 1e-3 / K        # average launch-to-launch time on the stream (HIP events)
    achieved = per_launch / launch_s / 1e9
    tag = f"{args.workload}_B{B}"
    out = {
        "metric": "env-steps/sec (edit+metrics+reward+obs) at 1 GPU; % of HBM roofline",
        "value": value, "unit": "env-steps/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "u8", "data": "synthetic",
        "config": {"workload": tag, "problem": ["binary", "maze", "dungeon"][cfg["problem"]],
                   "batch": B, "map": f"{cfg['max_h']}x{cfg['max_w']}",
                   "min_map": f"{cfg['min_h']}x{cfg['min_w']}", "obs_w": cfg["obs_w"],
                   "obs_bytes_per_env": wl.obs_bytes(cfg), "n_frozen": cfg["n_frozen"],
                   "regions": args.regions, "max_changes": cfg.get("max_changes", 0), "obs_store": args.obs_store, "launch": args.launch, "launches_per_step": 1, "reps": args.reps,
                   "algorithmic_bytes_per_env_step": abytes},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic_from_profiles(tag),
                     "kernel": "step_kernel", "avg_launch_us": launch_s * 1e6},
    }
    # The same K steps driven through pcgrl_rollout: T steps per launch, levels resident in
    # registers in between, every step still writes its observation, reward and done flag.  The
    # observations go into a slot per step (what a learner that keeps the whole rollout needs;
    # fewer slots only where T of them would exceed 16 GiB), so that every byte written has to
    # reach HBM: one slot rewritten T times would largely be absorbed by the caches.  Reported
    # beside the headline, never instead of it.
    if not args.no_rollout:
        T = min(chunk, 100)
        launches = max(1, K // T)
        racts = acts[:T].contiguous()
        slots = max(1, min(T, (16 << 30) // max(1, obs.numel())))
        robs = torch.empty((slots,) + tuple(obs.shape), dtype=torch.uint8, device=dev)
        rrew = torch.empty((T, B), dtype=torch.float32, device=dev)
        rdone = torch.empty((T, B), dtype=torch.uint8, device=dev)
        env.pcgrl_reset(seed, obs)
        env.pcgrl_rollout(racts, robs, rrew, rdone)
        r0 = torch.cuda.Event(enable_timing=True)
        r1 = torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        r0.record()
        for _ in range(launches):
            env.pcgrl_rollout(racts, robs, rrew, rdone)
        r1.record()
        torch.cuda.synchronize()
        rwall = time.perf_counter() - t0
        rbytes = wl.obs_bytes(cfg) + 4 + 4 + 1          # per env-step: obs + action + reward + done
        rlaunch_s = r0.elapsed_time(r1) * 1e-3 / launches
        out["rollout"] = {
            "value": B * T * launches / rwall, "unit": "env-steps/s", "steps_per_launch": T,
            "launches": launches, "obs_slots": slots, "us_per_step": rwall / (T * launches) * 1e6,
            "algorithmic_bytes_per_env_step": rbytes,
            "roofline": {"bound": "hbm", "achieved": rbytes * B * T / rlaunch_s / 1e9,
                         "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": rbytes * B * T / rlaunch_s / 1e9 / HBM_PEAK_GBS,
                         "kernel": "step_kernel<..., rollout>", "avg_launch_us": rlaunch_s * 1e6},
        }
    env.close()
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(cfg, seed, aseed)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
