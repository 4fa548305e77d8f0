#!/usr/bin/env python3
"""Benchmark of the batched PCGRL environment step on one MI355X.

A "step" is one pcgrl_step over the whole batch: edit, metrics, reward, bookkeeping and the
observation of every level, one kernel launch.  Inputs (levels, pre-generated random actions) are
resident in HBM before the timed region starts.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--batch B]

The headline workload is the 64x64 maze at a batch of 8192 (the configuration the bandwidth
target is quoted on); the `configs` object of the same line carries every other workload, and the
16x16 binary problem at a batch of 262 144 (the point the steps-per-second target is read at).
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
# plain integer vector work: 256 compute units x 4 SIMDs, one wave64 instruction per 4 cycles
# each, 2.4 GHz  ->  wave-instructions per second the chip can issue
VALU_PEAK_GINST = 256 * 4 * 2.4 / 4.0
MIN_REP_MS = 5.0       # a timed repetition lasts at least this long (the graph is replayed)
MALL_BYTES = 256 << 20  # memory-side cache: an observation ring has to be well beyond it
ACTION_STREAM_BYTES = 32 << 20  # the pre-generated actions of a run stay below this


def state_bytes_per_env(cfg) -> int:
    """Bytes of one level's resident state that a step reads: the tile code as bit-planes (P planes
    of S rows of S bits, S = 16 / 32 / 64 covering the buffer), the 32-byte record, and its rows of
    the metric cache and the target ranges."""
    from paper_2408_12525_amd import workloads as wl
    side = max(cfg["max_h"], cfg["max_w"])
    S = 16 if side <= 16 else 32 if side <= 32 else 64
    P = {wl.BINARY: 1, wl.MAZE: 2, wl.DUNGEON: 3}[cfg["problem"]]
    M = wl.num_metrics(cfg["problem"])
    return P * S * (8 if S == 64 else 4) + 32 + 4 * M + 4 * M


def algorithmic_bytes_per_env_step(cfg) -> int:
    """What one step of one level must move, with the level kept as bit-planes: read the state
    (planes, record, metric cache, target ranges) and the action; write the observation, the reward
    and the done flag, the record, and - after a modifying edit - one row of each plane and the
    metric cache."""
    from paper_2408_12525_amd import workloads as wl
    M = wl.num_metrics(cfg["problem"])
    return wl.obs_bytes(cfg) + state_bytes_per_env(cfg) + 4 + 4 + 1 + 32 + 4 * M


def rollout_bytes_per_env_step(cfg) -> int:
    """A resident rollout moves per step only the action in and observation, reward, done out."""
    from paper_2408_12525_amd import workloads as wl
    return wl.obs_bytes(cfg) + 4 + 4 + 1


def profile_table(fname: str, tag: str):
    """Second column of the line of profiles/<fname> that starts with `tag` (figures taken with
    rocprofv3 and committed there), or None."""
    path = os.path.join(ROOT, "profiles", fname)
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


def cpu_model() -> str:
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(cfg, seed, aseed):
    """The CPU oracle as it stands on a bounded sample of the same workload: one core on 256
    levels x 200 steps, then the same sample per thread sharded over the host threads this process
    may use (environments are independent)."""
    import numpy as np
    from concurrent.futures import ThreadPoolExecutor
    import oracle
    from paper_2408_12525_amd import workloads as wl

    threads = max(1, min(16, len(os.sched_getaffinity(0))))
    per = 256
    steps = 200
    envs = min(cfg["batch"], per * threads)
    threads = max(1, min(threads, envs // per)) if envs >= per else 1
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

    t0 = time.perf_counter()
    shard(bounds[0])                       # one core: the first shard, all its steps
    one_dt = time.perf_counter() - t0
    one = (bounds[0][1] - bounds[0][0]) * steps / one_dt
    env.reset(seed, want_obs=False)        # fresh episode so that every shard does the same work
    t0 = time.perf_counter()
    with ThreadPoolExecutor(threads) as ex:
        list(ex.map(shard, bounds))
    dt = time.perf_counter() - t0
    return {
        "value": envs * steps / dt, "unit": "env-steps/s", "cores": threads, "kind": "oracle",
        "value_1core": one, "cpu_model": cpu_model(),
        "sample": f"{envs} envs x {steps} steps of the same workload from the same seed "
                  f"(observation written every step), {threads} threads; 1-core figure on "
                  f"{bounds[0][1] - bounds[0][0]} envs x {steps} steps ({one_dt:.1f} s)",
    }


class GpuRun:
    """One workload on the GPU: a context, its buffers, and the two timed legs."""

    def __init__(self, name, batch, args):
        import torch
        from paper_2408_12525_amd import binding, workloads as wl
        self.torch, self.wl = torch, wl
        cfg = wl.workload(name, batch=batch)
        cfg["regions_mode"] = wl.REGIONS_RECOUNT if args.regions == "recount" else wl.REGIONS_INCREMENTAL
        cfg["obs_store_mode"] = ["auto", "cached", "stream", "through"].index(args.obs_store)
        if args.max_changes is not None:
            cfg["max_changes"] = args.max_changes
        cfg["obs_pitch"] = -1 if args.obs_pitch == "lines" else 0
        cfg["split_step"] = ["auto", "off", "on"].index(args.split)
        cfg["levels_per_wave"] = args.levels_per_wave
        self.cfg, self.name, self.args = cfg, name, args
        self.B = cfg["batch"]
        self.tag = f"{name}_B{self.B}"
        self.dev = torch.device("cuda", 0)
        self.env = binding.Pcgrl(cfg, 0)
        self.obs_env_bytes = wl.obs_bytes(cfg)        # the observation itself
        self.obs_stride = self.env.obs_stride          # what one level takes in an obs buffer
        self.rew = torch.empty(self.B, dtype=torch.float32, device=self.dev)
        self.done = torch.empty(self.B, dtype=torch.uint8, device=self.dev)

    def close(self):
        self.env.close()

    def obs_ring(self, want_slots, cap_bytes=16 << 30):
        """[slots, B, ...] observation buffers: a slot per step, as a learner that keeps its rollout
        has, and more of them than the memory-side cache holds, so that every byte written has to
        reach HBM (a single buffer rewritten every step would stay in that cache)."""
        one = self.B * self.obs_stride
        slots = max(1, min(want_slots, cap_bytes // max(1, one)))
        return self.torch.empty((slots,) + tuple(self.env.obs_shape), dtype=self.torch.uint8, device=self.dev)

    def per_step(self, K, W, reps, seed=0, aseed=1):
        """K pcgrl_step launches, replayed from a HIP graph (each launch a kernel node with its own
        slice of the action stream and its own observation slot); a repetition replays the graph
        until it has lasted MIN_REP_MS.  Returns wall and HIP-event time per step."""
        torch, wl, env, args = self.torch, self.wl, self.env, self.args
        # The pre-generated action stream repeats after 1000 steps, or sooner where 1000 steps of it
        # would not stay in the memory-side cache: a policy in the loop hands over actions that a
        # kernel has just written, not ones that have to come from HBM behind the step's own writes
        # (measured on the 16x16 binary problem at a batch of 262 144: 92 against 109 us per step).
        n_act = max(1, min(K, 1000, max(16, ACTION_STREAM_BYTES // (4 * self.B))))
        n_warm = max(1, min(W, n_act))
        acts = torch.from_numpy(wl.random_actions(self.cfg, aseed, n_act)).to(self.dev)
        warm = torch.from_numpy(wl.random_actions(self.cfg, aseed + 1, n_warm)).to(self.dev)
        chunk = min(1000, K)   # kernel nodes of one graph
        while K % chunk:
            chunk -= 1
        one = self.B * self.obs_stride
        slots = 1 if args.obs_ring == "one" else max(1, min(chunk, -(-4 * MALL_BYTES // one)))
        ring = self.obs_ring(slots)
        slots = ring.shape[0]
        graph = None
        if args.launch == "graph":
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.stream(side):
                env.pcgrl_reset(seed, ring[0])
                with torch.cuda.graph(graph, stream=side):
                    for t in range(chunk):
                        env.pcgrl_step(acts[t % n_act], ring[t % slots], self.rew, self.done)
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()

        def run_once():
            if graph is not None:
                for _ in range(K // chunk):
                    graph.replay()
            else:
                for t in range(K):
                    env.pcgrl_step(acts[t % n_act], ring[t % slots], self.rew, self.done)

        times_ms, ev_ms, rounds = [], [], 1
        for rep in range(reps):
            env.pcgrl_reset(seed, ring[0])
            for t in range(W):
                env.pcgrl_step(warm[t % n_warm], ring[t % slots], self.rew, self.done)
            if rep == 0:               # how many rounds of K steps make a repetition long enough
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                run_once()
                torch.cuda.synchronize()
                est_ms = (time.perf_counter() - t0) * 1e3
                rounds = max(1, int(-(-MIN_REP_MS // max(est_ms, 1e-3))))
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            e0.record()                      # on the current stream, the one the steps run on
            for _ in range(rounds):
                run_once()
            e1.record()
            torch.cuda.synchronize()
            times_ms.append((time.perf_counter() - t0) * 1e3)
            ev_ms.append(e0.elapsed_time(e1))
        if os.environ.get("PCGRL_BENCH_VERBOSE"):
            print(f"[bench] {self.tag}: us/step per repetition {[round(t * 1e3 / (K * rounds), 2) for t in ev_ms]}, "
                  f"rounds {rounds}, slots {slots}", file=sys.stderr)
        order = sorted(range(reps), key=lambda i: times_ms[i])
        mid = order[len(order) // 2]
        n = K * rounds
        del ring
        return {"wall_ms_per_step": times_ms[mid] / n, "event_ms_per_step": ev_ms[mid] / n,
                "timed_steps": n, "obs_slots": slots}

    def rollout(self, K, T=100, seed=0, aseed=1):
        """The same steps through pcgrl_rollout: T steps per launch, the levels resident in registers
        in between; every step still writes its observation (a slot per step), reward and done."""
        torch, wl, env = self.torch, self.wl, self.env
        T = max(1, min(T, K))
        launches = max(1, K // T)
        racts = torch.from_numpy(wl.random_actions(self.cfg, aseed, T)).to(self.dev)
        robs = self.obs_ring(T)
        slots = robs.shape[0]
        rrew = torch.empty((T, self.B), dtype=torch.float32, device=self.dev)
        rdone = torch.empty((T, self.B), dtype=torch.uint8, device=self.dev)
        env.pcgrl_reset(seed, robs[0])
        env.pcgrl_rollout(racts, robs, rrew, rdone)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        env.pcgrl_rollout(racts, robs, rrew, rdone)
        torch.cuda.synchronize()
        est_ms = (time.perf_counter() - t0) * 1e3
        launches = max(launches, int(-(-MIN_REP_MS // max(est_ms, 1e-3))))
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
        ev_s = r0.elapsed_time(r1) * 1e-3
        del robs
        return {"wall_s_per_step": rwall / (T * launches), "event_s_per_step": ev_s / (T * launches),
                "steps_per_launch": T, "launches": launches, "obs_slots": slots}


def store_rates(torch, binding, region_bytes, total=6 << 30):
    """What the memory system takes as a pure write stream, from the library's store-only kernel
    over a buffer far beyond the caches: one sweep over the whole buffer, and one wavefront per
    contiguous region of what one level's observation takes in the layout the benchmark uses (the
    pattern of the observation stores): with non-temporal stores in workgroup order, as a step
    launch with a slot per step issues them, and the way a large rollout stores (the same for
    whole lines per level; ordinary stores with consecutive regions on one die for dense ones)."""
    dev = torch.device("cuda", 0)
    buf = torch.empty(total, dtype=torch.uint8, device=dev)
    out = {}
    region = max(16, (region_bytes + 15) // 16 * 16)
    lines = region % 128 == 0
    for key, rb, order, mode in (("linear_fill", 1 << 10, 1, 3),
                                 ("region_stores_step", region, 0, 2),
                                 ("region_stores_rollout", region, 0 if lines else 2, 2 if lines else 1)):
        n = total // rb
        binding.pcgrl_store_rate(buf, n, rb, mode, order)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        for _ in range(3):
            binding.pcgrl_store_rate(buf, n, rb, mode, order)
        b.record()
        torch.cuda.synchronize()
        out[key] = n * rb * 3 / (a.elapsed_time(b) * 1e-3) / 1e9
    out["region_bytes"] = region
    out["unit"] = "GB/s"
    out["bytes"] = total
    del buf
    return out


def summarise(run: GpuRun, step, roll):
    """Per-step and rollout figures of one workload with the roofline they are held against."""
    cfg, B = run.cfg, run.B
    abytes = algorithmic_bytes_per_env_step(cfg)
    launch_s = step["event_ms_per_step"] * 1e-3
    achieved = abytes * B / launch_s / 1e9
    traffic = profile_table("hbm_traffic.txt", run.tag)
    valu = profile_table("valu_per_launch.txt", run.tag)      # wave-level vector instructions per launch
    valu_frac = valu / launch_s / 1e9 / VALU_PEAK_GINST if valu else None
    hbm_frac = achieved / HBM_PEAK_GBS
    # which ceiling is nearer: the launch itself (an empty launch is 1.5 us), the vector ALUs, or HBM
    if launch_s < 6.0e-6 and hbm_frac < 0.05:
        bound = "launch"
    elif valu_frac is not None and valu_frac > max(hbm_frac, (traffic or 0) / launch_s / 1e9 / HBM_PEAK_GBS):
        bound = "alu"
    else:
        bound = "hbm"
    out = {
        "value": B / (step["wall_ms_per_step"] * 1e-3), "us_per_step": step["wall_ms_per_step"] * 1e3,
        "kernel_us_per_step": launch_s * 1e6, "bound": bound, "frac": hbm_frac,
        "achieved_GBs": achieved, "algorithmic_bytes_per_env_step": abytes,
        "obs_slots": step["obs_slots"], "timed_steps": step["timed_steps"],
    }
    if traffic:
        out["traffic"] = traffic
        out["frac_traffic"] = traffic / launch_s / 1e9 / HBM_PEAK_GBS
    if valu_frac is not None:
        out["valu_wave_insts_per_launch"] = valu
        out["valu_issue_frac"] = valu_frac
    if roll is not None:
        rbytes = rollout_bytes_per_env_step(cfg)
        rs = roll["event_s_per_step"]
        out["rollout"] = {
            "value": B / roll["wall_s_per_step"], "us_per_step": roll["wall_s_per_step"] * 1e6,
            "frac": rbytes * B / rs / 1e9 / HBM_PEAK_GBS, "achieved_GBs": rbytes * B / rs / 1e9,
            "algorithmic_bytes_per_env_step": rbytes, "steps_per_launch": roll["steps_per_launch"],
            "launches": roll["launches"], "obs_slots": roll["obs_slots"],
        }
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="maze64")
    ap.add_argument("--batch", type=int, default=None)
    ap.add_argument("--reps", type=int, default=3, help="timed repetitions; the median is reported")
    ap.add_argument("--regions", choices=["incremental", "recount"], default="incremental")
    ap.add_argument("--max-changes", type=int, default=None, metavar="N",
                    help="end an episode after N modifying edits as well (episodes then end, and "
                         "levels restart, at different steps; default: the workload's own setting)")
    ap.add_argument("--obs-store", choices=["auto", "cached", "stream", "through"], default="auto",
                    help="how observations are stored (default: the library's own rule)")
    ap.add_argument("--obs-ring", choices=["ring", "one"], default="ring",
                    help="per-step launches write a ring of observation buffers four times the "
                         "memory-side cache (default: every byte reaches HBM) or rewrite one buffer")
    ap.add_argument("--obs-pitch", choices=["dense", "lines"], default="lines",
                    help="observation layout: one level's observation directly after the other, or "
                         "every level's observation padded to whole 128-byte lines (obs_pitch; default)")
    ap.add_argument("--split", choices=["auto", "off", "on"], default="auto",
                    help="tuning: one wavefront per level group, or a metrics and an observation wavefront")
    ap.add_argument("--levels-per-wave", type=int, default=0, choices=[0, 1, 2, 4],
                    help="tuning: levels packed into one wavefront (0 = the library's rule)")
    ap.add_argument("--launch", choices=["graph", "eager"], default="graph",
                    help="replay a HIP graph of pcgrl_step launches (default) or call it from Python")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle leg")
    ap.add_argument("--no-rollout", action="store_true", help="skip the pcgrl_rollout leg")
    ap.add_argument("--no-table", action="store_true", help="skip the per-workload table and the store rates")
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

    torch.cuda.set_device(0)
    if args.copy_calibration:
        n = args.copy_calibration << 20
        src = torch.full((n,), 7, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(20):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes": n, "copies": 20}))
        return

    W = args.warmup
    head = GpuRun(args.workload, args.batch, args)
    cfg, B = head.cfg, head.B
    K = args.steps if args.steps is not None else cfg["max_steps"]
    step = head.per_step(K, W, args.reps)
    roll = None if args.no_rollout else head.rollout(max(K, 100))
    hs = summarise(head, step, roll)
    head.close()

    attain = None
    if not args.no_table:
        attain = store_rates(torch, binding, head.obs_stride)
    ms_per_step = step["wall_ms_per_step"]
    out = {
        "metric": "env-steps/sec (edit+metrics+reward+obs) at 1 GPU; % of HBM roofline",
        "value": hs["value"], "unit": "env-steps/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "u8", "data": "synthetic",
        "config": {"workload": head.tag, "problem": ["binary", "maze", "dungeon"][cfg["problem"]],
                   "batch": B, "map": f"{cfg['max_h']}x{cfg['max_w']}",
                   "min_map": f"{cfg['min_h']}x{cfg['min_w']}", "obs_w": cfg["obs_w"],
                   "obs_bytes_per_env": head.obs_env_bytes, "obs_pitch_bytes": head.obs_stride,
                   "n_frozen": cfg["n_frozen"],
                   "regions": args.regions, "max_changes": cfg.get("max_changes", 0),
                   "obs_store": args.obs_store, "launch": args.launch, "launches_per_step": 1,
                   "reps": args.reps, "timed_steps_per_rep": step["timed_steps"],
                   "obs_slots": step["obs_slots"],
                   "algorithmic_bytes_per_env_step": hs["algorithmic_bytes_per_env_step"]},
        "roofline": {"bound": hs["bound"], "achieved": hs["achieved_GBs"], "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": hs["frac"], "traffic": hs.get("traffic"),
                     "frac_traffic": hs.get("frac_traffic"), "kernel": "step_kernel",
                     "avg_launch_us": hs["kernel_us_per_step"]},
    }
    if attain:
        out["roofline"]["attainable"] = attain
        out["roofline"]["frac_attainable"] = hs["achieved_GBs"] / attain["region_stores_step"]
    if "valu_issue_frac" in hs:
        out["roofline"]["valu_issue_frac"] = hs["valu_issue_frac"]
    if "rollout" in hs:
        r = hs["rollout"]
        out["rollout"] = dict(r, unit="env-steps/s",
                              roofline={"bound": "hbm", "achieved": r["achieved_GBs"], "peak": HBM_PEAK_GBS,
                                        "unit": "GB/s", "frac": r["frac"],
                                        "kernel": "rollout_kernel"})
        if attain:
            out["rollout"]["roofline"]["frac_attainable"] = r["achieved_GBs"] / attain["region_stores_rollout"]

    # every other workload, shorter (300 steps per repetition, one repetition of >= 5 ms), and the
    # 16x16 binary problem at the batch the steps-per-second target is read at
    if not args.no_table:
        table = {head.tag: {k: v for k, v in hs.items()}}
        todo = [(n, None) for n in wl.WORKLOADS] + [("binary16", 262144)]
        for name, batch in todo:
            run = GpuRun(name, batch, args)
            if run.tag in table:
                run.close()
                continue
            Kt = min(300, run.cfg["max_steps"])
            s = run.per_step(Kt, W, 1)
            r = None if args.no_rollout else run.rollout(Kt)
            table[run.tag] = summarise(run, s, r)
            run.close()
        out["configs"] = table
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(cfg, 0, 1)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
