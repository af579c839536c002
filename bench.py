#!/usr/bin/env python3
"""Benchmark of the Craftax hot path on one MI355X.

A "step" is one craftax_step call over all environments of the workload: rules, mob update,
auto-reset of finished episodes and the symbolic observation write, with every input already
resident in HBM.  Prints ONE JSON line: metric / value / unit (environment steps per second),
ms_per_step, config.workload, "roofline" (algorithmic bytes per launch over the launch time measured
with HIP events on the library's stream, against the 8 TB/s HBM peak; "traffic" = HBM bytes per
launch from the rocprofv3 counter runs summarised under profiles/) and "cpu_baseline" (the CPU
oracle timed on a bounded sample of the same workload).  The headline
workload is the 65,536-environment Craftax-Classic step; the 4,096-environment Classic step and
the 4,096-environment full-Craftax step are measured next to it ("also", "also_craftax"), or
alone with --workload craftax.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--envs N] [--workload classic|craftax|craftax_pixels|rollout] [--no-cpu-baseline]
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published peak
# The paper's own speed figures (its table of steps per second): whole PPO training runs, networks and
# updates included, on another machine.  Context for a reader, not a baseline for vs_baseline.
PAPER_CONTEXT = {
    "note": "steps/s of complete PPO training runs (environment + learner), 1x RTX 4090, 4,096 workers; context only",
    "craftax_classic_symbolic_ppo_sps": 405618,
    "craftax_symbolic_ppo_sps": 266961,
}
OBS_ALG_BYTES = 1323 + 22 * 4  # uint8 cells + fp32 scalars actually produced per env-step


def algorithmic_bytes_per_env_step(mean_episode_len: float) -> dict:
    """What the method itself has to move per environment step (not what cache lines carry)."""
    parts = {
        "obs_write": OBS_ALG_BYTES,
        "action_reward_done": 4 + 4 + 1,
        "record_rw": 128 + 128,               # packed record (player 40 B, 12 mob words, 10 plant words), read + write
        "map_reads": 63 + 9 + 12 + 3 + 10,    # view, 3x3 neighbourhood, mob targets, spawn probes, plant cells
        "map_writes": 2,
        "reset_amortised": (4096 + 128 + 16) / max(mean_episode_len, 1.0),   # new map + record + done-list entry
    }
    parts["total"] = float(sum(parts.values()))
    return parts


FULL_OBS_ALG_BYTES = 99 * 83 + 51 * 4   # uint8 cells + fp32 scalars of the full game


def full_algorithmic_bytes_per_env_step(mean_episode_len: float) -> dict:
    parts = {
        "obs_write": FULL_OBS_ALG_BYTES,
        "action_reward_done": 4 + 4 + 1,
        "record_rw": 256 + 256,               # packed record incl. ladders and plants, read + write
        "mob_table_rw": 56 + 56,              # 14 slots of the current floor
        "map_reads": 2 * 99 + 14 + 3 + 10,    # view in both maps, mob targets, spawn probes, plant cells
        "map_writes": 2,
        "reset_amortised": (9 * 2 * 2304 + 1024 + 16) / max(mean_episode_len, 1.0),
    }
    parts["total"] = float(sum(parts.values()))
    return parts


def read_profile_traffic(name: str):
    """HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE + WRITE_SIZE), taken from
    the committed summary; None if that summary is absent."""
    path = os.path.join(ROOT, "profiles", name)
    if not os.path.exists(path):
        return None
    m = re.search(r"^traffic_bytes_per_launch:\s*([0-9.eE+]+)", open(path).read(), flags=re.M)
    return float(m.group(1)) if m else None


SPIN_UP_STEPS = 2000       # untimed steps before any timed region: episodes last ~180 steps, so every
                           # environment has been through several and the batch is in its steady state
LENGTH_WINDOW = 1000       # the last steps of the spin-up, over which the mean episode length is taken


def episode_sum(sim) -> int:
    """Episodes finished since the reset, summed over all environments (craftax_stats)."""
    return int(sim.stats()["episodes"])


def advance(cx, sim, kind_id: int, first_step: int, steps: int, use_rollout: bool) -> int:
    """Untimed: `steps` steps of the workload's own action stream without rendering, through
    craftax_rollout where the configuration allows it (faster), else step by step."""
    import torch

    n, chunk = sim.n, 250
    actions = torch.empty((chunk, n), dtype=torch.int32, device=sim.device)
    reward = torch.empty((chunk, n), dtype=torch.float32, device=sim.device)
    done = torch.empty((chunk, n), dtype=torch.uint8, device=sim.device)
    for s0 in range(first_step, first_step + steps, chunk):
        k = min(chunk, first_step + steps - s0)
        cx.craftax_synth_actions(actions, n, s0, k, 0, kind_id, sim.stream)
        if use_rollout:
            cx.craftax_rollout(sim.state, actions, k, None, reward, done, n, sim.stream)
        else:
            for j in range(k):
                cx.craftax_step(sim.state, actions[j], None, reward[j], done[j], n, sim.stream)
    torch.cuda.synchronize()
    return first_step + steps


def spin_up(cx, sim, kind_id: int, use_rollout: bool):
    """Brings a freshly reset batch to its steady state (outside every timed region) and measures
    the mean episode length over a fixed window.  Returns (next action step, mean episode length)."""
    s = advance(cx, sim, kind_id, 0, SPIN_UP_STEPS - LENGTH_WINDOW, use_rollout)
    before = episode_sum(sim)
    s = advance(cx, sim, kind_id, s, LENGTH_WINDOW, use_rollout)
    finished = episode_sum(sim) - before
    return s, sim.n * LENGTH_WINDOW / max(finished, 1)


def gpu_run(n: int, steps: int, warmup: int, kind: str, repeats: int = 3, variant: str = "classic", pixels: bool = False,
            pool_resets: bool = False):
    import torch
    from paper_2402_16801_amd import binding as cx, synth

    dev = torch.device("cuda:0")
    if variant == "craftax":
        cfg = cx.default_config(cx.VARIANT_CRAFTAX, obs_mode=cx.OBS_PIXELS_F32 if pixels else cx.OBS_SYM_U8_F32)
    else:
        cfg = cx.default_config(obs_mode=cx.OBS_SYM_U8_F32, max_episode_steps=10000,
                                reset_mode=cx.RESET_POOL if pool_resets else cx.RESET_EXACT)
    sim = cx.Craftax(n, cfg)
    sim.reset(synth.seeds_for(n))
    kind_id = {"uniform": 0, "skewed": 1}[kind] + (2 if variant == "craftax" else 0)
    step0, mean_len = spin_up(cx, sim, kind_id, use_rollout=not (pixels or pool_resets))
    total_steps = warmup + repeats * steps
    actions = torch.empty((total_steps, n), dtype=torch.int32, device=dev)
    cx.craftax_synth_actions(actions, n, step0, total_steps, 0, kind_id, sim.stream)
    torch.cuda.synchronize()

    # the launches go to torch's current stream, so torch events bracket exactly that stream
    state, obs, rew, done, stream = sim.state, sim.obs, sim.reward, sim.done, sim.stream
    s = 0
    for _ in range(warmup):
        cx.craftax_step(state, actions[s], obs, rew, done, n, stream)
        s += 1
    torch.cuda.synchronize()
    wall, evt = [], []
    for _ in range(repeats):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        e0.record(stream)
        for _ in range(steps):
            cx.craftax_step(state, actions[s], obs, rew, done, n, stream)
            s += 1
        e1.record(stream)
        torch.cuda.synchronize()
        wall.append(time.perf_counter() - t0)
        evt.append(e0.elapsed_time(e1) * 1e-3)
    draw_s = None
    if pixels:      # the drawing kernel alone: craftax_observe launches just that kernel
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for _ in range(5):
            cx.craftax_observe(state, obs, n, stream)
        e0.record(stream)
        for _ in range(steps):
            cx.craftax_observe(state, obs, n, stream)
        e1.record(stream)
        torch.cuda.synchronize()
        draw_s = e0.elapsed_time(e1) * 1e-3 / steps
    sim.close()
    med = int(np.argsort(wall)[len(wall) // 2])
    return {"wall_s": wall[med], "event_s": evt[med], "all_wall_s": wall, "mean_episode_len": mean_len, "draw_s": draw_s}


def rollout_run(n: int, steps: int, warmup: int, kind: str, repeats: int = 3, variant: str = "classic"):
    """craftax_rollout: the same steps, actions and outputs as `steps` craftax_step calls, in one launch."""
    import torch
    from paper_2402_16801_amd import binding as cx, synth

    if variant == "classic":
        cfg = cx.default_config(obs_mode=cx.OBS_SYM_U8_F32, max_episode_steps=10000)
        kind_id = {"uniform": 0, "skewed": 1}[kind]
    else:
        cfg = cx.default_config(cx.VARIANT_CRAFTAX, obs_mode=cx.OBS_SYM_U8_F32)
        kind_id = {"uniform": 2, "skewed": 3}[kind]
    sim = cx.Craftax(n, cfg)
    sim.reset(synth.seeds_for(n))
    step0, _ = spin_up(cx, sim, kind_id, use_rollout=True)
    total = max(warmup, 1) + repeats * steps
    warmup = max(warmup, 1)
    actions = torch.empty((total, n), dtype=torch.int32, device=sim.device)
    cx.craftax_synth_actions(actions, n, step0, total, 0, kind_id, sim.stream)
    reward = torch.zeros((max(steps, warmup), n), dtype=torch.float32, device=sim.device)
    done = torch.zeros((max(steps, warmup), n), dtype=torch.uint8, device=sim.device)
    cx.craftax_rollout(sim.state, actions[:warmup], warmup, sim.obs, reward[:warmup], done[:warmup], n, sim.stream)
    torch.cuda.synchronize()
    wall = []
    for r in range(repeats):
        a = actions[warmup + r * steps: warmup + (r + 1) * steps]
        t0 = time.perf_counter()
        cx.craftax_rollout(sim.state, a, steps, sim.obs, reward, done, n, sim.stream)
        torch.cuda.synchronize()
        wall.append(time.perf_counter() - t0)
    sim.close()
    return sorted(wall)[len(wall) // 2]


def copy_ceiling_gbs(mib: int = 1024, repeats: int = 10) -> float:
    """Measured device-to-device copy rate (bytes read + bytes written per second), as context
    for the nominal peak: a buffer larger than the last-level cache, copied `repeats` times."""
    import torch

    src = torch.empty(mib << 20, dtype=torch.uint8, device="cuda:0").fill_(1)
    dst = torch.empty_like(src)
    dst.copy_(src)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(repeats):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    return 2.0 * (mib << 20) * repeats / (e0.elapsed_time(e1) * 1e-3) / 1e9


CPU_SAMPLE_ENVS, CPU_SAMPLE_STEPS = 8192, 1000         # one core: about 10 s of oracle work
CPU_ALL_ENVS, CPU_ALL_STEPS = 65536, 300               # all cores: the whole population of the headline workload


def cpu_baseline(kind: str, variant: str = "classic", pixels: bool = False, n_sample: int | None = None, steps: int | None = None):
    """The CPU oracle, as it stands, on a bounded sample of the same workload (its size does not
    depend on --steps): the first environments, from their reset on, on one core; and the same
    oracle over more environments on all host cores (slices of environments on threads: the
    environments are independent).  The resets are not timed."""
    from oracle import pyoracle as po
    from paper_2402_16801_amd import synth

    def make(n):
        if variant == "craftax":
            return po.FullOracle(n, po.full_default_config(), po.FULL_OBS_PIXELS_F32 if pixels else po.FULL_OBS_U8_F32)
        return po.Oracle(n, po.default_config(max_episode_steps=10000), po.OBS_SYM_U8_F32)

    n_actions = 43 if variant == "craftax" else 17
    what = "pixel" if pixels else "symbolic"
    if n_sample is None:
        n_sample, steps = (CPU_SAMPLE_ENVS, CPU_SAMPLE_STEPS) if variant == "classic" else (1024, 1000)
    orc = make(n_sample)
    orc.reset_many(synth.seeds_for(n_sample))
    t0, done_steps = time.perf_counter(), 0
    for s in range(steps):
        orc.step(synth.actions(np.arange(n_sample), s, kind, 0, n_actions))
        done_steps += 1
        if time.perf_counter() - t0 > 20.0:
            break
    dt = time.perf_counter() - t0
    one = {"value": n_sample * done_steps / dt, "unit": "env_steps/s", "cores": 1, "kind": "oracle",
           "sample": f"first {n_sample} envs x {done_steps} steps of the same workload from the reset on, single thread, "
                     f"including the {what} observation of every step and the action draws ({dt:.1f} s)"}
    if pixels:
        return one, None
    threads = po._host_threads()
    n_all, k_all = (CPU_ALL_ENVS, CPU_ALL_STEPS) if variant == "classic" else (4096, 1000)
    orc = make(n_all)
    orc.reset_many(synth.seeds_for(n_all))
    chunk, done_steps, dt = 50, 0, 0.0
    for s0 in range(0, k_all, chunk):
        acts = synth.action_block(n_all, chunk, kind, 0, s0, n_actions)
        t0 = time.perf_counter()
        # every step renders nothing but the last of a chunk: the rules are timed, as in the parity runs
        orc.step_many(acts, threads=threads)
        dt += time.perf_counter() - t0
        done_steps += chunk
        if dt > 20.0:
            break
    allc = {"value": n_all * done_steps / dt, "unit": "env_steps/s", "cores": threads, "kind": "oracle",
            "sample": f"all {n_all} envs x {done_steps} steps of the same workload from the reset on, {threads} threads over slices "
                      f"of environments, rules and auto-resets of every step, observation once per {chunk} steps ({dt:.1f} s)"}
    return one, allc


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="classic", choices=["classic", "craftax", "craftax_pixels", "rollout"])
    ap.add_argument("--envs", type=int, default=None, help="default 65536 (classic) or 4096 (craftax)")
    ap.add_argument("--kind", default=None, choices=["uniform", "skewed"], help="default skewed (classic) or uniform (craftax)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-small", action="store_true", help="skip the secondary 4096-env measurement")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="first run one plain elementwise kernel that reads and writes 256 MiB (reference for "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; environments are independent and would shard "
              "without communication, but no multi-GPU path is built or measured (--gpus must be 1).",
              file=sys.stderr)
        sys.exit(2)

    if args.calibrate_copy:
        import torch
        # one elementwise kernel that reads 256 MiB and writes 256 MiB
        src = torch.full((64 << 20,), 7, dtype=torch.int32, device="cuda:0")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        torch.add(src, 1, out=dst)
        torch.cuda.synchronize()
        del src, dst

    if args.workload == "craftax":
        print(json.dumps(craftax_line(args)))
        return
    if args.workload == "craftax_pixels":
        print(json.dumps(craftax_pixels_line(args)))
        return
    if args.workload == "rollout":
        print(json.dumps(rollout_line(args)))
        return
    args.envs = 65536 if args.envs is None else args.envs
    args.kind = "skewed" if args.kind is None else args.kind
    n, K, W = args.envs, args.steps, args.warmup
    main_run = gpu_run(n, K, W, args.kind)
    alg = algorithmic_bytes_per_env_step(main_run["mean_episode_len"])
    per_launch_bytes = alg["total"] * n
    launch_s = main_run["event_s"] / K             # average per-launch time from HIP events
    achieved = per_launch_bytes / launch_s / 1e9
    value = n * K / main_run["wall_s"]

    out = {
        "metric": "env steps/sec at 1 GPU (4096 / 65536 envs, symbolic obs) + % HBM roofline",
        "value": value,
        "unit": "env_steps/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": W,
        "ms_per_step": main_run["wall_s"] / K * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u8",
        "data": "synthetic",
        "config": {
            "workload": f"configs[2]: Craftax-Classic symbolic step, {n} envs, 64x64 map, fixed-seed action stream "
                        f"skewed 50% toward move/do, episode cap 10000, auto-reset regenerating terrain, "
                        f"obs uint8[1323]+fp32[22]",
            "envs": n, "obs_mode": "SYM_U8_F32", "actions": args.kind,
            "mean_episode_len": round(main_run["mean_episode_len"], 1),
            "spin_up_steps": SPIN_UP_STEPS, "episode_length_window": LENGTH_WINDOW,
        },
        "roofline": {
            "bound": "hbm",
            "achieved": achieved,
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS,
            "traffic": read_profile_traffic("craftax_step_sym_u8_f32_65536env.txt"),
            "kernel": "k_step<4 lanes, SYM_U8_F32>: step blocks + regeneration blocks, one launch per craftax_step call",
            "alg_bytes_per_env_step": round(alg["total"], 1),
            "alg_bytes_per_launch": per_launch_bytes,
            "avg_launch_us": launch_s * 1e6,
            "measured_copy_gbs": copy_ceiling_gbs(),
        },
    }
    if not args.no_small:
        small = gpu_run(4096, K, W, "uniform")
        out["also"] = {"workload": "configs[1]: 4096 envs, uniform actions", "value": 4096 * K / small["wall_s"],
                       "unit": "env_steps/s", "ms_per_step": small["wall_s"] / K * 1e3}
        small_roll = rollout_run(4096, K, W, "uniform")
        out["also"]["rollout_value"] = 4096 * K / small_roll
        out["also"]["rollout_ms_per_step"] = small_roll / K * 1e3
        roll = rollout_run(n, K, W, args.kind)
        out["also_rollout"] = {"workload": f"the same {n} environments and action stream through craftax_rollout: {K} steps per launch, "
                                           "observation written after every step, reward and done of every step kept",
                               "value": n * K / roll, "unit": "env_steps/s", "ms_per_step": roll / K * 1e3,
                               # the records stay on chip between the steps of a launch: 256 bytes less per env-step
                               "roofline_frac": (alg["total"] - 256.0) * n / (roll / K) / 1e9 / HBM_PEAK_GBS}
        pool = gpu_run(n, K, W, args.kind, repeats=1, pool_resets=True)
        out["also_pool_resets"] = {"workload": f"the same {n} environments and action stream with reset_mode POOL (the paper's optimistic "
                                               "resets: finished environments draw their worlds from a pool of n/16 per step)",
                                   "value": n * K / pool["wall_s"], "unit": "env_steps/s", "ms_per_step": pool["wall_s"] / K * 1e3}
        full = craftax_line(args, with_cpu=False)
        out["also_craftax"] = {"workload": full["config"]["workload"], "value": full["value"], "unit": "env_steps/s",
                               "ms_per_step": full["ms_per_step"], "roofline": full["roofline"],
                               "rollout_value": full["also"]["rollout_value"],
                               "rollout_ms_per_step": full["also"]["rollout_ms_per_step"]}
    if not args.no_cpu_baseline:
        out["cpu_baseline"], out["cpu_baseline_all_cores"] = cpu_baseline(args.kind)
    out["paper_context"] = PAPER_CONTEXT
    print(json.dumps(out))


def rollout_line(args) -> dict:
    """The headline workload through craftax_rollout: all K steps of a repeat in one launch."""
    n = 65536 if args.envs is None else args.envs
    kind = "skewed" if args.kind is None else args.kind
    K, W = args.steps, args.warmup
    wall = rollout_run(n, K, W, kind)
    alg = algorithmic_bytes_per_env_step(180.0)["total"] - 256.0     # the record stays on chip between the steps of a launch (episodes last ~180 steps)
    achieved = alg * n / (wall / K) / 1e9
    return {
        "metric": "env steps/sec at 1 GPU (65536 envs, symbolic obs, K steps per launch) + % HBM roofline",
        "value": n * K / wall, "unit": "env_steps/s", "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": wall / K * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u8", "data": "synthetic",
        "config": {"workload": f"Craftax-Classic symbolic steps through craftax_rollout, {n} envs, {K} steps per launch, {kind} "
                               f"actions, observation written after every step, reward and done of every step kept",
                   "envs": n, "obs_mode": "SYM_U8_F32", "actions": kind},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": read_profile_traffic("craftax_rollout_sym_u8_f32_65536env.txt"),
                     "kernel": "k_rollout<SYM_U8_F32>: one launch of 1024 blocks for all K steps",
                     "alg_bytes_per_env_step": round(alg, 1), "alg_bytes_per_launch": alg * n * K, "avg_launch_us": wall * 1e6},
    }


PIXEL_BYTES_PER_ENV = 130 * 110 * 3 * 4 + 1024 + 2 * 99      # the picture + the record and mob table + the 99 view cells of two maps


def craftax_pixels_line(args) -> dict:
    """Full Craftax with the 110 x 130 x 3 pixel observation: step kernel + drawing kernel."""
    n = 4096 if args.envs is None else args.envs
    kind = "uniform" if args.kind is None else args.kind
    K, W = args.steps, args.warmup
    run = gpu_run(n, K, W, kind, variant="craftax", pixels=True)
    achieved = PIXEL_BYTES_PER_ENV * n / run["draw_s"] / 1e9
    return {
        "metric": "env steps/sec at 1 GPU (pixel obs) + % HBM roofline",
        "value": n * K / run["wall_s"], "unit": "env_steps/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": run["wall_s"] / K * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {
            "workload": f"full Craftax step with pixel observation, {n} envs, 43 actions {kind}, obs fp32[130][110][3] "
                        f"from a seeded 127-tile atlas",
            "envs": n, "obs_mode": "PIXELS_F32", "actions": kind, "mean_episode_len": round(run["mean_episode_len"], 1),
        },
        "roofline": {
            "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
            "traffic": read_profile_traffic("craftax_full_pixels_4096env.txt"),
            "kernel": "kf_pixels: one block per environment, launched after the step kernel",
            "alg_bytes_per_env_step": PIXEL_BYTES_PER_ENV, "alg_bytes_per_launch": PIXEL_BYTES_PER_ENV * n,
            "avg_launch_us": run["draw_s"] * 1e6,
            "measured_copy_gbs": copy_ceiling_gbs(),
        },
        **({} if args.no_cpu_baseline else {"cpu_baseline": cpu_baseline(kind, variant="craftax", pixels=True, n_sample=64, steps=40)[0]}),
    }


def craftax_line(args, with_cpu: bool = True) -> dict:
    """configs[3]: the full game, 4096 environments, 43 uniform actions."""
    n = 4096 if (args.envs is None or args.workload != "craftax") else args.envs
    kind = "uniform" if (args.kind is None or args.workload != "craftax") else args.kind
    K, W = args.steps, args.warmup
    run = gpu_run(n, K, W, kind, variant="craftax")
    alg = full_algorithmic_bytes_per_env_step(run["mean_episode_len"])
    launch_s = run["event_s"] / K
    achieved = alg["total"] * n / launch_s / 1e9
    out = {
        "metric": "env steps/sec at 1 GPU (4096 / 65536 envs, symbolic obs) + % HBM roofline",
        "value": n * K / run["wall_s"], "unit": "env_steps/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": run["wall_s"] / K * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u8", "data": "synthetic",
        "config": {
            "workload": f"configs[3]: full Craftax step, {n} envs, 9 floors x 48x48 block + item/light maps, 43 actions "
                        f"{kind}, per-floor mob tables 3/2/3/3/3, episode cap 100000, obs uint8[8217]+fp32[51]",
            "envs": n, "obs_mode": "SYM_U8_F32", "actions": kind, "mean_episode_len": round(run["mean_episode_len"], 1),
        },
        "roofline": {
            "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
            "traffic": read_profile_traffic("craftax_full_step_sym_u8_f32_4096env.txt"),
            "kernel": "kf_step<SYM_U8_F32>: step blocks + regeneration blocks, one launch per craftax_step call",
            "alg_bytes_per_env_step": round(alg["total"], 1), "alg_bytes_per_launch": alg["total"] * n,
            "avg_launch_us": launch_s * 1e6,
        },
    }
    roll = rollout_run(n, K, W, kind, variant="craftax")
    out["also"] = {"workload": f"the same {n} environments and action stream through craftax_rollout, {K} steps per launch",
                   "rollout_value": n * K / roll, "rollout_ms_per_step": roll / K * 1e3, "unit": "env_steps/s"}
    if with_cpu and not args.no_cpu_baseline:
        out["cpu_baseline"], out["cpu_baseline_all_cores"] = cpu_baseline(kind, variant="craftax")
    return out


if __name__ == "__main__":
    main()
