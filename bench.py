#!/usr/bin/env python3
"""Benchmark of the Tag roll-out hot path on one MI355X.

A "step" is one roll-out iteration of the whole batch: sample an action for every agent from
its policy probabilities, advance every environment by one Tag step, reset the environments
that finished (paper Sec. 4.5 items 3-6), all through libwd's C ABI, one wd_iterate launch per
iteration, so that every iteration's observations and rewards can be read before the next (as a
policy would).  --mode rollout times wd_rollout instead: 25 iterations per launch with the
same writes in every iteration, of which only the last iteration's survive; the default run
reports it among the extras.  The metric is the paper's
(Sec. 5.3): environment steps per second at 2000 environments x 1000 agents; agent-steps/s and
the fraction of the HBM roofline are reported next to it, and the CPU oracle is timed on the
host cores as a baseline.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--mode fused|rollout|separate]

Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth
RING = 8               # steps of policy outputs resident before the timed region
PAPER_ENV_STEPS_PER_S = 2.9e6  # Sec. 5.3, one A100: context only


def read_traffic(workload, iterations_per_launch):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 counter summary, and
    where it comes from: (None, None) unless that summary was taken with the same number of
    iterations per launch.  The counters cannot be read inside this run; the figure is the one of the
    profile run that the file names."""
    rel = os.path.join("profiles", f"hbm_traffic_{workload}.txt")
    path = os.path.join(ROOT, rel)
    if not os.path.exists(path):
        return None, None
    found = {}
    window = ""
    for line in open(path):
        parts = line.split()
        if len(parts) == 2 and parts[0] in ("traffic_bytes_per_launch", "iterations_per_launch"):
            found[parts[0]] = float(parts[1])
        if line.startswith("window "):
            window = line[len("window "):].strip()
    if found.get("iterations_per_launch", 1) != iterations_per_launch or "traffic_bytes_per_launch" not in found:
        return None, None
    return found["traffic_bytes_per_launch"], f"{rel} (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, not measured in this run; {window})"


def run_iterations(env, ring, first_g, count, mode, per_launch=1):
    """Enqueues `count` roll-out iterations; returns the number of launches of the dominant kernel."""
    import paper_2108_13976_amd as wd

    if mode == "rollout":  # several iterations per launch, every output in place as with wd_iterate
        launches = 0
        while count > 0:
            k = min(per_launch, count)
            wd.wd_rollout(env.handle, ring.data_ptr(), RING, k, None)
            count -= k
            launches += 1
        return launches
    for k in range(count):
        probs = ring[(first_g + k) % RING]
        if mode == "fused":
            env.iterate(probs)
        else:
            env.sample(probs)
            env.step()
            env.reset(wd.WD_RESET_DONE)
    return count


def wake_device(cfg, ring, iterations=400):
    """Untimed: runs the workload for a moment so that the device has left its idle clocks before
    anything is timed (the first few hundred launches of a process run up to 15 % slower)."""
    import torch
    import paper_2108_13976_amd as wd

    env = wd.TagEnvs(device="cuda:0", **cfg.kwargs())
    env.reset(wd.WD_RESET_ALL)
    run_iterations(env, ring, 0, iterations, "fused")
    torch.cuda.synchronize()
    env.close()


def contract_window(cfg, ring, repetitions=5, warmup=50):
    """The measurement window of the method's roll-out throughput whatever --steps says: 2 T iterations
    (two episode lengths: runners leaving the game, envs ending early, staggered resets are all
    inside) after `warmup` iterations from the reset state, `repetitions` times; one wd_iterate launch
    per iteration, HIP events on the launch stream."""
    steps = 2 * cfg.episode_length
    launch_us, rates = [], []
    bytes_per_iteration = None
    for _ in range(repetitions):
        wall, event_s, _, bytes_per_iteration, launches = time_gpu(cfg, ring, steps, warmup, "fused")
        launch_us.append(event_s / launches * 1e6)
        rates.append(steps / wall * cfg.num_envs)
    launch_us.sort()
    rates.sort()
    mid = len(launch_us) // 2
    gbs = bytes_per_iteration / (launch_us[mid] * 1e-6) / 1e9
    out = {"iterations": steps, "warmup": warmup, "repetitions": repetitions,
           "avg_launch_us": launch_us[mid], "avg_launch_us_min": launch_us[0], "avg_launch_us_max": launch_us[-1],
           "env_steps_per_s": rates[mid], "env_steps_per_s_min": rates[0], "env_steps_per_s_max": rates[-1],
           "achieved": gbs, "frac": gbs / HBM_PEAK_GBS}
    out.update(window_statistics(cfg, ring, steps, warmup))
    return out


def time_gpu(cfg, ring, steps, warmup, mode, per_launch=1, **over):
    """Returns (seconds for `steps` iterations by the host clock, same by HIP events, final state
    stats, algorithmic bytes per iteration, launches of the dominant kernel in the timed region)."""
    import torch
    import paper_2108_13976_amd as wd

    kw = cfg.kwargs()
    kw.update(over)
    env = wd.TagEnvs(device="cuda:0", **kw)
    env.reset(wd.WD_RESET_ALL)
    run_iterations(env, ring, 0, warmup, mode, per_launch)
    start_ev, end_ev = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    start_ev.record(env.torch_stream)
    launches = run_iterations(env, ring, warmup, steps, mode, per_launch)
    end_ev.record(env.torch_stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    event_s = start_ev.elapsed_time(end_ev) / 1e3
    stats = {
        "live_fraction_at_end": float(env.live.float().mean().item()),
        "mean_t_at_end": float(env.t.float().mean().item()),
    }
    bytes_per_iteration = env.layout.bytes_per_iteration
    env.close()
    return wall, event_s, stats, bytes_per_iteration, launches


def window_statistics(cfg, ring, steps, warmup):
    """Untimed pass over the timed window's iterations: mean fraction of agents in play and mean
    number of envs reset per iteration (state read back after every iteration)."""
    import torch
    import paper_2108_13976_amd as wd

    env = wd.TagEnvs(device="cuda:0", **cfg.kwargs())
    env.reset(wd.WD_RESET_ALL)
    run_iterations(env, ring, 0, warmup, "fused")
    live = torch.zeros((), dtype=torch.float64, device="cuda:0")
    resets = torch.zeros((), dtype=torch.int64, device="cuda:0")
    for k in range(steps):
        env.iterate(ring[(warmup + k) % RING])
        live += env.live.sum(dtype=torch.float64)
        resets += (env.t == 0).sum()
    torch.cuda.synchronize()
    out = {"mean_live_fraction": float(live.item()) / (steps * cfg.num_envs * cfg.num_agents),
           "resets_per_iteration": float(resets.item()) / steps}
    env.close()
    return out


def device_copy_gbs(mib=1024, reps=10):
    """Bytes read plus bytes written per second by a plain device-to-device copy of `mib` MiB."""
    import torch

    src = torch.empty(mib << 20, dtype=torch.uint8, device="cuda:0")
    dst = torch.empty_like(src)
    dst.copy_(src)
    start_ev, end_ev = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    start_ev.record()
    for _ in range(reps):
        dst.copy_(src)
    end_ev.record()
    torch.cuda.synchronize()
    return 2.0 * (mib << 20) * reps / (start_ev.elapsed_time(end_ev) / 1e3) / 1e9


def time_sampler(cfg, ring, reps=200):
    """wd_sample and torch.multinomial on the same [E*N, 5] probabilities: actions per second."""
    import torch
    import paper_2108_13976_amd as wd

    env = wd.TagEnvs(device="cuda:0", **cfg.kwargs())
    env.reset(wd.WD_RESET_ALL)
    flat = [r.view(-1, 5) for r in ring]

    def timed(fn):
        for k in range(10):
            fn(k)
        s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        s.record(env.torch_stream)
        for k in range(reps):
            fn(k)
        e.record(env.torch_stream)
        torch.cuda.synchronize()
        return s.elapsed_time(e) / 1e3 / reps

    t_wd = timed(lambda k: env.sample(ring[k % RING]))
    t_torch = timed(lambda k: torch.multinomial(flat[k % RING], 1))
    agents = cfg.num_envs * cfg.num_agents
    env.close()
    return {"sampler_actions_per_s": agents / t_wd, "torch_multinomial_actions_per_s": agents / t_torch,
            "sampler_over_torch": t_torch / t_wd, "sampler_us": t_wd * 1e6}


def rollout_offered(cfg):
    """wd_rollout has a multi-step kernel for partial observations (K <= 8, small layout); other
    configurations run it as one launch per iteration.  With full observations the recorded
    roll-out arrays would not fit, so the extras leave that mode out."""
    return cfg.obs_mode == 0


def time_rollout(cfg, ring, k=25, steps=1000, warmup=50):
    """wd_rollout with every iteration's action, reward, done and observations recorded in
    [k, ...] arrays (paper Sec. 4.5 item 7: roll-out data gathered into a training batch), over
    the same iterations as the main timing."""
    import torch
    import paper_2108_13976_amd as wd
    from paper_2108_13976_amd.binding import wd_rollout_buffers

    env = wd.TagEnvs(device="cuda:0", **cfg.kwargs())
    env.reset(wd.WD_RESET_ALL)
    E, N, D = env.E, env.N, env.D
    out = {"action": torch.empty((k, E, N), dtype=torch.int32, device=env.device),
           "reward": torch.empty((k, E, N), dtype=torch.float32, device=env.device),
           "done": torch.empty((k, E), dtype=torch.int32, device=env.device),
           "obs": torch.empty((k, E, N, D), dtype=torch.float32, device=env.device)}
    bufs = wd_rollout_buffers(*[out[n].data_ptr() for n in ("action", "reward", "done", "obs")])
    launches = max(1, steps // k)
    for _ in range(max(1, warmup // k)):
        wd.wd_rollout(env.handle, ring.data_ptr(), RING, k, bufs)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(launches):
        wd.wd_rollout(env.handle, ring.data_ptr(), RING, k, bufs)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    env.close()
    return {"rollout_recorded_k": k, "rollout_recorded_env_steps_per_s": launches * k * cfg.num_envs / dt,
            "rollout_recorded_us_per_iteration": dt / (launches * k) * 1e6}


def time_oracle(cfg, ring, envs_per_thread, iterations, threads):
    """The oracle as it stands on a bounded slice of the same workload: the first envs, from the
    reset state, the same probabilities.  Returns env-steps/s."""
    import numpy as np
    from oracle import tag_oracle

    n_envs = envs_per_thread * threads
    kw = cfg.kwargs()
    kw["num_envs"] = n_envs
    orc = tag_oracle.TagOracle(**kw)
    host_probs = [ring[g % RING][:n_envs].cpu().numpy() for g in range(min(iterations, RING))]

    def work(shard):
        lo = shard.cfg.env_offset
        shard.reset()
        for g in range(iterations):
            shard.iterate(np.ascontiguousarray(host_probs[g % len(host_probs)][lo:lo + shard.E]), g)

    t0 = time.perf_counter()
    used = tag_oracle.run_sharded(orc, work, threads)
    dt = time.perf_counter() - t0
    return n_envs * iterations / dt, used, dt


def continuous_ring(cfg, device="cuda:0"):
    """A ring of RING steps of [E, N, 2, 5] probabilities (softmax of N(0,1) logits per category) on the device."""
    import torch

    gen = torch.Generator(device=device)
    gen.manual_seed(int(cfg.seed))
    logits = torch.randn((RING, cfg.num_envs, cfg.num_agents, 2, 5), generator=gen, device=device, dtype=torch.float32)
    return torch.softmax(logits, dim=-1).contiguous()


def time_continuous(cfg, ring, steps, warmup):
    """Continuous Tag (paper Sec. 5.1, second variant; Sec. 5.3 quotes it at 2000 envs x 5 agents): `steps`
    wdc_iterate launches after `warmup` from the reset state.  Returns (wall seconds, event seconds,
    algorithmic bytes per iteration)."""
    import torch
    import paper_2108_13976_amd as wd

    env = wd.CTagEnvs(device="cuda:0", **cfg.kwargs())
    env.reset(wd.WD_RESET_ALL)
    for k in range(warmup):
        env.iterate(ring[k % RING])
    s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    s.record(env.torch_stream)
    for k in range(steps):
        env.iterate(ring[(warmup + k) % RING])
    e.record(env.torch_stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    out = wall, s.elapsed_time(e) / 1e3, env.layout.bytes_per_iteration
    env.close()
    return out


def time_continuous_rollout(cfg, ring, steps, warmup, k=25):
    """The same iterations through wdc_rollout, k per launch, outputs in place."""
    import torch
    import paper_2108_13976_amd as wd

    env = wd.CTagEnvs(device="cuda:0", **cfg.kwargs())
    env.reset(wd.WD_RESET_ALL)
    for _ in range(max(1, warmup // k)):
        wd.wdc_rollout(env.handle, ring.data_ptr(), RING, k, None)
    s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    s.record(env.torch_stream)
    launches = max(1, steps // k)
    for _ in range(launches):
        wd.wdc_rollout(env.handle, ring.data_ptr(), RING, k, None)
    e.record(env.torch_stream)
    torch.cuda.synchronize()
    us = s.elapsed_time(e) * 1e3 / (launches * k)
    env.close()
    return us


def continuous_figures(cfg, steps=None, warmup=50):
    steps = steps or 2 * cfg.episode_length
    ring = continuous_ring(cfg)
    runs = sorted(time_continuous(cfg, ring, steps, warmup) for _ in range(3))
    wall, ev, nbytes = runs[1]
    roll_us = sorted(time_continuous_rollout(cfg, ring, steps, warmup) for _ in range(3))[1]
    return {"rollout_us_per_iteration": roll_us, "rollout_env_steps_per_s": cfg.num_envs / (roll_us * 1e-6),
            "rollout_iterations_per_launch": 25,"us_per_iteration": ev / steps * 1e6, "env_steps_per_s": steps / wall * cfg.num_envs,
            "agent_steps_per_s": steps / wall * cfg.num_envs * cfg.num_agents, "iterations": steps, "warmup": warmup,
            "algorithmic_bytes_per_iteration": nbytes, "hbm_frac": nbytes / (ev / steps) / 1e9 / HBM_PEAK_GBS}


def time_continuous_oracle(cfg, envs, iterations, threads):
    import numpy as np
    from oracle import ctag_oracle, tag_oracle
    from workloads import ctag_probs_for_step

    kw = cfg.kwargs()
    kw["num_envs"] = envs
    orc = ctag_oracle.CTagOracle(**kw)
    probs = [ctag_probs_for_step(cfg.seed, g, envs, cfg.num_agents) for g in range(RING)]

    def work(shard):
        lo = shard.cfg.env_offset
        shard.reset()
        for g in range(iterations):
            shard.iterate(np.ascontiguousarray(probs[g % RING][lo:lo + shard.E]), g)

    t0 = time.perf_counter()
    used = tag_oracle.run_sharded(orc, work, threads)
    dt = time.perf_counter() - t0
    return envs * iterations / dt, used, dt


def main_continuous(args):
    """bench.py --workload ctag_*: the same JSON line for a continuous-Tag workload."""
    from workloads import CTAG_CONFIGS

    cfg = CTAG_CONFIGS[args.workload]
    ring = continuous_ring(cfg)
    time_continuous(cfg, ring, 400, 0)  # untimed: the device leaves its idle clocks
    wall, ev, nbytes = time_continuous(cfg, ring, args.steps, args.warmup)
    gbs = nbytes / (ev / args.steps) / 1e9
    out = {
        "metric": "env_steps_per_s", "value": args.steps / wall * cfg.num_envs, "unit": "env-steps/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": 1e3 * wall / args.steps, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32 state, rewards and observations", "data": "synthetic",
        "config": {"workload": args.workload, "num_envs": cfg.num_envs, "num_agents": cfg.num_agents,
                   "num_taggers": cfg.num_taggers, "world_size": cfg.world_size, "num_headings": cfg.num_headings,
                   "episode_length": cfg.episode_length, "obs": f"partial K={cfg.obs_k}", "seed": cfg.seed, "mode": "fused",
                   "probs": f"softmax(N(0,1)) float32 per action category, ring of {RING} steps resident in HBM"},
        "agent_steps_per_s": args.steps / wall * cfg.num_envs * cfg.num_agents,
        "paper_env_steps_per_s_a100": 8.3e6 if args.workload == "ctag_2000x5" else None,
        "roofline": {"bound": "hbm", "kernel": "wdc env_kernel (sample + step + reset fused)", "achieved": gbs,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS,
                     "algorithmic_bytes_per_launch": nbytes, "avg_launch_us": ev / args.steps * 1e6, "traffic": None,
                     "window": f"{args.steps} iterations after {args.warmup} from the reset state"},
    }
    if not args.no_cpu_baseline:
        threads = max(1, min(16, os.cpu_count() or 1))
        envs = min(cfg.num_envs, 64 * threads)
        probe, _, _ = time_continuous_oracle(cfg, envs, 20, threads)
        iters = int(max(40, min(20000, 10.0 * probe / envs)))  # about 10 s of oracle work
        value, used, dt = time_continuous_oracle(cfg, envs, iters, threads)
        out["cpu_baseline"] = {"value": value, "unit": "env-steps/s", "cores": used, "kind": "oracle",
                               "sample": f"first {envs} envs of {args.workload} x {iters} iterations from the reset state, "
                                         f"one single-threaded oracle per core on disjoint envs ({dt:.1f} s wall)"}
    print(json.dumps(out), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="tag_2000x1000")
    ap.add_argument("--mode", choices=("fused", "rollout", "separate"), default="fused",
                    help="fused: one wd_iterate launch per iteration (every iteration's outputs can be read "
                         "before the next); rollout: wd_rollout, several iterations per launch, outputs in "
                         "place (only the last iteration's survive); separate: wd_sample, wd_step, wd_reset "
                         "per iteration")
    ap.add_argument("--iterations-per-launch", type=int, default=25, help="rollout mode only")
    ap.add_argument("--obs", choices=("partial", "full"), default="partial",
                    help="observation mode; full = one slot per agent (D = 5 + 4N), HBM-write bound")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true")
    ap.add_argument("--copy-probe-mib", type=int, default=0,
                    help="instead of the benchmark, run a plain device copy of this many MiB ten times "
                         "(the known-size kernel that calibrates the FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; envs would shard across GPUs with no exchange, "
              "but no multi-GPU figure is produced here (use --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2108_13976_amd as wd
    from workloads import CONFIGS, device_probs_ring

    wd.load_library()  # fails loudly if the HIP library has not been built
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    if args.copy_probe_mib:
        n = args.copy_probe_mib * 1024 * 1024 // 4
        src = torch.ones(n, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_probe_mib": args.copy_probe_mib, "reads_kib": args.copy_probe_mib * 1024,
                          "writes_kib": args.copy_probe_mib * 1024}))
        return
    if args.workload.startswith("ctag_"):
        main_continuous(args)
        return
    cfg = CONFIGS[args.workload]
    if args.obs == "full":
        import dataclasses
        cfg = dataclasses.replace(cfg, obs_mode=1)
    ring = device_probs_ring(cfg.seed, RING, cfg.num_envs, cfg.num_agents, "cuda:0")
    torch.cuda.synchronize()
    if args.obs == "partial":
        wake_device(cfg, ring)

    mode = args.mode
    if mode == "rollout" and not rollout_offered(cfg):
        print("bench.py: the library does not offer wd_rollout for this configuration", file=sys.stderr)
        sys.exit(2)
    per_launch = args.iterations_per_launch if mode == "rollout" else 1
    wall, event_s, stats, bytes_per_iteration, launches = time_gpu(cfg, ring, args.steps, args.warmup, mode, per_launch)
    iters_per_s = args.steps / wall
    env_steps = iters_per_s * cfg.num_envs
    agent_steps = env_steps * cfg.num_agents
    launch_s = event_s / launches  # average duration of one launch on its stream (gaps included)
    bytes_per_launch = bytes_per_iteration * args.steps / launches
    achieved_gbs = bytes_per_launch / launch_s / 1e9
    traffic, traffic_source = (read_traffic(args.workload, per_launch) if (args.obs == "partial" and mode != "separate")
                               else (None, None))
    kernel_name = {"rollout": f"rollout_kernel ({per_launch} iterations of sample + step + reset per launch)",
                   "fused": "env_kernel (sample + step + reset fused)",
                   "separate": "sample + step + reset kernels"}[mode]

    out = {
        "metric": "env_steps_per_s",
        "value": env_steps,
        "unit": "env-steps/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": 1e3 * wall / args.steps,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int32 state, f32 rewards/observations",
        "data": "synthetic",
        "config": {
            "workload": args.workload, "num_envs": cfg.num_envs, "num_agents": cfg.num_agents,
            "num_taggers": cfg.num_taggers, "grid_size": cfg.grid_size, "episode_length": cfg.episode_length,
            "obs": f"partial K={cfg.obs_k}" if cfg.obs_mode == 0 else f"full D={cfg.obs_dim}", "tag_r2": cfg.tag_r2, "seed": cfg.seed, "mode": mode,
            "iterations_per_launch": per_launch,
            "probs": f"softmax(N(0,1)) float32, ring of {RING} steps resident in HBM",
        },
        "agent_steps_per_s": agent_steps,
        "paper_env_steps_per_s_a100": PAPER_ENV_STEPS_PER_S,
        "roofline": {
            "bound": "hbm",
            "kernel": kernel_name,
            "achieved": achieved_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved_gbs / HBM_PEAK_GBS,
            "algorithmic_bytes_per_launch": bytes_per_launch, "avg_launch_us": launch_s * 1e6,
            "traffic": traffic,
            "traffic_source": traffic_source,
            "window": f"{args.steps} iterations after {args.warmup} from the reset state (the arguments of this run)",
            **({"note": "inside a launch positions, live flags and env scalars stay on chip (36 of the 140 "
                        "algorithmic bytes per agent-step are not moved in 24 of 25 iterations)"}
               if mode == "rollout" else {}),
            **({"note": "rows of agents that were already out of play are kept in place, only their time feature "
                        "is rewritten: fewer bytes move than the algorithmic figure, so frac can exceed 1; "
                        "extras.all_live_hbm_frac is the figure with every row written"}
               if args.obs == "full" else {}),
        },
        "state_at_end": stats,
    }

    if not args.no_extras and args.obs == "partial" and mode == "fused":
        # the contracted window, independent of --steps / --warmup
        out["roofline"]["window_2T"] = contract_window(cfg, ring)

    if not args.no_extras:
        extras = {}
        # the same timed window four more times (each from a fresh reset): median and spread of five
        runs = [env_steps]
        for _ in range(4):
            w_rep, _, _, _, _ = time_gpu(cfg, ring, args.steps, args.warmup, mode, per_launch)
            runs.append(args.steps / w_rep * cfg.num_envs)
        runs.sort()
        extras["env_steps_per_s_5_runs"] = {"median": runs[2], "min": runs[0], "max": runs[-1]}
        extras.update(window_statistics(cfg, ring, args.steps, args.warmup))
        # the roofline fraction again, against a plain device-to-device copy instead of the published peak
        copy_gbs = device_copy_gbs()
        extras["device_copy_gbs"] = copy_gbs
        extras["frac_of_device_copy"] = achieved_gbs / copy_gbs
        # what a brute-force step would evaluate (runner x tagger pairs for the tag check, agent x
        # agent pairs for the neighbour search); the kernels evaluate far fewer, by bucket
        pairs = (cfg.num_agents - cfg.num_taggers) * cfg.num_taggers + cfg.num_agents * (cfg.num_agents - 1)
        extras["brute_force_pair_evaluations_per_s"] = env_steps * pairs
        # worst case for the neighbour search: tagging disabled, every agent live in every step
        short = min(args.steps, 300)
        w2, e2, _, _, _ = time_gpu(cfg, ring, short, 25, mode, per_launch, tag_r2=-1)
        extras["all_live_env_steps_per_s"] = short / w2 * cfg.num_envs
        extras["all_live_hbm_frac"] = bytes_per_iteration / (e2 / short) / 1e9 / HBM_PEAK_GBS
        # the sampler alone against the framework's operator on the same probabilities
        # (paper Sec. 5.4 compares its sampler with the PyTorch one)
        extras.update(time_sampler(cfg, ring))
        if rollout_offered(cfg):
            extras.update(time_rollout(cfg, ring, k=per_launch if mode == "rollout" else 25))
        # the other launch shapes over the same iterations as the main timing
        for other in ("rollout", "fused", "separate"):
            if other == mode or (other == "rollout" and not rollout_offered(cfg)):
                continue
            k_other = args.iterations_per_launch if other == "rollout" else 1
            w3, _, _, _, _ = time_gpu(cfg, ring, args.steps, args.warmup, other, k_other)
            extras[f"{other}_env_steps_per_s"] = args.steps / w3 * cfg.num_envs
        if args.obs == "partial" and mode == "fused" and cfg.num_envs * cfg.num_agents * (5 + 4 * cfg.num_agents) * 4 <= 64 << 30:
            # the same workload with full observations (one slot per agent, paper Sec. 5.1 / 5.5): a short
            # window from the reset state, and the same with tagging switched off (every row written)
            import dataclasses
            full_cfg = dataclasses.replace(cfg, obs_mode=1)
            wf, ef, _, bf, lf = time_gpu(full_cfg, ring, 20, 5, "fused")
            wa, ea, _, _, la = time_gpu(full_cfg, ring, 20, 5, "fused", tag_r2=-1)
            extras["full_observations"] = {
                "obs_dim": full_cfg.obs_dim, "iterations": 20, "warmup": 5,
                "us_per_iteration": ef / lf * 1e6, "env_steps_per_s": 20 / wf * cfg.num_envs,
                "algorithmic_bytes_per_iteration": bf, "hbm_frac": bf / (ef / lf) / 1e9 / HBM_PEAK_GBS,
                "all_rows_written_us_per_iteration": ea / la * 1e6,
                "all_rows_written_hbm_frac": bf / (ea / la) / 1e9 / HBM_PEAK_GBS,
            }
        if args.obs == "partial" and mode == "fused":
            # all five workloads over their own 2 T windows (one wd_iterate launch per iteration)
            per_config = {}
            for name, other in CONFIGS.items():
                other_ring = ring if name == args.workload else device_probs_ring(other.seed, RING, other.num_envs,
                                                                                   other.num_agents, "cuda:0")
                w = contract_window(other, other_ring, repetitions=3)
                # the same window through wd_rollout, 25 iterations per call, outputs in place
                _, ev_roll, _, _, _ = time_gpu(other, other_ring, w["iterations"], 50, "rollout", 25)
                per_config[name] = {"us_per_iteration": w["avg_launch_us"], "env_steps_per_s": w["env_steps_per_s"],
                                    "rollout_us_per_iteration": ev_roll / w["iterations"] * 1e6,
                                    "agent_steps_per_s": w["env_steps_per_s"] * other.num_agents,
                                    "hbm_frac": w["frac"], "iterations": w["iterations"],
                                    "mean_live_fraction": w["mean_live_fraction"],
                                    "resets_per_iteration": w["resets_per_iteration"]}
                del other_ring
            extras["configs"] = per_config
            # the paper's other discrete-Tag shape (Sec. 5.3 quotes its throughput at 2000 envs x 5 agents as well):
            # tag_10x5 with 2000 envs, same windows
            import dataclasses
            small = dataclasses.replace(CONFIGS["tag_10x5"], name="tag_2000x5", num_envs=2000, seed=5)
            small_ring = device_probs_ring(small.seed, RING, small.num_envs, small.num_agents, "cuda:0")
            w = contract_window(small, small_ring, repetitions=3)
            _, ev_roll, _, _, _ = time_gpu(small, small_ring, w["iterations"], 50, "rollout", 25)
            extras["tag_2000x5"] = {"us_per_iteration": w["avg_launch_us"], "env_steps_per_s": w["env_steps_per_s"],
                                    "rollout_us_per_iteration": ev_roll / w["iterations"] * 1e6,
                                    "rollout_env_steps_per_s": small.num_envs / (ev_roll / w["iterations"]),
                                    "iterations": w["iterations"]}
            del small_ring
            # continuous Tag (paper Sec. 5.1, second variant): its three workloads, 2 T iterations after 50
            from workloads import CTAG_CONFIGS
            extras["continuous_tag"] = {name: continuous_figures(c) for name, c in CTAG_CONFIGS.items()}
        out["extras"] = extras

    if not args.no_cpu_baseline:
        threads = max(1, min(16, os.cpu_count() or 1))
        iters = 40
        # about 12 s of oracle work per thread (its cost grows with the square of the agent count)
        per_thread = int(12.0 / (iters * 1e-9 * cfg.num_agents ** 2 + 1e-6))
        per_thread = max(1, min(per_thread, cfg.num_envs // threads))
        one, _, dt1 = time_oracle(cfg, ring, per_thread, iters, 1)
        allc, used, dtn = time_oracle(cfg, ring, per_thread, iters, threads)
        out["cpu_baseline"] = {
            "value": allc, "unit": "env-steps/s", "cores": used, "kind": "oracle",
            "sample": f"first {per_thread * used} envs of {args.workload} x {iters} iterations from the reset state, "
                      f"one single-threaded oracle per core on disjoint envs ({dtn:.1f} s wall)",
            "value_1core": one,
            "sample_1core": f"first {per_thread} envs x {iters} iterations ({dt1:.1f} s)",
            "gpu_over_cpu": env_steps / allc,
        }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
