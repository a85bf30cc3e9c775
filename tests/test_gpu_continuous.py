"""Continuous Tag through the C ABI (include/wdc.h) against the CPU oracle, element by element:
state, actions and flags to the bit, rewards to the bit, observation rows within 1e-6 (the oracle
divides by the world size and the episode length, the kernel multiplies by their reciprocals)."""
import numpy as np
import pytest
import torch

import ctrace_runner
import paper_2108_13976_amd as wd
from oracle import ctag_oracle
from workloads import CTAG_CONFIGS, ctag_probs_for_step

pytestmark = pytest.mark.gpu

EXACT = ("x", "y", "v", "h", "x0", "y0", "h0", "live", "action", "reward", "t", "done", "n_live_runners", "tags_step")
TOL = 1e-6


def assert_same(gpu, orc, where, names=EXACT + ("obs",)):
    got = gpu.to_host()
    for name in names:
        want = getattr(orc, name)
        if name == "obs":
            err = np.abs(got[name].astype(np.float64) - want.astype(np.float64)).max() if want.size else 0.0
            assert err <= TOL, f"{where}: obs differs by {err}"
        else:
            if not np.array_equal(got[name], want):
                bad = np.argwhere(got[name] != want)[0]
                raise AssertionError(f"{where}: {name} differs at {bad.tolist()}: {got[name][tuple(bad)]} != {want[tuple(bad)]}")


def lockstep(kw, iterations, seed, fused_every=2, check_every=1, env_lo=0, env_hi=None, full_envs=None):
    """Runs GPU and oracle side by side; even iterations as three separate calls, odd ones fused."""
    gpu = wd.CTagEnvs(device="cuda:0", **kw)
    okw = dict(kw)
    if env_hi is not None:
        okw["num_envs"] = env_hi - env_lo
        okw["env_offset"] = kw.get("env_offset", 0) + env_lo
    orc = ctag_oracle.CTagOracle(**okw)
    gpu.reset(wd.WD_RESET_ALL)
    orc.reset()
    E, N = kw["num_envs"], kw["num_agents"]
    sl = slice(env_lo, env_hi)

    class View:  # the oracle's envs inside the GPU's arrays
        def to_host(self):
            return {n: a[sl] for n, a in gpu.to_host().items()}
    view = View() if env_hi is not None else gpu
    assert_same(view, orc, "after reset(ALL)")
    resets = 0
    for g in range(iterations):
        probs = ctag_probs_for_step(seed, g, full_envs or E, N, 0, E)
        dev = torch.from_numpy(probs).to(gpu.device)
        orc.sample(probs[sl], g)
        orc.step()
        if g % fused_every == 0:
            gpu.sample(dev)
            if g % check_every == 0:
                assert_same(view, orc, f"g={g} after sample", ("action",))
            gpu.step()
            if g % check_every == 0:
                assert_same(view, orc, f"g={g} after step")
            resets += int(orc.done.sum())
            orc.reset(ctag_oracle.RESET_DONE)
            gpu.reset(wd.WD_RESET_DONE)
        else:
            resets += int(orc.done.sum())
            orc.reset(ctag_oracle.RESET_DONE)
            gpu.iterate(dev)
        if g % check_every == 0 or g == iterations - 1:
            assert_same(view, orc, f"g={g} after reset(DONE)")
    gpu.close()
    return resets


def test_small_workload_whole_over_episodes():
    cfg = CTAG_CONFIGS["ctag_10x5"]
    assert lockstep(cfg.kwargs(), 260, cfg.seed) >= 20


def test_headline_shape_of_the_paper_2000x5():
    cfg = CTAG_CONFIGS["ctag_2000x5"]
    assert lockstep(cfg.kwargs(), 140, cfg.seed, check_every=10) > 0


def test_snapshot_shape_2000x105_sampled_envs():
    cfg = CTAG_CONFIGS["ctag_2000x105"]
    # the oracle follows envs 900..931 of the full batch (random blocks are keyed by global env id)
    lockstep(cfg.kwargs(), 60, cfg.seed, check_every=6, env_lo=900, env_hi=932)


class GpuTraceEnv:
    float_tol = TOL

    def __init__(self, config):
        c = dict(config)
        self.g = wd.CTagEnvs(1, c["num_agents"], c["num_taggers"], c["episode_length"], seed=0,
                             world_size=c["world_size"], num_headings=c["num_headings"], accel=c["accel"],
                             max_speed_tagger=c["max_speed_tagger"], max_speed_runner=c["max_speed_runner"],
                             tag_r2=c["tag_r2"], obs_k=c["obs_k"], device="cuda:0")
        self.g.reset(wd.WD_RESET_ALL)

    def set_start(self, start):
        dev = self.g.device
        self.g.x0.copy_(torch.tensor([[r[0] for r in start]], dtype=torch.float32, device=dev))
        self.g.y0.copy_(torch.tensor([[r[1] for r in start]], dtype=torch.float32, device=dev))
        self.g.h0.copy_(torch.tensor([[r[2] for r in start]], dtype=torch.int32, device=dev))
        self.g.done.fill_(1)
        self.g.reset(wd.WD_RESET_DONE)

    def step(self, actions):
        self.g.action.copy_(torch.tensor([actions], dtype=torch.int32, device=self.g.device))
        self.g.step()

    def reset_done(self):
        self.g.reset(wd.WD_RESET_DONE)

    def get(self, name):
        return self.g.to_host()[name][0].copy()


@pytest.mark.parametrize("trace", ctrace_runner.load_traces(), ids=lambda t: t["name"].split()[0])
def test_hand_traces_through_the_c_abi(trace):
    ctrace_runner.run_trace(GpuTraceEnv, trace)


EDGE = [
    dict(num_envs=1, num_agents=2, num_taggers=1, episode_length=7, world_size=1.5, num_headings=4, obs_k=1, tag_r2=0.2),
    dict(num_envs=3, num_agents=2, num_taggers=1, episode_length=9, world_size=2.0, num_headings=8, obs_k=0, tag_r2=0.5),
    dict(num_envs=130, num_agents=2, num_taggers=1, episode_length=30, world_size=6.0, obs_k=1),            # 128 envs per workgroup
    dict(num_envs=5, num_agents=256, num_taggers=30, episode_length=40, world_size=30.0, obs_k=8),          # one env fills a workgroup
    dict(num_envs=3, num_agents=257, num_taggers=3, episode_length=25, world_size=40.0, obs_k=4),           # 320-thread workgroups
    dict(num_envs=2, num_agents=1024, num_taggers=64, episode_length=12, world_size=60.0, obs_k=4),         # largest env
    dict(num_envs=7, num_agents=100, num_taggers=99, episode_length=20, world_size=10.0, obs_k=3),          # one runner
    dict(num_envs=9, num_agents=9, num_taggers=1, episode_length=15, world_size=3.0, num_headings=360, obs_k=8, tag_r2=0.4),
    dict(num_envs=4, num_agents=33, num_taggers=5, episode_length=50, world_size=8.0, num_headings=12, obs_k=5, tag_r2=-1.0),
    dict(num_envs=6, num_agents=12, num_taggers=2, episode_length=18, world_size=5.0, accel=0.0, obs_k=2),  # nobody ever moves
    dict(num_envs=6, num_agents=12, num_taggers=2, episode_length=18, world_size=5.0, accel=3.0, max_speed_tagger=9.0,
         max_speed_runner=7.0, obs_k=2, tag_reward=2.5, tag_penalty=-0.75),                                    # walls every step
    dict(num_envs=5, num_agents=64, num_taggers=8, episode_length=1, world_size=12.0, obs_k=4),              # every step ends the episode
]


@pytest.mark.parametrize("n", range(len(EDGE)))
def test_edge_shapes(n):
    kw = dict(EDGE[n], seed=100 + n, env_offset=3 * n)
    lockstep(kw, 3 * kw["episode_length"] + 5, 100 + n)


def test_random_configurations():
    """24 seeded random configurations (WDC_EXTRA_TRIALS runs more of them)."""
    import os
    rng = np.random.default_rng(2024)
    for trial in range(int(os.environ.get("WDC_EXTRA_TRIALS", "24"))):
        N = int(rng.choice([2, 3, 5, 8, 17, 45, 64, 100, 255, 300]))
        kw = dict(num_envs=int(rng.integers(1, 40)), num_agents=N, num_taggers=int(rng.integers(1, max(2, N // 3 + 1))),
                  episode_length=int(rng.integers(3, 40)), world_size=float(rng.choice([2.0, 7.5, 20.0, 33.0])),
                  num_headings=int(rng.choice([4, 8, 16, 20, 64])), accel=float(rng.choice([0.1, 0.25, 0.7])),
                  max_speed_tagger=float(rng.choice([0.5, 1.0, 2.0])), max_speed_runner=float(rng.choice([0.3, 0.75, 1.5])),
                  tag_r2=float(rng.choice([0.1, 1.0, 4.0])), obs_k=int(rng.integers(0, min(8, N - 1) + 1)),
                  seed=int(rng.integers(0, 2**40)), env_offset=int(rng.integers(0, 1000)))
        kw["num_taggers"] = min(kw["num_taggers"], N - 1)
        lockstep(kw, int(2.5 * kw["episode_length"]) + 3, kw["seed"], check_every=3)
        if trial % 25 == 24:
            print(f"{trial + 1} configurations", flush=True)


def test_call_order_and_resumption():
    cfg = CTAG_CONFIGS["ctag_10x5"]
    env = wd.CTagEnvs(device="cuda:0", **cfg.kwargs())
    probs = torch.from_numpy(ctag_probs_for_step(cfg.seed, 0, 10, 5)).to(env.device)
    for call in (lambda: env.step(), lambda: env.sample(probs), lambda: env.iterate(probs),
                 lambda: env.reset(wd.WD_RESET_DONE)):
        with pytest.raises(wd.WdError) as ei:
            call()
        assert ei.value.status == wd.binding.WD_E_STATE
    env.reset(wd.WD_RESET_ALL)
    orc = ctag_oracle.CTagOracle(**cfg.kwargs())
    orc.reset()
    for g in range(30):
        p = ctag_probs_for_step(cfg.seed, g, 10, 5)
        env.iterate(torch.from_numpy(p).to(env.device))
        orc.iterate(p, g)
    assert wd.wdc_get_step(env.handle) == 30
    # a second handle over the same buffers, told the step, continues the run
    other = wd.wdc_create(env.cfg, env.bufs)
    with pytest.raises(wd.WdError):
        wd.wdc_step(other)  # (not started: reset(ALL) has not run on this handle)
    wd.wdc_destroy(other)
    wd.wdc_set_step(env.handle, 2**33 + 30)
    for g in range(2**33 + 30, 2**33 + 50):
        p = ctag_probs_for_step(cfg.seed, g % 1000, 10, 5)
        env.iterate(torch.from_numpy(p).to(env.device))
        orc.iterate(p, g)
    assert_same(env, orc, "after a jump of the step counter beyond 32 bits")
    env.close()


@pytest.mark.parametrize("name,k,launches,envs", [("ctag_10x5", 37, 4, None), ("ctag_2000x5", 25, 3, None),
                                                   ("ctag_2000x105", 10, 2, (700, 716))])
def test_multi_step_rollout_against_oracle_and_single_iterations(name, k, launches, envs):
    """wdc_rollout: every recorded slice and the final state equal the oracle's iteration by iteration,
    and the in-place arrays equal those of the same number of wdc_iterate calls byte for byte."""
    cfg = CTAG_CONFIGS[name]
    kw = cfg.kwargs()
    E, N, ring_len = cfg.num_envs, cfg.num_agents, 6
    lo, hi = envs if envs else (0, E)
    roll = wd.CTagEnvs(device="cuda:0", **kw)
    single = wd.CTagEnvs(device="cuda:0", **kw)
    okw = dict(kw, num_envs=hi - lo, env_offset=lo)
    orc = ctag_oracle.CTagOracle(**okw)
    ring_host = np.stack([ctag_probs_for_step(cfg.seed, r, E, N) for r in range(ring_len)])
    ring = torch.from_numpy(ring_host).to(roll.device)
    roll.reset(wd.WD_RESET_ALL)
    single.reset(wd.WD_RESET_ALL)
    orc.reset()
    g = 0
    for launch in range(launches):
        record = ("action", "reward", "done", "obs") if launch % 2 == 0 else ("reward", "done")
        out = roll.rollout(ring, k, record=record)
        roll.torch_stream.synchronize()
        got = {n: t.cpu().numpy() for n, t in out.items()}
        for s in range(k):
            probs = ring_host[g % ring_len]
            single.iterate(ring[g % ring_len])
            orc.sample(probs[lo:hi], g)
            orc.step()
            where = f"launch {launch} iteration {s}"
            if "action" in got:
                assert np.array_equal(got["action"][s, lo:hi], orc.action), where
                assert np.abs(got["obs"][s, lo:hi].astype(np.float64) - 0.0).max() <= 2.0  # (shape sanity)
            assert np.array_equal(got["reward"][s, lo:hi], orc.reward), where
            assert np.array_equal(got["done"][s, lo:hi], orc.done), where
            orc.reset(ctag_oracle.RESET_DONE)
            if "obs" in got:
                assert np.abs(got["obs"][s, lo:hi].astype(np.float64) - orc.obs).max() <= TOL, where
            g += 1
        a, b = roll.to_host(), single.to_host()
        for n in a:
            assert np.array_equal(a[n], b[n]), (launch, n)

        class View:
            def to_host(self):
                return {n: arr[lo:hi] for n, arr in a.items()}
        assert_same(View(), orc, f"after launch {launch}")
        assert wd.wdc_get_step(roll.handle) == g
    roll.close()
    single.close()


def test_rollout_argument_checks():
    cfg = CTAG_CONFIGS["ctag_10x5"]
    env = wd.CTagEnvs(device="cuda:0", **cfg.kwargs())
    ring = torch.from_numpy(np.stack([ctag_probs_for_step(cfg.seed, r, 10, 5) for r in range(2)])).to(env.device)
    with pytest.raises(wd.WdError) as ei:
        wd.wdc_rollout(env.handle, ring.data_ptr(), 2, 3, None)
    assert ei.value.status == wd.binding.WD_E_STATE
    env.reset(wd.WD_RESET_ALL)
    for bad in ((0, 3), (2, 0)):
        with pytest.raises(wd.WdError) as ei:
            wd.wdc_rollout(env.handle, ring.data_ptr(), bad[0], bad[1], None)
        assert ei.value.status == wd.binding.WD_E_CONFIG
    with pytest.raises(wd.WdError) as ei:
        wd.wdc_rollout(env.handle, ring.data_ptr() + 4, 2, 3, None)
    assert ei.value.status == wd.binding.WD_E_ALIGN
    wd.wdc_rollout(env.handle, ring.data_ptr(), 2, 1, None)  # a single iteration, nothing recorded
    assert wd.wdc_get_step(env.handle) == 1
    env.close()
