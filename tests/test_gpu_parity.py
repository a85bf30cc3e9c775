"""Parity of the HIP path (through the C ABI) with the CPU oracle, element by element, on
the same seeded inputs: bit-exact on positions, actions, live/tag/done flags and counters,
<= 1e-6 absolute on float32 rewards and observations."""
import numpy as np
import pytest

import trace_runner
from gpu_common import FLOAT_TOL, assert_equal_state, make_gpu, make_oracle, upload
from invariants import check_obs_invariants, check_step_invariants
from workloads import CONFIGS, probs_for_step

pytestmark = pytest.mark.gpu


# ---- hand traces through the C ABI ------------------------------------------------------------
class GpuTraceEnv:
    float_tol = FLOAT_TOL

    def __init__(self, config):
        import paper_2108_13976_amd as wd

        c = dict(config)
        self.wd = wd
        self.env = wd.TagEnvs(1, c["num_agents"], c["num_taggers"], c["grid_size"], c["episode_length"],
                              seed=0, tag_r2=c["tag_r2"], obs_k=c["obs_k"], obs_mode=c.get("obs_mode", 0))
        self.env.reset(wd.WD_RESET_ALL)

    def set_start(self, start):
        import torch

        s = torch.tensor(start, dtype=torch.int32, device=self.env.device)
        self.env.pos_x0[0] = s[:, 0]
        self.env.pos_y0[0] = s[:, 1]
        self.env.done[0] = 1
        self.env.reset(self.wd.WD_RESET_DONE)

    def step(self, actions):
        import torch

        self.env.action[0] = torch.tensor(actions, dtype=torch.int32, device=self.env.device)
        self.env.step()

    def reset_done(self):
        self.env.reset(self.wd.WD_RESET_DONE)

    def get(self, name):
        return self.env.to_host()[name][0]


TRACES = trace_runner.load_traces()


@pytest.mark.parametrize("trace", TRACES, ids=[t["name"].split()[0] for t in TRACES])
def test_hand_trace_on_gpu(trace):
    trace_runner.run_trace(GpuTraceEnv, trace)


# ---- lockstep roll-outs ---------------------------------------------------------------------------
def lockstep(kw, steps, probs_seed, fused, env_lo=0, env_hi=None, full_envs=None, check_every=1, sharded=0):
    """Run the GPU on envs [env_lo, env_hi) of a workload of ``full_envs`` envs next to the oracle."""
    import paper_2108_13976_amd as wd
    from oracle import tag_oracle

    full_envs = full_envs or kw["num_envs"]
    env_hi = kw["num_envs"] if env_hi is None else env_hi
    sub = dict(kw, num_envs=env_hi - env_lo, env_offset=env_lo)
    gpu = make_gpu(sub)
    orc = make_oracle(sub)
    gpu.reset(wd.WD_RESET_ALL)
    if sharded:
        tag_oracle.run_sharded(orc, lambda s: s.reset(), sharded)
    else:
        orc.reset()
    assert_equal_state(gpu.to_host(), orc, "after reset(ALL)")
    resets = 0
    for g in range(steps):
        probs = probs_for_step(probs_seed, g, full_envs, kw["num_agents"], env_lo, env_hi)
        dprobs = upload(probs, gpu.device)
        if fused:
            gpu.iterate(dprobs)
            if sharded:
                tag_oracle.run_sharded(orc, lambda s: s.iterate(probs[s.cfg.env_offset - env_lo:s.cfg.env_offset - env_lo + s.E], g), sharded)
            else:
                orc.iterate(probs, g)
            if g % check_every == 0 or g == steps - 1:
                assert_equal_state(gpu.to_host(), orc, f"after iterate {g}")
        else:
            def on_oracle(fn):
                if sharded:
                    tag_oracle.run_sharded(orc, fn, sharded)
                else:
                    fn(orc)

            gpu.sample(dprobs)
            on_oracle(lambda s: s.sample(probs[s.cfg.env_offset - env_lo:s.cfg.env_offset - env_lo + s.E], g))
            assert_equal_state(gpu.to_host(), orc, f"after sample {g}", names=("action",))
            gpu.step()
            on_oracle(lambda s: s.step())
            assert_equal_state(gpu.to_host(), orc, f"after step {g}")
            resets += int(orc.done.sum())
            gpu.reset(wd.WD_RESET_DONE)
            on_oracle(lambda s: s.reset(tag_oracle.RESET_DONE))
            assert_equal_state(gpu.to_host(), orc, f"after reset(DONE) {g}")
        assert gpu.global_step == g + 1
    gpu.close()
    return resets


def test_rollout_10x5_separate_calls():
    cfg = CONFIGS["tag_10x5"]
    resets = lockstep(cfg.kwargs(), 260, cfg.seed, fused=False)
    assert resets >= 10


def test_rollout_10x5_fused():
    cfg = CONFIGS["tag_10x5"]
    lockstep(cfg.kwargs(), 260, cfg.seed, fused=True)


def test_rollout_100x50_separate_calls():
    cfg = CONFIGS["tag_100x50"]
    lockstep(cfg.kwargs(), 150, cfg.seed, fused=False)


def test_rollout_100x50_fused_across_episode_ends():
    cfg = CONFIGS["tag_100x50"]
    lockstep(cfg.kwargs(), 2 * cfg.episode_length + 20, cfg.seed, fused=True, check_every=7)


def test_rollout_2000x1000_env_slice():
    """320 envs of the headline workload (global ids 1000..1319: enough of them for the
    one-workgroup-per-env layout the whole workload runs in), separate calls, 40 steps."""
    cfg = CONFIGS["tag_2000x1000"]
    lockstep(cfg.kwargs(), 40, cfg.seed, fused=False, env_lo=1000, env_hi=1320, full_envs=cfg.num_envs, sharded=16)


def test_rollout_2000x1000_small_env_slice():
    """24 envs of the headline workload (global ids 1000..1023): a batch this small runs in the
    large-env pair of kernels.  Fused, 40 steps."""
    cfg = CONFIGS["tag_2000x1000"]
    lockstep(cfg.kwargs(), 40, cfg.seed, fused=True, env_lo=1000, env_hi=1024, full_envs=cfg.num_envs, sharded=8)


def test_rollout_20000x100_env_slice():
    """300 envs (an odd count: the last workgroup is ragged) of the many-small-envs workload,
    fused, across episode ends."""
    cfg = CONFIGS["tag_20000x100"]
    lockstep(cfg.kwargs(), 2 * cfg.episode_length + 10, cfg.seed, fused=True, env_lo=7001, env_hi=7302,
             full_envs=cfg.num_envs, check_every=5, sharded=8)


def test_rollout_10x8192_all_envs():
    """The agent-parallel stress workload (one env exceeds a workgroup's LDS: large-env layout),
    all 10 envs, separate calls, oracle sharded over threads."""
    cfg = CONFIGS["tag_10x8192"]
    lockstep(cfg.kwargs(), 12, cfg.seed, fused=False, sharded=10)


def test_rollout_10x8192_fused_across_episode_ends():
    cfg = CONFIGS["tag_10x8192"]
    kw = dict(cfg.kwargs(), num_envs=3, episode_length=7)
    lockstep(kw, 17, cfg.seed, fused=True, full_envs=3, sharded=3)


def test_rollout_10x8192_full_episode():
    """tag_10x8192 as configured (T = 200), all 10 envs, fused, over a whole episode and the
    reset that ends it; oracle sharded one env per thread."""
    cfg = CONFIGS["tag_10x8192"]
    lockstep(cfg.kwargs(), cfg.episode_length + 5, cfg.seed, fused=True, check_every=20, sharded=10)


def largest_accepted_agent_count(**kw):
    """Largest N (with N / 10 taggers) that wd_create accepts for the rest of the configuration;
    found by bisection with placeholder buffers, which wd_create never dereferences."""
    import paper_2108_13976_amd as wd
    from paper_2108_13976_amd import binding

    bufs = binding.wd_buffers(*[0x10000 + 0x1000 * i for i in range(len(binding.BUFFER_NAMES))])

    def accepted(n):
        try:
            wd.wd_destroy(wd.wd_create(binding.make_config(num_agents=n, num_taggers=n // 10, **kw), bufs))
            return True
        except wd.WdError as err:
            assert err.status == binding.WD_E_UNSUPPORTED, err
            return False

    lo, hi = 2000, 32768
    assert accepted(lo) and not accepted(hi)
    while hi - lo > 1:
        mid = (lo + hi) // 2
        lo, hi = (mid, hi) if accepted(mid) else (lo, mid)
    return lo


@pytest.mark.parametrize("grid_size,tag_r2", [(100, 2), (700, 30)], ids=["32_bit_keys", "64_bit_keys"])
def test_largest_env_the_library_accepts(grid_size, tag_r2):
    """The largest env one workgroup's tables hold (about 13 900 agents with 32-bit keys, 11 600
    with 64-bit ones): two envs, three iterations, every element against the oracle."""
    rest = dict(num_envs=2, grid_size=grid_size, episode_length=2, tag_r2=tag_r2)
    n = largest_accepted_agent_count(**rest)
    assert n > 10000
    kw = dict(rest, num_agents=n, num_taggers=n // 10, obs_k=4, seed=77)
    lockstep(kw, 3, 78, fused=True, sharded=2)


# ---- the headline workload at full size, in the launch configuration the benchmark times ----------
def test_headline_workload_full_size_sampled_envs_and_invariants():
    import paper_2108_13976_amd as wd
    from oracle import tag_oracle

    cfg = CONFIGS["tag_2000x1000"]
    kw = cfg.kwargs()
    gpu = make_gpu(kw)
    gpu.reset(wd.WD_RESET_ALL)
    rng = np.random.default_rng(5)
    sample_envs = sorted(int(e) for e in rng.choice(cfg.num_envs, size=12, replace=False)) + [cfg.num_envs - 1]
    oracles = {e: make_oracle(kw, e, e + 1) for e in sample_envs}
    for o in oracles.values():
        o.reset()
    state = gpu.to_host()
    for e, o in oracles.items():
        assert_equal_state(state, o, f"reset env {e}", env_lo=e)
    check_obs_invariants(cfg, state, FLOAT_TOL)
    steps = 30
    for g in range(steps):
        probs = probs_for_step(cfg.seed, g, cfg.num_envs, cfg.num_agents)
        before = state
        gpu.iterate(upload(probs, gpu.device))
        state = gpu.to_host()
        for e, o in oracles.items():
            o.iterate(probs[e:e + 1], g)
            assert_equal_state(state, o, f"iterate {g} env {e}", env_lo=e)
        if g % 10 == 0:
            # no env of this workload can finish within 30 steps, so iterate == step here
            assert (state["done"] == 0).all() and (state["t"] == g + 1).all()
            check_step_invariants(cfg, before, state, FLOAT_TOL)
    gpu.close()


def test_many_small_envs_workload_full_size_sampled_envs():
    """tag_20000x100 at full size (2500 workgroups of eight envs, more than fit the chip at
    once), one wd_iterate launch per iteration as the benchmark runs it, across an episode end
    (T = 200): sampled envs against the oracle every few iterations."""
    import paper_2108_13976_amd as wd

    cfg = CONFIGS["tag_20000x100"]
    kw = cfg.kwargs()
    E, N = cfg.num_envs, cfg.num_agents
    ring_len = 4
    host_ring = np.stack([probs_for_step(cfg.seed, r, E, N) for r in range(ring_len)])
    gpu = make_gpu(kw)
    ring = upload(host_ring, gpu.device)
    gpu.reset(wd.WD_RESET_ALL)
    rng = np.random.default_rng(23)
    sample_envs = sorted(int(e) for e in rng.choice(E, size=14, replace=False)) + [0, E - 1]
    oracles = {e: make_oracle(kw, e, e + 1) for e in sample_envs}
    for o in oracles.values():
        o.reset()
    steps = cfg.episode_length + 12
    for g in range(steps):
        gpu.iterate(ring[g % ring_len])
        for e, o in oracles.items():
            o.iterate(host_ring[g % ring_len][e:e + 1], g)
        if g % 35 == 0 or g >= cfg.episode_length - 2:
            state = gpu.to_host()
            for e, o in oracles.items():
                assert_equal_state(state, o, f"iteration {g} env {e}", env_lo=e)
    check_obs_invariants(cfg, state, FLOAT_TOL)
    assert (state["t"] <= cfg.episode_length).all()
    gpu.close()


def test_headline_workload_full_size_multi_step_launches():
    """The launch shape the benchmark times: wd_rollout, 25 iterations per launch, outputs in
    place, at 2000 x 1000.  Sampled envs against the oracle after every launch; then one launch
    that records every iteration, each slice of the sampled envs against the oracle."""
    import paper_2108_13976_amd as wd

    cfg = CONFIGS["tag_2000x1000"]
    kw = cfg.kwargs()
    E, N = cfg.num_envs, cfg.num_agents
    k, ring_len = 25, 5
    host_ring = np.stack([probs_for_step(cfg.seed, r, E, N) for r in range(ring_len)])
    gpu = make_gpu(kw)
    ring = upload(host_ring, gpu.device)
    gpu.reset(wd.WD_RESET_ALL)
    rng = np.random.default_rng(11)
    sample_envs = sorted(int(e) for e in rng.choice(E, size=10, replace=False)) + [0, E - 1]
    oracles = {e: make_oracle(kw, e, e + 1) for e in sample_envs}
    for o in oracles.values():
        o.reset()
    g = 0
    for launch in range(2):
        gpu.rollout(ring, k, record=())
        for s in range(k):
            for e, o in oracles.items():
                o.iterate(host_ring[(g + s) % ring_len][e:e + 1], g + s)
        g += k
        assert gpu.global_step == g
        state = gpu.to_host()
        for e, o in oracles.items():
            assert_equal_state(state, o, f"after launch {launch} env {e}", env_lo=e)
        check_obs_invariants(cfg, state, FLOAT_TOL)
    k2 = 4
    rec = gpu.rollout(ring, k2)
    rec = {n: v.cpu().numpy() for n, v in rec.items()}
    for s in range(k2):
        for e, o in oracles.items():
            pr = host_ring[(g + s) % ring_len][e:e + 1]
            o.sample(pr, g + s)
            o.step()
            assert np.array_equal(rec["action"][s][e], o.action[0]), (s, e)
            assert np.array_equal(rec["done"][s][e:e + 1], o.done), (s, e)
            assert np.abs(rec["reward"][s][e] - o.reward[0]).max() <= FLOAT_TOL, (s, e)
            o.reset(1)
            assert np.abs(rec["obs"][s][e].astype(np.float64) - o.obs[0]).max() <= FLOAT_TOL, (s, e)
    gpu.close()


def test_headline_workload_every_env_fifty_iterations():
    """tag_2000x1000 at full size, every one of the 2000 envs against the oracle (sharded over
    the host's threads) for 50 wd_iterate launches from the reset state: the whole state after
    the reset and after iterations 1, 2, 10, 25 and 50."""
    import paper_2108_13976_amd as wd
    from oracle import tag_oracle

    cfg = CONFIGS["tag_2000x1000"]
    kw = cfg.kwargs()
    threads = 16
    gpu = make_gpu(kw)
    orc = make_oracle(kw)
    gpu.reset(wd.WD_RESET_ALL)
    tag_oracle.run_sharded(orc, lambda s: s.reset(), threads)
    assert_equal_state(gpu.to_host(), orc, "after reset(ALL)")
    for g in range(50):
        probs = probs_for_step(cfg.seed, g, cfg.num_envs, cfg.num_agents)
        gpu.iterate(upload(probs, gpu.device))
        tag_oracle.run_sharded(orc, lambda s: s.iterate(probs[s.cfg.env_offset:s.cfg.env_offset + s.E], g), threads)
        if g + 1 in (1, 2, 10, 25, 50):
            assert_equal_state(gpu.to_host(), orc, f"after iteration {g + 1}")
    gpu.close()


def test_headline_workload_full_size_two_episodes_sampled_envs():
    """tag_2000x1000 at full size for more than two episode lengths (T = 500: every env is reset at least twice),
    one wd_iterate launch per iteration; 32 random envs against the oracle at checkpoints on both
    sides of each episode end.  Between checkpoints every sampled env's oracle advances on its own
    thread (the policy outputs come from a ring, so nothing but the step counter is shared)."""
    import paper_2108_13976_amd as wd
    from concurrent.futures import ThreadPoolExecutor

    cfg = CONFIGS["tag_2000x1000"]
    kw = cfg.kwargs()
    E, N, T = cfg.num_envs, cfg.num_agents, cfg.episode_length
    ring_len = 4
    host_ring = np.stack([probs_for_step(cfg.seed, r, E, N) for r in range(ring_len)])
    gpu = make_gpu(kw)
    ring = upload(host_ring, gpu.device)
    gpu.reset(wd.WD_RESET_ALL)
    rng = np.random.default_rng(41)
    sample_envs = sorted(int(e) for e in rng.choice(E, size=32, replace=False))
    oracles = {e: make_oracle(kw, e, e + 1) for e in sample_envs}
    for o in oracles.values():
        o.reset()
    checkpoints = [60, T - 1, T, T + 1, T + 200, 2 * T - 1, 2 * T, 2 * T + 15]
    g = 0
    with ThreadPoolExecutor(max_workers=16) as pool:
        for stop in checkpoints:
            def advance(item, g0=g, g1=stop):
                e, o = item
                for s in range(g0, g1):
                    o.iterate(host_ring[s % ring_len][e:e + 1], s)
            futures = [pool.submit(advance, item) for item in oracles.items()]
            for s in range(g, stop):
                gpu.iterate(ring[s % ring_len])
            for f in futures:
                f.result()
            g = stop
            assert gpu.global_step == g
            state = gpu.to_host()
            for e, o in oracles.items():
                assert_equal_state(state, o, f"after iteration {g} env {e}", env_lo=e)
            assert (state["t"] <= T).all() and (state["done"] == 0).all()
    check_obs_invariants(cfg, state, FLOAT_TOL)
    gpu.close()


def test_full_observations_at_headline_size_sampled_envs():
    """Full observations at 2000 x 1000 (rows of 4005 floats: 8 * 10^9 observation elements,
    32 GB), the shape the benchmark times with --obs full.  Whole envs against the oracle: the
    first and the last env, the envs whose rows straddle element 2^31 and element 2^32 of the
    observation array (offsets that need 64 bits), and two more."""
    import paper_2108_13976_amd as wd

    cfg = CONFIGS["tag_2000x1000"]
    kw = dict(cfg.kwargs(), obs_mode=1)
    E, N = cfg.num_envs, cfg.num_agents
    per_env = N * (5 + 4 * N)
    sample_envs = sorted({0, (1 << 31) // per_env, (1 << 32) // per_env, 777, 1600, E - 1})
    assert sample_envs[1] * per_env < (1 << 31) < (sample_envs[1] + 1) * per_env
    gpu = make_gpu(kw)
    gpu.reset(wd.WD_RESET_ALL)
    oracles = {e: make_oracle(kw, e, e + 1) for e in sample_envs}
    for o in oracles.values():
        o.reset()

    def check(where):
        gpu.torch_stream.synchronize()
        for e, o in oracles.items():
            one = {n: t[e:e + 1].cpu().numpy() for n, t in gpu.tensors.items()}
            assert_equal_state(one, o, f"{where} env {e}")

    check("after reset(ALL)")
    for g in range(5):
        probs = probs_for_step(cfg.seed, g, E, N)
        gpu.iterate(upload(probs, gpu.device))
        for e, o in oracles.items():
            o.iterate(probs[e:e + 1], g)
        check(f"after iteration {g + 1}")
    gpu.close()


def test_headline_workload_long_recorded_launch():
    """One wd_rollout launch of 110 recorded iterations at 2000 x 1000: the recorded observations
    hold 4.6 * 10^9 floats (18 GB), so slice offsets need 64 bits.  Sampled envs against the
    oracle in the first slice, in the slices that straddle element 2^31 and element 2^32, and in
    the last; every recorded action, reward and done flag of those envs as well."""
    import paper_2108_13976_amd as wd

    cfg = CONFIGS["tag_2000x1000"]
    kw = cfg.kwargs()
    E, N, D = cfg.num_envs, cfg.num_agents, 5 + 4 * cfg.obs_k
    k, ring_len = 110, 3
    per_slice = E * N * D
    watch = sorted({0, (1 << 31) // per_slice, (1 << 32) // per_slice, k - 1})
    assert watch[-2] < k - 1
    host_ring = np.stack([probs_for_step(cfg.seed, r, E, N) for r in range(ring_len)])
    gpu = make_gpu(kw)
    ring = upload(host_ring, gpu.device)
    gpu.reset(wd.WD_RESET_ALL)
    sample_envs = [0, 1023, E - 1]  # and the envs that hold element 2^31 and element 2^32 in their slices
    sample_envs += [((1 << 31) % per_slice) // (N * D), ((1 << 32) % per_slice) // (N * D)]
    sample_envs = sorted(set(sample_envs))
    oracles = {e: make_oracle(kw, e, e + 1) for e in sample_envs}
    for o in oracles.values():
        o.reset()
    rec = gpu.rollout(ring, k)
    gpu.torch_stream.synchronize()
    assert gpu.global_step == k
    small = {n: rec[n][:, sample_envs].cpu().numpy() for n in ("action", "reward", "done")}
    obs_slices = {s: rec["obs"][s][sample_envs].cpu().numpy() for s in watch}
    for s in range(k):
        for j, (e, o) in enumerate(oracles.items()):
            o.sample(host_ring[s % ring_len][e:e + 1], s)
            o.step()
            assert np.array_equal(small["action"][s][j], o.action[0]), (s, e)
            assert small["done"][s][j] == o.done[0], (s, e)
            assert np.abs(small["reward"][s][j] - o.reward[0]).max() <= FLOAT_TOL, (s, e)
            o.reset(1)
            if s in obs_slices:
                assert np.abs(obs_slices[s][j].astype(np.float64) - o.obs[0]).max() <= FLOAT_TOL, (s, e)
    state = {n: t[sample_envs].cpu().numpy() for n, t in gpu.tensors.items()}
    for j, (e, o) in enumerate(oracles.items()):
        one = {n: v[j:j + 1] for n, v in state.items()}
        assert_equal_state(one, o, f"state after the launch, env {e}")
    gpu.close()


@pytest.mark.parametrize("name,k,rounds", [("tag_10x5", 37, 8), ("tag_100x50", 16, 5), ("tag_20000x100", 6, 2)])
def test_multi_step_rollout_equals_single_iterations(name, k, rounds):
    """wd_rollout (k iterations in one launch, per-iteration outputs) against k calls of the
    separate entry points, and both against the oracle at the end."""
    import torch
    import paper_2108_13976_amd as wd
    from oracle import tag_oracle

    cfg = CONFIGS[name]
    kw = cfg.kwargs()
    if cfg.num_envs > 500:
        kw.update(num_envs=203, env_offset=900)
    E, N = kw["num_envs"], cfg.num_agents
    lo = kw.get("env_offset", 0)
    ring_len = 5
    host_ring = np.stack([probs_for_step(cfg.seed, r, cfg.num_envs, N, lo, lo + E) for r in range(ring_len)])
    a, b = make_gpu(kw), make_gpu(kw)
    orc = make_oracle(kw)
    ring = upload(host_ring, a.device)
    a.reset(wd.WD_RESET_ALL), b.reset(wd.WD_RESET_ALL), orc.reset()
    g = 0
    for _ in range(rounds):
        rec = a.rollout(ring, k)
        for s in range(k):
            pr = ring[(g + s) % ring_len]
            b.sample(pr), b.step()
            sb = b.to_host()
            assert np.array_equal(rec["action"][s].cpu().numpy(), sb["action"])
            assert np.array_equal(rec["done"][s].cpu().numpy(), sb["done"])
            assert rec["reward"][s].cpu().numpy().tobytes() == sb["reward"].tobytes()
            b.reset(wd.WD_RESET_DONE)
            assert rec["obs"][s].cpu().numpy().tobytes() == b.to_host()["obs"].tobytes()
            orc.iterate(host_ring[(g + s) % ring_len], g + s)
        g += k
        assert a.global_step == g
        sa, sb = a.to_host(), b.to_host()
        for n in sa:
            assert sa[n].tobytes() == sb[n].tobytes(), n
        assert_equal_state(sa, orc, f"after {g} iterations")
    a.close(), b.close()


@pytest.mark.parametrize("name,k", [("large_env_k_two", 3), ("full_obs_fifty", 4), ("k_all_others", 5),
                                    ("fifteen_hundred_many_envs", 4), ("thirty_five_hundred_many_envs", 3),
                                    ("k_one_packed_envs", 5), ("k_two_odd_agent_count", 4), ("k_three", 6),
                                    ("k_eight", 5), ("k_seven_packed_envs", 4), ("k_three_one_workgroup", 6),
                                    ("k_eight_one_workgroup", 5), ("wave_full", 5), ("wave_k_seven", 4), ("wave_two_agents", 7), ("wave_k_sixteen", 4),
                                    ("beyond_wave_batch", 4), ("many_small_envs_k_two", 3)])
def test_multi_step_rollout_of_other_launch_shapes(name, k):
    """Large-env layout, full observations, K > 8 (wd_rollout runs one launch per iteration), the
    multi-step kernel in 512- and 1024-thread workgroups and its variants for other K than 4, the
    kernel with a wave per env: slices
    and final state against k calls of wd_iterate."""
    import paper_2108_13976_amd as wd

    kw = dict(EDGE[name], seed=77)
    E, N = kw["num_envs"], kw["num_agents"]
    ring_len = 3
    host_ring = np.stack([probs_for_step(77, r, E, N) for r in range(ring_len)])
    a, b = make_gpu(kw), make_gpu(kw)
    ring = upload(host_ring, a.device)
    a.reset(wd.WD_RESET_ALL), b.reset(wd.WD_RESET_ALL)
    g = 0
    for _ in range(2):
        rec = a.rollout(ring, k)
        for s in range(k):
            b.sample(ring[(g + s) % ring_len]), b.step()
            sb = b.to_host()
            assert np.array_equal(rec["action"][s].cpu().numpy(), sb["action"])
            assert np.array_equal(rec["done"][s].cpu().numpy(), sb["done"])
            assert rec["reward"][s].cpu().numpy().tobytes() == sb["reward"].tobytes()
            b.reset(wd.WD_RESET_DONE)
            assert rec["obs"][s].cpu().numpy().tobytes() == b.to_host()["obs"].tobytes()
        g += k
        assert a.global_step == g
        sa, sb = a.to_host(), b.to_host()
        for n in sa:
            assert sa[n].tobytes() == sb[n].tobytes(), n
    a.close(), b.close()


def test_multi_step_rollout_entered_with_envs_that_are_done():
    """wd_rollout called on a state in which some envs are done and not yet reset (the caller
    stepped without resetting): the first iteration must not step them, and resets them."""
    import paper_2108_13976_amd as wd

    kw = dict(num_envs=37, num_agents=12, num_taggers=3, grid_size=5, episode_length=6, obs_k=4, seed=5, tag_r2=2)
    E, N = kw["num_envs"], kw["num_agents"]
    ring_len = 4
    host_ring = np.stack([probs_for_step(5, r, E, N) for r in range(ring_len)])
    a, b = make_gpu(kw), make_gpu(kw)
    orc = make_oracle(kw)
    ring = upload(host_ring, a.device)
    a.reset(wd.WD_RESET_ALL), b.reset(wd.WD_RESET_ALL), orc.reset()
    g = 0
    for _ in range(5):  # no resets: envs finish one after another (all tagged) and stay done
        for env in (a, b):
            env.sample(ring[g % ring_len]), env.step()
        orc.sample(host_ring[g % ring_len], g), orc.step()
        g += 1
    done = a.to_host()["done"]
    assert 0 < done.sum() < E, "the case needs a mix of done and running envs"
    k = 7
    rec = a.rollout(ring, k)
    for s in range(k):
        b.iterate(ring[(g + s) % ring_len])
        orc.iterate(host_ring[(g + s) % ring_len], g + s)
        assert rec["obs"][s].cpu().numpy().tobytes() == b.to_host()["obs"].tobytes(), s
    sa, sb = a.to_host(), b.to_host()
    for n in sa:
        assert sa[n].tobytes() == sb[n].tobytes(), n
    assert_equal_state(sa, orc, "after the roll-out")
    a.close(), b.close()


def test_caller_supplied_stream_and_env_slices():
    """Two env slices of one batch, each on a stream of its own (default priority), against the
    whole batch on the default stream: the library enqueues on the stream it was given and the
    random streams are keyed by global env id."""
    import torch
    import paper_2108_13976_amd as wd

    cfg = CONFIGS["tag_100x50"]
    kw = cfg.kwargs()
    E, N = cfg.num_envs, cfg.num_agents
    whole = make_gpu(kw)
    whole.reset(wd.WD_RESET_ALL)
    cuts = [(0, 37), (37, E)]
    parts = []
    for lo, hi in cuts:
        st = torch.cuda.Stream()
        with torch.cuda.stream(st):
            env = wd.TagEnvs(stream=st, **dict(kw, num_envs=hi - lo, env_offset=lo))
        env.reset(wd.WD_RESET_ALL)
        parts.append(env)
    for g in range(25):
        probs = upload(probs_for_step(cfg.seed, g, E, N), whole.device)
        torch.cuda.synchronize()
        whole.iterate(probs)
        for env, (lo, hi) in zip(parts, cuts):
            env.iterate(probs[lo:hi])
        torch.cuda.synchronize()  # probs is released below: no stream may still be reading it
    ref = whole.to_host()
    for env, (lo, hi) in zip(parts, cuts):
        got = env.to_host()
        for n in ref:
            assert got[n].tobytes() == ref[n][lo:hi].tobytes(), (n, lo)
        env.close()
    whole.close()


def random_configuration(seed):
    """A small random configuration: every size, radius, K, observation mode and reward constant
    drawn from a seeded generator, the shapes skewed towards the layout boundaries."""
    rng = np.random.default_rng(1000 + seed)
    N = int(rng.choice([2, 3, 4, 5, 7, 8, 9, 15, 16, 17, 31, 33, 63, 64, 65, 100, 127, 129, 200, 257, 300, 511, 520]))
    G = int(rng.choice([1, 2, 3, 5, 8, 13, 21, 40, 64, 100, 300, 1000, 5000, 32767]))
    kw = dict(num_envs=int(rng.integers(1, 70)), num_agents=N, num_taggers=int(rng.integers(1, N)), grid_size=G,
              episode_length=int(rng.integers(1, 14)), seed=int(rng.integers(0, 2**31)),
              tag_r2=int(rng.choice([-1, 0, 1, 2, 4, 9, 50, 2 * G * G])),
              tag_reward=float(rng.choice([1.0, 0.5, 2.25])), tag_penalty=float(rng.choice([-1.0, -0.125, 0.0])))
    if rng.random() < 0.2 and N <= 129:
        kw["obs_mode"] = 1
    else:
        kw["obs_k"] = int(min(N - 1, rng.choice([0, 1, 2, 3, 4, 4, 4, 5, 8, 9, 16, 17, 40])))
    # batches of at most 256 envs run one env per workgroup: every other small-env configuration gets
    # more envs than that, so that the workgroups that hold several envs are exercised as well
    if seed % 2 == 1 and N <= 129 and kw.get("obs_mode", 0) == 0:
        kw["num_envs"] = 257 + int(rng.integers(0, 300))
        # envs of at most 64 agents in batches of at most 8192 envs run a wave per env: every other of these
        # configurations gets a batch beyond that, which the workgroups of several small envs serve
        if seed % 4 == 1 and N <= 64:
            kw["num_envs"] += 8192
    return kw


@pytest.mark.parametrize("seed", range(40))
def test_random_configuration(seed):
    kw = random_configuration(seed)
    steps = 2 * kw["episode_length"] + 3
    lockstep(kw, steps, kw["seed"] % 1000, fused=bool(seed & 1))


def _extra_seed_chunks(per_chunk=20):
    import os

    count = int(os.environ.get("WD_EXTRA_SEEDS", "240"))
    return [range(lo, min(lo + per_chunk, 5000 + count)) for lo in range(5000, 5000 + count, per_chunk)]


@pytest.mark.parametrize("seeds", _extra_seed_chunks(), ids=lambda r: f"seeds{r.start}-{r.stop - 1}")
def test_many_more_random_configurations(seeds):
    """Further random configurations, twenty to a test (WD_EXTRA_SEEDS of them in all, 240 by default):
    every third with 384 .. 8192 agents in a few envs, the shapes that run in either form of the
    large-env pair of kernels or in wide workgroups, with K from 0 to 16."""
    for seed in seeds:
        kw = random_configuration(seed)
        large = seed % 3 == 0
        if large:
            rng = np.random.default_rng(77000 + seed)
            n = int(rng.choice([384, 385, 640, 700, 1023, 1024, 1025, 1300, 2050, 3073, 4100, 8192]))
            taggers = int(rng.integers(1, n)) if rng.random() < 0.25 else int(rng.integers(1, max(2, n // 8)))
            kw.update(num_agents=n, num_taggers=taggers, num_envs=int(rng.integers(1, 6)),
                      episode_length=int(rng.integers(1, 5)), obs_k=int(rng.choice([0, 1, 2, 3, 4, 5, 6, 8, 9, 16])))
            kw.pop("obs_mode", None)
        try:
            lockstep(kw, 2 * kw["episode_length"] + 3, kw["seed"] % 1000, fused=bool(seed & 1), sharded=4 if large else 0)
        except AssertionError as err:
            raise AssertionError(f"seed {seed}, configuration {kw}: {err}") from err


def _multi_step_seeds():
    import os

    return range(100, 116 + int(os.environ.get("WD_EXTRA_ROLLOUT_SEEDS", "0")))


@pytest.mark.parametrize("seed", _multi_step_seeds())
def test_random_configuration_multi_step(seed):
    """wd_rollout on a random configuration: every recorded slice and the final state against one
    wd_iterate per iteration, the final state also against the oracle (WD_EXTRA_ROLLOUT_SEEDS runs
    that many further seeds)."""
    import paper_2108_13976_amd as wd

    kw = random_configuration(seed)
    E, N = kw["num_envs"], kw["num_agents"]
    ring_len, k = 3, 2 * kw["episode_length"] + 2
    host_ring = np.stack([probs_for_step(kw["seed"] % 1000, r, E, N) for r in range(ring_len)])
    a, b, orc = make_gpu(kw), make_gpu(kw), make_oracle(kw)
    ring = upload(host_ring, a.device)
    a.reset(wd.WD_RESET_ALL), b.reset(wd.WD_RESET_ALL), orc.reset()
    rec = {n: v.cpu().numpy() for n, v in a.rollout(ring, k).items()}
    for s in range(k):
        b.sample(ring[s % ring_len]), b.step()
        sb = b.to_host()
        assert np.array_equal(rec["action"][s], sb["action"]), s
        assert np.array_equal(rec["done"][s], sb["done"]), s
        assert rec["reward"][s].tobytes() == sb["reward"].tobytes(), s
        b.reset(wd.WD_RESET_DONE)
        assert rec["obs"][s].tobytes() == b.to_host()["obs"].tobytes(), s
        orc.iterate(host_ring[s % ring_len], s)
    sa, sb = a.to_host(), b.to_host()
    for n in sa:
        assert sa[n].tobytes() == sb[n].tobytes(), n
    assert_equal_state(sa, orc, "after the roll-out")
    a.close(), b.close()


@pytest.mark.parametrize("name", ["full_obs_fifty", "full_obs_one_wave", "k_seventeen", "large_env_narrow_keys",
                                  "wide_radius"])
def test_observations_overwritten_by_the_caller(name):
    """Rows of agents that were out of play before a step are kept up to date in place (only their
    time feature is rewritten by some kernels).  A caller that overwrites the observation buffer
    says so with wd_set_step; the next call then writes every row whole."""
    import paper_2108_13976_amd as wd

    kw = dict(seed=77, **EDGE[name])
    E, N = kw["num_envs"], kw["num_agents"]
    gpu, orc = make_gpu(kw), make_oracle(kw)
    gpu.reset(wd.WD_RESET_ALL), orc.reset()
    tagged = False
    for g in range(min(2 * kw["episode_length"], 40)):
        probs = probs_for_step(77, g, E, N)
        if g % 3 == 2:
            tagged = tagged or bool((orc.live == 0).any())
            gpu.tensors["obs"].fill_(-123.5)
            if g % 2:
                gpu.global_step = g  # (wd_set_step implies it)
            else:
                wd.wd_invalidate_obs(gpu.handle)
        gpu.iterate(upload(probs, gpu.device))
        orc.iterate(probs, g)
        assert_equal_state(gpu.to_host(), orc, f"after iteration {g}")
    assert tagged, "the case never had an agent out of play when the buffer was overwritten"
    gpu.close()


def test_two_handles_of_different_lds_size_used_alternately():
    """Two live handles on the same kernel variant whose workgroups need different amounts of LDS
    (the limit on dynamic LDS is a property of the kernel, not of the handle), stepped in turn;
    and two handles that drive the same buffers in turn, with wd_invalidate_obs at each change."""
    import paper_2108_13976_amd as wd

    small = dict(num_envs=3, num_agents=40, num_taggers=4, grid_size=16, episode_length=9, seed=5)
    large = dict(num_envs=5, num_agents=900, num_taggers=90, grid_size=90, episode_length=9, seed=6)
    pairs = [(make_gpu(kw), make_oracle(kw), kw) for kw in (large, small)]
    for gpu, orc, _ in pairs:
        gpu.reset(wd.WD_RESET_ALL), orc.reset()
    for g in range(12):
        for gpu, orc, kw in reversed(pairs) if g % 2 else pairs:
            probs = probs_for_step(kw["seed"], g, kw["num_envs"], kw["num_agents"])
            gpu.iterate(upload(probs, gpu.device))
            orc.iterate(probs, g)
            assert_equal_state(gpu.to_host(), orc, f"{kw['num_agents']} agents, iteration {g}")
    for gpu, _, _ in pairs:
        gpu.close()
    # one set of buffers, two handles (full observations keep rows of agents out of play)
    kw = dict(seed=77, **EDGE["full_obs"]) if "full_obs" in EDGE else dict(num_envs=4, num_agents=24, num_taggers=6, grid_size=8, episode_length=30, seed=77, obs_mode=1)
    a, orc = make_gpu(kw), make_oracle(kw)
    b_handle = wd.wd_create(a.cfg, a.bufs)
    a.reset(wd.WD_RESET_ALL), orc.reset()
    a.torch_stream.synchronize()
    wd.wd_reset(b_handle, wd.WD_RESET_ALL)  # (same start state again; makes the second handle usable)
    for g in range(24):
        probs = probs_for_step(77, g, kw["num_envs"], kw["num_agents"])
        h = a.handle if (g // 2) % 2 == 0 else b_handle
        wd.wd_set_step(h, g)  # the other handle advanced the run (also invalidates what h knows of obs)
        wd.wd_iterate(h, upload(probs, a.device).data_ptr())
        orc.iterate(probs, g)
        assert_equal_state(a.to_host(), orc, f"shared buffers, iteration {g}")
    wd.wd_destroy(b_handle)
    a.close()


def test_two_runs_are_byte_identical():
    import paper_2108_13976_amd as wd

    cfg = CONFIGS["tag_100x50"]
    runs = []
    for _ in range(2):
        gpu = make_gpu(cfg.kwargs())
        gpu.reset(wd.WD_RESET_ALL)
        for g in range(80):
            gpu.iterate(upload(probs_for_step(cfg.seed, g, cfg.num_envs, cfg.num_agents), gpu.device))
        runs.append(gpu.to_host())
        gpu.close()
    for n in runs[0]:
        assert runs[0][n].tobytes() == runs[1][n].tobytes(), n


def test_resume_from_saved_state_and_step_counter():
    """All state lives in the caller's buffers plus the step counter: copying both resumes exactly."""
    import paper_2108_13976_amd as wd

    cfg = CONFIGS["tag_100x50"]
    a = make_gpu(cfg.kwargs())
    a.reset(wd.WD_RESET_ALL)
    probs = [upload(probs_for_step(cfg.seed, g, cfg.num_envs, cfg.num_agents), a.device) for g in range(40)]
    for g in range(20):
        a.iterate(probs[g])
    b = make_gpu(cfg.kwargs())
    b.reset(wd.WD_RESET_ALL)
    a.torch_stream.synchronize()
    for n, ten in a.tensors.items():
        b.tensors[n].copy_(ten)
    b.global_step = a.global_step
    for g in range(20, 40):
        a.iterate(probs[g])
        b.iterate(probs[g])
    sa, sb = a.to_host(), b.to_host()
    for n in sa:
        assert sa[n].tobytes() == sb[n].tobytes(), n
    a.close(), b.close()


# ---- edge cases -------------------------------------------------------------------------------------
EDGE = {
    "two_agents": dict(num_envs=70, num_agents=2, num_taggers=1, grid_size=4, episode_length=9, obs_k=1),
    "k_zero": dict(num_envs=33, num_agents=12, num_taggers=3, grid_size=7, episode_length=15, obs_k=0),
    "k_three": dict(num_envs=9, num_agents=40, num_taggers=5, grid_size=13, episode_length=30, obs_k=3),
    "k_eight": dict(num_envs=9, num_agents=40, num_taggers=5, grid_size=11, episode_length=30, obs_k=8),
    "k_three_one_workgroup": dict(num_envs=9, num_agents=70, num_taggers=8, grid_size=15, episode_length=30, obs_k=3),
    "k_eight_one_workgroup": dict(num_envs=9, num_agents=70, num_taggers=8, grid_size=13, episode_length=30, obs_k=8),
    "k_twelve": dict(num_envs=7, num_agents=60, num_taggers=6, grid_size=14, episode_length=25, obs_k=12),
    "k_sixteen_wide_keys": dict(num_envs=3, num_agents=200, num_taggers=15, grid_size=9000, episode_length=8, obs_k=16,
                                tag_r2=10**7),
    "k_seventeen": dict(num_envs=4, num_agents=30, num_taggers=4, grid_size=10, episode_length=15, obs_k=17),
    "k_thirty_three": dict(num_envs=3, num_agents=200, num_taggers=20, grid_size=25, episode_length=12, obs_k=33),
    "k_forty_nine_wide_keys": dict(num_envs=2, num_agents=120, num_taggers=10, grid_size=9000, episode_length=8, obs_k=49,
                                   tag_r2=10**7),
    "k_all_others_seventy": dict(num_envs=3, num_agents=70, num_taggers=8, grid_size=12, episode_length=20, obs_k=69),
    "k_thirty_two_one_cell": dict(num_envs=2, num_agents=50, num_taggers=5, grid_size=1, episode_length=4, obs_k=32),
    "large_env_k_ten": dict(num_envs=2, num_agents=4200, num_taggers=50, grid_size=150, episode_length=3, obs_k=10),
    "k_all_others": dict(num_envs=5, num_agents=14, num_taggers=4, grid_size=9, episode_length=25, obs_k=13),
    "one_cell_grid": dict(num_envs=4, num_agents=6, num_taggers=2, grid_size=1, episode_length=5, obs_k=4),
    "tagging_disabled": dict(num_envs=6, num_agents=30, num_taggers=6, grid_size=6, episode_length=12, obs_k=4, tag_r2=-1),
    "whole_grid_in_range": dict(num_envs=6, num_agents=30, num_taggers=6, grid_size=9, episode_length=12, obs_k=4, tag_r2=10**9),
    "wide_radius": dict(num_envs=6, num_agents=90, num_taggers=3, grid_size=40, episode_length=40, obs_k=4, tag_r2=50),
    "sparse_big_grid": dict(num_envs=3, num_agents=20, num_taggers=2, grid_size=3000, episode_length=10, obs_k=4),
    "wide_keys": dict(num_envs=3, num_agents=300, num_taggers=20, grid_size=20000, episode_length=10, obs_k=4, tag_r2=10**8),
    "thousand_agents_dense": dict(num_envs=3, num_agents=1000, num_taggers=100, grid_size=12, episode_length=20, obs_k=4, tag_r2=0),
    "thousand_twenty_four": dict(num_envs=2, num_agents=1024, num_taggers=1, grid_size=64, episode_length=8, obs_k=2),
    "many_agents_one_team": dict(num_envs=2, num_agents=1500, num_taggers=50, grid_size=90, episode_length=8, obs_k=4),
    "large_env_narrow_keys": dict(num_envs=2, num_agents=8192, num_taggers=700, grid_size=100, episode_length=4, obs_k=4),
    # 8000 agents on a 500 grid: (distance, index) keys need exactly 32 bits (dead mark in the index array)
    "large_env_full_32_bit_keys": dict(num_envs=2, num_agents=8000, num_taggers=900, grid_size=500, episode_length=3, obs_k=3,
                                       tag_r2=8),
    # 5000 agents on a 1000 grid: 64-bit keys
    "large_env_wide_keys": dict(num_envs=2, num_agents=5000, num_taggers=600, grid_size=1000, episode_length=3, obs_k=4,
                                tag_r2=18),
    "large_env_k_zero": dict(num_envs=2, num_agents=4100, num_taggers=40, grid_size=200, episode_length=3, obs_k=0),
    # every runner is tagged in the first step: rows of zeros for all of them, then the reset
    "large_env_all_tagged_at_once": dict(num_envs=2, num_agents=4500, num_taggers=30, grid_size=60, episode_length=5,
                                         obs_k=4, tag_r2=10**7),
    "large_env_k_two": dict(num_envs=2, num_agents=6001, num_taggers=3, grid_size=300, episode_length=3, obs_k=2),
    "full_obs_tiny": dict(num_envs=40, num_agents=5, num_taggers=1, grid_size=6, episode_length=12, obs_mode=1),
    "full_obs_fifty": dict(num_envs=9, num_agents=50, num_taggers=10, grid_size=20, episode_length=30, obs_mode=1),
    "full_obs_odd_count": dict(num_envs=5, num_agents=131, num_taggers=7, grid_size=15, episode_length=10, obs_mode=1),
    # N % 4 == 0 and at least one wave per env: rows leave as aligned 16-byte pieces
    "full_obs_one_wave": dict(num_envs=3, num_agents=132, num_taggers=9, grid_size=12, episode_length=8, obs_mode=1),
    "full_obs_two_waves": dict(num_envs=3, num_agents=260, num_taggers=20, grid_size=16, episode_length=6, obs_mode=1),
    "full_obs_thousand": dict(num_envs=2, num_agents=1000, num_taggers=100, grid_size=30, episode_length=5, obs_mode=1),
    # enough envs for the one-workgroup-per-env layout at these agent counts (fewer envs run in the
    # large-env pair of kernels): 256, 512 and 1024 threads per env
    "five_hundred_twenty_many_envs": dict(num_envs=170, num_agents=520, num_taggers=40, grid_size=60, episode_length=6),
    "fifteen_hundred_many_envs": dict(num_envs=460, num_agents=1500, num_taggers=100, grid_size=120, episode_length=3),
    "three_thousand_many_envs": dict(num_envs=910, num_agents=3000, num_taggers=250, grid_size=170, episode_length=2),
    "thirty_five_hundred_many_envs": dict(num_envs=455, num_agents=3500, num_taggers=300, grid_size=180, episode_length=2),
    # the any-K variant and full observations in 512-thread workgroups
    "k_seventeen_fifteen_hundred": dict(num_envs=3, num_agents=1500, num_taggers=90, grid_size=70, episode_length=4, obs_k=17),
    "full_obs_twelve_hundred": dict(num_envs=2, num_agents=1200, num_taggers=100, grid_size=40, episode_length=3, obs_mode=1),
    # K = 1, 2, 3 compiled in (one env per 256-thread workgroup, whole 64-row chunks and a ragged last one)
    "k_one_thousand_agents": dict(num_envs=310, num_agents=1000, num_taggers=100, grid_size=100, episode_length=3, obs_k=1),
    "k_two_thousand_agents": dict(num_envs=305, num_agents=1000, num_taggers=100, grid_size=90, episode_length=3, obs_k=2),
    "k_three_six_hundred_agents": dict(num_envs=190, num_agents=600, num_taggers=50, grid_size=70, episode_length=4, obs_k=3),
    "k_one_packed_envs": dict(num_envs=37, num_agents=90, num_taggers=9, grid_size=30, episode_length=8, obs_k=1),
    "k_two_odd_agent_count": dict(num_envs=21, num_agents=101, num_taggers=9, grid_size=30, episode_length=8, obs_k=2),
    # K = 5 .. 8 compiled in
    "k_six_thousand_agents": dict(num_envs=305, num_agents=1000, num_taggers=100, grid_size=100, episode_length=3, obs_k=6),
    "k_seven_packed_envs": dict(num_envs=30, num_agents=120, num_taggers=12, grid_size=25, episode_length=8, obs_k=7),
    "k_five_odd_agent_count": dict(num_envs=11, num_agents=203, num_taggers=20, grid_size=45, episode_length=8, obs_k=5),
    # the large-env pair at the smallest agent count it is chosen for
    "large_env_pair_smallest": dict(num_envs=3, num_agents=384, num_taggers=30, grid_size=50, episode_length=10, obs_k=16),
    "odd_rewards": dict(num_envs=12, num_agents=25, num_taggers=5, grid_size=8, episode_length=20, obs_k=2,
                        tag_reward=0.3, tag_penalty=-2.5),
    # The large-env layout has two forms: few envs get the step spread over a workgroup per 512 agents (the
    # large_env_* cases above), more envs or more than 2048 taggers the step with one workgroup per env.
    "large_env_one_workgroup_step": dict(num_envs=60, num_agents=2100, num_taggers=100, grid_size=150, episode_length=3),
    "large_env_many_taggers": dict(num_envs=2, num_agents=5000, num_taggers=2500, grid_size=140, episode_length=3),
    # spread step: a tag radius of many cells (one coarse cell of the taggers' table per reach), a group of four
    # that holds taggers and runners with more than one group of taggers per lane, a crowded grid
    "large_env_wide_reach": dict(num_envs=2, num_agents=4200, num_taggers=20, grid_size=300, episode_length=4, tag_r2=900),
    "large_env_odd_taggers": dict(num_envs=3, num_agents=4099, num_taggers=513, grid_size=210, episode_length=4, obs_k=4,
                                  tag_r2=5),
    "large_env_crowded": dict(num_envs=2, num_agents=4200, num_taggers=100, grid_size=16, episode_length=6, tag_r2=0),
    # a wave per env (at most 64 agents, 8192 envs, a grid of 4096 cells a side, K <= 16), and the general kernel just beyond
    "wave_full": dict(num_envs=7, num_agents=64, num_taggers=63, grid_size=30, episode_length=12, obs_k=8),
    "wave_sixty_four_runners": dict(num_envs=5, num_agents=64, num_taggers=1, grid_size=9, episode_length=30, obs_k=4, tag_r2=1),
    "wave_two_agents": dict(num_envs=9, num_agents=2, num_taggers=1, grid_size=3, episode_length=6, obs_k=1),
    "wave_k_zero": dict(num_envs=5, num_agents=33, num_taggers=5, grid_size=20, episode_length=9, obs_k=0),
    "wave_k_seven": dict(num_envs=5, num_agents=9, num_taggers=2, grid_size=7, episode_length=9, obs_k=7),
    "k_twelve_small_layout": dict(num_envs=5, num_agents=100, num_taggers=9, grid_size=20, episode_length=9, obs_k=12),
    "wave_k_sixteen": dict(num_envs=6, num_agents=40, num_taggers=5, grid_size=12, episode_length=9, obs_k=16),
    "wave_k_nine_few_agents": dict(num_envs=6, num_agents=10, num_taggers=2, grid_size=5, episode_length=9, obs_k=9),
    "wave_grid_limit": dict(num_envs=3, num_agents=40, num_taggers=4, grid_size=4096, episode_length=8, obs_k=4, tag_r2=10**6),
    "wave_batch_limit": dict(num_envs=8192, num_agents=6, num_taggers=2, grid_size=8, episode_length=6, obs_k=4),
    "beyond_wave_batch": dict(num_envs=8193, num_agents=6, num_taggers=2, grid_size=8, episode_length=6, obs_k=4),
    "beyond_wave_agents": dict(num_envs=300, num_agents=65, num_taggers=7, grid_size=25, episode_length=10, obs_k=4),
    "beyond_wave_grid": dict(num_envs=3, num_agents=40, num_taggers=4, grid_size=4097, episode_length=8, obs_k=4, tag_r2=10**6),
    "many_small_envs_k_two": dict(num_envs=8500, num_agents=30, num_taggers=3, grid_size=12, episode_length=8, obs_k=2),
    "large_env_two_thousand": dict(num_envs=4, num_agents=2000, num_taggers=2000 - 1, grid_size=64, episode_length=3, obs_k=8),
}


@pytest.mark.parametrize("name", list(EDGE))
@pytest.mark.parametrize("fused", [False, True], ids=["separate", "fused"])
def test_edge_case(name, fused):
    kw = dict(seed=77, **EDGE[name])
    steps = min(3 * kw["episode_length"], 60)
    work = kw["num_envs"] * kw["num_agents"] ** 2  # pairs the oracle looks at per step
    lockstep(kw, steps, 77, fused=fused, sharded=0 if work < 5e7 else min(16, kw["num_envs"]))
