"""The oracle against an independent brute-force statement on tiny inputs, invariants on the
small workloads, and the special cases with closed forms."""
import numpy as np
import pytest

import pyref
from invariants import check_obs_invariants, check_step_invariants
from oracle import tag_oracle
from workloads import CONFIGS, probs_for_step

STATE = ("pos_x", "pos_y", "live", "action", "reward", "obs", "t", "done", "n_live_runners", "tags_step")


def snapshot(o):
    return {n: getattr(o, n).copy() for n in STATE}


@pytest.mark.parametrize("N,n_tag,G,T,K,r2,seed", [
    (2, 1, 3, 6, 1, 2, 1), (3, 1, 4, 8, 2, 2, 2), (4, 2, 4, 10, 3, 2, 3), (5, 1, 6, 12, 4, 2, 4),
    (6, 3, 5, 9, 2, 0, 5), (7, 2, 7, 15, 6, 5, 6), (9, 4, 6, 20, 3, 1, 7), (8, 1, 12, 25, 0, 2, 8),
    (6, 2, 3, 30, 5, -1, 9), (12, 3, 9, 40, 4, 8, 10),
])
def test_against_python_brute_force(N, n_tag, G, T, K, r2, seed):
    """Full roll-outs (sample, step, reset) on random tiny envs, every array every step."""
    E = 6
    o = tag_oracle.TagOracle(E, N, n_tag, G, T, seed=seed, tag_r2=r2, obs_k=K, tag_reward=1.5, tag_penalty=-0.75)
    o.reset()
    envs = []
    for e in range(E):
        start = [pyref.start_position(seed, e, i, G) for i in range(N)]
        assert o.pos_x0[e].tolist() == [p[0] for p in start] and o.pos_y0[e].tolist() == [p[1] for p in start]
        envs.append(pyref.PyTagEnv(start, n_tag, G, T, K, r2, 1.5, -0.75))

    def compare(tag):
        for e, env in enumerate(envs):
            assert o.pos_x[e].tolist() == [p[0] for p in env.pos], tag
            assert o.pos_y[e].tolist() == [p[1] for p in env.pos], tag
            assert o.live[e].tolist() == [int(v) for v in env.live], tag
            assert (o.t[e], o.done[e], o.n_live_runners[e], o.tags_step[e]) == \
                (env.t, int(env.done), env.n_live_runners, env.tags_step), tag
            assert np.array_equal(o.obs[e], env.obs()), tag

    compare("reset")
    n_resets = 0
    for g in range(3 * T):
        probs = probs_for_step(seed, g, E, N)
        o.sample(probs, g)
        o.step()
        for e, env in enumerate(envs):
            acts = [pyref.sample_action(seed, e, i, g, probs[e, i]) for i in range(N)]
            assert o.action[e].tolist() == acts
            was_done = env.done
            env.step(acts)
            if not was_done:
                assert np.array_equal(o.reward[e], np.array(env.reward, dtype=np.float32))
        compare(f"step {g}")
        o.reset(tag_oracle.RESET_DONE)
        for env in envs:
            if env.done:
                env.restore()
                n_resets += 1
        compare(f"reset after {g}")
    assert n_resets >= E  # every roll-out crossed episode ends


def test_full_observation_mode_against_python_brute_force():
    N, n_tag, G, T, seed = 6, 2, 5, 12, 3
    o = tag_oracle.TagOracle(3, N, n_tag, G, T, seed=seed, obs_mode=1)
    o.reset()
    assert o.D == 5 + 4 * N
    envs = [pyref.PyTagEnv([pyref.start_position(seed, e, i, G) for i in range(N)], n_tag, G, T, 0, 2, obs_mode=1)
            for e in range(3)]
    for g in range(2 * T):
        for e, env in enumerate(envs):
            assert np.array_equal(o.obs[e], env.obs())
        probs = probs_for_step(seed, g, 3, N)
        o.iterate(probs, g)
        for e, env in enumerate(envs):
            env.step(o.action[e])
            if env.done:
                env.restore()


@pytest.mark.parametrize("name,steps", [("tag_10x5", 250), ("tag_100x50", 120)])
def test_invariants_on_small_workloads(name, steps):
    cfg = CONFIGS[name]
    o = tag_oracle.TagOracle(**cfg.kwargs())
    o.reset()
    check_obs_invariants(cfg, snapshot(o))
    assert (o.pos_x0 >= 0).all() and (o.pos_x0 < cfg.grid_size).all()
    total_tags = 0
    for g in range(steps):
        probs = probs_for_step(cfg.seed, g, cfg.num_envs, cfg.num_agents)
        before = snapshot(o)
        o.sample(probs, g)
        assert (o.action >= 0).all() and (o.action < 5).all()
        o.step()
        after = snapshot(o)
        check_step_invariants(cfg, before, after)
        total_tags += int(after["tags_step"].sum())
        done_before = o.done.copy()
        o.reset(tag_oracle.RESET_DONE)
        s = snapshot(o)
        assert (s["done"] == 0).all()
        rs = done_before == 1
        assert np.array_equal(s["pos_x"][rs], o.pos_x0[rs]) and (s["live"][rs] == 1).all() and (s["t"][rs] == 0).all()
        assert np.array_equal(s["reward"], after["reward"])  # reset leaves rewards alone
        for n in ("pos_x", "pos_y", "live", "t", "obs"):
            assert np.array_equal(s[n][~rs], after[n][~rs])  # other envs untouched
        check_obs_invariants(cfg, s)
    assert total_tags > 0


def test_start_positions_are_uniform_on_the_grid():
    o = tag_oracle.TagOracle(200, 100, 10, 7, 10, seed=17)
    o.reset()
    for arr in (o.pos_x0, o.pos_y0):
        counts = np.bincount(arr.ravel(), minlength=7)
        assert counts.size == 7
        chi2 = ((counts - arr.size / 7) ** 2 / (arr.size / 7)).sum()
        assert chi2 < 35  # 6 degrees of freedom
    joint = np.bincount((o.pos_x0 * 7 + o.pos_y0).ravel(), minlength=49)
    assert ((joint - 20000 / 49) ** 2 / (20000 / 49)).sum() < 110  # 48 degrees of freedom


def test_everyone_stays_then_nothing_moves_and_tags_happen_only_once():
    cfg = CONFIGS["tag_100x50"]
    o = tag_oracle.TagOracle(**cfg.kwargs())
    o.reset()
    o.action[:] = 0
    x, y = o.pos_x.copy(), o.pos_y.copy()
    o.step()
    first = o.tags_step.copy()
    # brute-force count of runners within range of some tagger at the start positions
    d2 = (x[:, 10:, None] - x[:, None, :10]) ** 2 + (y[:, 10:, None] - y[:, None, :10]) ** 2
    assert np.array_equal(first, (d2.min(axis=2) <= 2).sum(axis=1))
    for _ in range(5):
        o.step()
        assert np.array_equal(o.pos_x, x) and np.array_equal(o.pos_y, y)
        assert (o.tags_step[o.done == 0] == 0).all() and (o.reward[o.done == 0] == 0).all()


def test_tagging_disabled_means_every_episode_runs_to_the_step_limit():
    cfg = CONFIGS["tag_10x5"]
    kw = cfg.kwargs()
    kw["tag_r2"] = -1
    o = tag_oracle.TagOracle(**kw)
    o.reset()
    for g in range(2 * cfg.episode_length):
        o.sample(probs_for_step(cfg.seed, g, cfg.num_envs, cfg.num_agents), g)
        o.step()
        assert (o.tags_step == 0).all() and (o.live == 1).all() and (o.reward == 0).all()
        assert (o.done == int((g + 1) % cfg.episode_length == 0)).all()
        o.reset(tag_oracle.RESET_DONE)


def test_k_equal_all_others_is_the_sorted_live_part_of_the_full_row():
    N, n_tag, G, T, seed = 9, 3, 6, 30, 21
    part = tag_oracle.TagOracle(4, N, n_tag, G, T, seed=seed, obs_k=N - 1)
    full = tag_oracle.TagOracle(4, N, n_tag, G, T, seed=seed, obs_mode=1)
    part.reset(), full.reset()
    for g in range(20):
        probs = probs_for_step(seed, g, 4, N)
        part.sample(probs, g), full.sample(probs, g)
        part.step(), full.step()
        assert np.array_equal(part.live, full.live)
        for e in range(4):
            for i in range(N):
                f = full.obs[e, i, 5:].reshape(N, 4)
                p = part.obs[e, i, 5:].reshape(N - 1, 4)
                if not part.live[e, i]:
                    assert (p == 0).all() and (f == 0).all()
                    continue
                js = [j for j in range(N) if j != i and part.live[e, j]]
                js.sort(key=lambda j: ((part.pos_x[e, j] - part.pos_x[e, i]) ** 2 + (part.pos_y[e, j] - part.pos_y[e, i]) ** 2, j))
                assert np.array_equal(p[:len(js)], f[js]) and (p[len(js):] == 0).all()


def test_env_slices_reproduce_the_full_run():
    cfg = CONFIGS["tag_100x50"]
    full = tag_oracle.TagOracle(**cfg.kwargs())
    kw = cfg.kwargs()
    kw["num_envs"] = 7
    part = tag_oracle.TagOracle(env_offset=40, **kw)
    full.reset(), part.reset()
    for g in range(60):
        full.iterate(probs_for_step(cfg.seed, g, cfg.num_envs, cfg.num_agents), g)
        part.iterate(probs_for_step(cfg.seed, g, cfg.num_envs, cfg.num_agents, 40, 47), g)
        for n in STATE:
            assert np.array_equal(getattr(full, n)[40:47], getattr(part, n)), n


def test_sharded_threads_equal_the_single_thread_run():
    cfg = CONFIGS["tag_100x50"]
    a = tag_oracle.TagOracle(**cfg.kwargs())
    b = tag_oracle.TagOracle(**cfg.kwargs())
    a.reset()
    tag_oracle.run_sharded(b, lambda sh: sh.reset(), threads=4)
    for g in range(30):
        probs = probs_for_step(cfg.seed, g, cfg.num_envs, cfg.num_agents)
        a.iterate(probs, g)
        lo = {}
        used = tag_oracle.run_sharded(b, lambda sh: sh.iterate(probs[sh.cfg.env_offset:sh.cfg.env_offset + sh.E], g), threads=4)
        assert used == 4
    for n in STATE:
        assert np.array_equal(getattr(a, n), getattr(b, n)), n


def test_bad_arguments_are_rejected():
    with pytest.raises(ValueError):
        tag_oracle.TagOracle(1, 1, 1, 5, 5)          # fewer than two agents
    with pytest.raises(ValueError):
        tag_oracle.TagOracle(1, 4, 4, 5, 5)          # no runner
    with pytest.raises(ValueError):
        tag_oracle.TagOracle(1, 4, 1, 5, 5, obs_k=4)  # K above N - 1
    with pytest.raises(ValueError):
        tag_oracle.TagOracle(1, 4, 1, 40000, 5)      # grid too large
