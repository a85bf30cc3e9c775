"""Pins of the continuous-Tag oracle (readings C1-C14; paper Sec. 5.1, continuous variant of Tag).

The paper fixes none of the numbers, so the oracle is pinned to what the readings and the
mathematics fix: hand traces with exactly representable values, closed forms of the heading table
and of straight-line motion, the table's symmetries, statements of the start state and of the
draws in terms of the already pinned random-block and sampler routines, an independent Python
statement of the rules, and invariants over seeded roll-outs.
"""
from decimal import Decimal, getcontext
from fractions import Fraction

import numpy as np
import pytest

import cpyref
import ctrace_runner
from oracle import ctag_oracle, tag_oracle
from oracle_backend import CTagOracleTraceEnv
from workloads import CTAG_CONFIGS, ctag_probs_for_step

TRACES = ctrace_runner.load_traces()


@pytest.mark.parametrize("trace", TRACES, ids=[t["name"].split()[0] for t in TRACES])
def test_hand_trace(trace):
    ctrace_runner.run_trace(CTagOracleTraceEnv, trace)


# ---------------------------------------------------------------- C5: heading table
@pytest.mark.parametrize("H", [4, 8, 12, 16, 32, 360])
def test_heading_table_symmetries_and_axes(H):
    cx, cy = ctag_oracle.heading_table(H)
    q = H // 4
    assert (cx[0], cy[0]) == (1.0, 0.0) and (cx[q], cy[q]) == (0.0, 1.0)
    assert (cx[2 * q], cy[2 * q]) == (-1.0, 0.0) and (cx[3 * q], cy[3 * q]) == (0.0, -1.0)
    for h in range(H):
        assert cx[(h + H // 2) % H] == -cx[h] and cy[(h + H // 2) % H] == -cy[h]   # half turn
        assert cx[(h + q) % H] == -cy[h] and cy[(h + q) % H] == cx[h]               # quarter turn
        assert cx[(-h) % H] == cx[h] and cy[(-h) % H] == -cy[h]                      # mirror in the x axis
        assert cx[(q - h) % H] == cy[h]                                               # mirror in the diagonal
        assert abs(float(cx[h]) ** 2 + float(cy[h]) ** 2 - 1.0) < 2e-7
        assert not np.signbit(cx[h]) or cx[h] != 0  # zeros are +0
        assert not np.signbit(cy[h]) or cy[h] != 0
    # strictly decreasing cosine over the first quadrant: no entry misplaced
    assert all(cx[h] > cx[h + 1] for h in range(q))


def test_heading_table_closed_forms():
    getcontext().prec = 60
    two, three = Decimal(2), Decimal(3)
    f32 = lambda d: np.float32(float(d))  # noqa: E731  (float() of a 60-digit decimal is correctly rounded; then to float32)
    cx, cy = ctag_oracle.heading_table(8)
    assert cx[1] == cy[1] == f32(two.sqrt() / 2)
    cx, cy = ctag_oracle.heading_table(12)
    assert cx[1] == f32(three.sqrt() / 2) and cy[1] == np.float32(0.5)          # 30 degrees
    assert cx[2] == np.float32(0.5) and cy[2] == f32(three.sqrt() / 2)          # 60 degrees, by reflection
    cx, cy = ctag_oracle.heading_table(16)
    assert cx[1] == f32((two + two.sqrt()).sqrt() / 2) and cy[1] == f32((two - two.sqrt()).sqrt() / 2)  # 22.5 degrees
    assert cx[2] == cy[2] == f32(two.sqrt() / 2)
    assert cx[3] == cy[1] and cy[3] == cx[1]
    assert cx[7] == -cx[1] and cy[7] == cy[1]


def test_heading_table_rejects_bad_sizes():
    for H in (0, 3, 6, 10, -4):
        with pytest.raises(ValueError):
            ctag_oracle.heading_table(H)


# ---------------------------------------------------------------- C2: start state
def test_start_state_statement_and_spread():
    cfg = CTAG_CONFIGS["ctag_2000x5"]
    o = ctag_oracle.CTagOracle(400, 5, 1, 500, seed=cfg.seed, env_offset=7)
    o.reset()
    L = np.float32(o.cfg.world_size)
    for e, i in [(0, 0), (3, 4), (399, 2), (123, 1)]:
        w = tag_oracle.random_block(cfg.seed, 7 + e, i, 0, 3)
        assert o.x0[e, i] == np.float32(w[0] >> 8) * np.float32(2.0 ** -24) * L
        assert o.y0[e, i] == np.float32(w[1] >> 8) * np.float32(2.0 ** -24) * L
        assert o.h0[e, i] == (w[2] * 16) >> 32
    assert np.array_equal(o.x, o.x0) and np.array_equal(o.y, o.y0) and np.array_equal(o.h, o.h0)
    assert not o.v.any() and o.live.all() and not o.t.any() and not o.done.any()
    assert (o.n_live_runners == 4).all()
    assert (o.x0 >= 0).all() and (o.x0 < L).all() and (o.y0 >= 0).all() and (o.y0 < L).all()
    # chi-square of the 16 headings and of 10 x 10 position bins over 2000 agents
    n = o.h0.size
    counts = np.bincount(o.h0.ravel(), minlength=16)
    assert ((counts - n / 16) ** 2 / (n / 16)).sum() < 45.0      # 15 dof, p ~ 1e-4
    bins = (np.floor(o.x0 / 2).astype(int) * 10 + np.floor(o.y0 / 2).astype(int)).ravel()
    counts = np.bincount(bins, minlength=100)
    assert ((counts - n / 100) ** 2 / (n / 100)).sum() < 160.0   # 99 dof, p ~ 1e-4


# ---------------------------------------------------------------- C3: draws
def test_draws_statement():
    E, N, seed = 6, 5, 99
    o = ctag_oracle.CTagOracle(E, N, 1, 50, seed=seed, env_offset=3)
    o.reset()
    for g in (0, 1, 2**32 + 5):
        probs = ctag_probs_for_step(seed, g % 1000, E, N)
        o.sample(probs, g)
        for e in range(E):
            for i in range(N):
                w = tag_oracle.random_block(seed, 3 + e, i, g, 2)
                for c in range(2):
                    want = tag_oracle.sample_from_u(probs[e, i, c], tag_oracle.uniform_from_word(w[c]))
                    assert o.action[e, i, c] == want
    # a one-hot distribution is drawn with certainty, whatever the random word
    probs = np.zeros((E, N, 2, 5), dtype=np.float32)
    probs[..., 0, 4] = 1.0
    probs[..., 1, 1] = 1.0
    o.sample(probs, 77)
    assert (o.action[..., 0] == 4).all() and (o.action[..., 1] == 1).all()


# ---------------------------------------------------------------- C6, C7: closed form of straight-line motion
def test_straight_line_closed_form():
    """From rest, heading +x, one acceleration step per iteration: v_k = min(k a, vmax) and
    x_k = x_0 + sum v_k, exactly (a = 1/4, vmax = 1, start on a multiple of 1/4: every value is
    a dyadic rational that float32 holds)."""
    o = ctag_oracle.CTagOracle(1, 2, 1, 100, seed=0, world_size=64.0, num_headings=8, accel=0.25,
                               max_speed_tagger=1.0, max_speed_runner=0.75, tag_r2=-1.0, obs_k=1)
    o.reset()
    o.x0[0], o.y0[0], o.h0[0] = [1.25, 60.0], [3.0, 40.0], [0, 4]
    o.done[0] = 1
    o.reset(ctag_oracle.RESET_DONE)
    x_t, v_t, x_r, v_r = Fraction(5, 4), Fraction(0), Fraction(60), Fraction(0)
    for k in range(1, 30):
        o.action[0] = [[3, 2], [3, 2]]
        o.step()
        v_t = min(v_t + Fraction(1, 4), Fraction(1))
        v_r = min(v_r + Fraction(1, 4), Fraction(3, 4))
        x_t += v_t
        x_r -= v_r
        assert Fraction(float(o.v[0, 0])) == v_t and Fraction(float(o.x[0, 0])) == x_t
        assert Fraction(float(o.v[0, 1])) == v_r and Fraction(float(o.x[0, 1])) == x_r
        assert o.y[0, 0] == 3.0 and o.y[0, 1] == 40.0 and o.t[0] == k
        assert o.obs[0, 0, 8] == np.float32(float(x_r - x_t)) / np.float32(64.0)
        assert o.obs[0, 0, 10] == np.float32(float(-v_r))


# ---------------------------------------------------------------- independent Python statement
PYREF_CASES = [
    dict(E=3, N=2, N_tag=1, T=12, L=3.0, H=8, K=1, tag_r2=0.5, seed=21),
    dict(E=3, N=5, N_tag=1, T=40, L=4.0, H=16, K=4, tag_r2=1.0, seed=22),
    dict(E=2, N=7, N_tag=3, T=25, L=5.0, H=12, K=2, tag_r2=1.5, seed=23),
    dict(E=2, N=6, N_tag=2, T=30, L=2.5, H=4, K=5, tag_r2=0.3, seed=24),
    dict(E=2, N=4, N_tag=1, T=15, L=6.0, H=360, K=0, tag_r2=2.0, seed=25),
    dict(E=2, N=9, N_tag=2, T=20, L=3.5, H=32, K=8, tag_r2=-1.0, seed=26),
]


@pytest.mark.parametrize("case", PYREF_CASES, ids=[f"seed{c['seed']}" for c in PYREF_CASES])
def test_against_python_statement(case):
    c = case
    o = ctag_oracle.CTagOracle(c["E"], c["N"], c["N_tag"], c["T"], seed=c["seed"], world_size=c["L"],
                               num_headings=c["H"], accel=0.25, max_speed_tagger=1.0, max_speed_runner=0.75,
                               tag_r2=c["tag_r2"], obs_k=c["K"], env_offset=5)
    o.reset()
    refs = [cpyref.PyCTagEnv(5 + e, c["N"], c["N_tag"], c["T"], c["seed"], L=c["L"], H=c["H"], tag_r2=c["tag_r2"],
                             K=c["K"]) for e in range(c["E"])]

    def compare(where):
        for e, r in enumerate(refs):
            for name, want in (("x", r.x), ("y", r.y), ("v", r.v), ("h", r.h), ("live", r.live)):
                assert np.array_equal(getattr(o, name)[e], np.array(want, dtype=getattr(o, name).dtype)), (where, e, name)
            assert (o.t[e], o.done[e], o.n_live_runners[e], o.tags_step[e]) == (r.t, r.done, r.n_live, r.tags_step), (where, e)
            assert np.array_equal(o.obs[e], r.obs()), (where, e, "obs")

    compare("reset")
    resets = 0
    for g in range(3 * c["T"]):
        probs = ctag_probs_for_step(c["seed"], g, c["E"], c["N"])
        o.sample(probs, g)
        o.step()
        for e, r in enumerate(refs):
            r.sample(probs[e], g)
            r.step()
            assert np.array_equal(o.action[e], np.array(r.action, dtype=np.int32))
            assert np.array_equal(o.reward[e], np.array(r.reward, dtype=np.float32))
        compare(f"step {g}")
        resets += int(o.done.sum())
        o.reset(ctag_oracle.RESET_DONE)
        for r in refs:
            r.reset_if_done()
        compare(f"reset after step {g}")
    assert resets >= 2 * c["E"]


# ---------------------------------------------------------------- invariants over seeded roll-outs
@pytest.mark.parametrize("name,envs,iters", [("ctag_10x5", 10, 250), ("ctag_2000x105", 6, 120)])
def test_invariants(name, envs, iters):
    cfg = CTAG_CONFIGS[name]
    kw = cfg.kwargs()
    kw["num_envs"] = envs
    o = ctag_oracle.CTagOracle(**kw)
    o.reset()
    N, N_tag, L = cfg.num_agents, cfg.num_taggers, np.float32(cfg.world_size)
    vmax = np.where(np.arange(N) < N_tag, np.float32(cfg.max_speed_tagger), np.float32(cfg.max_speed_runner))
    total_tags = 0
    for g in range(iters):
        before = {n: getattr(o, n).copy() for n in ("x", "y", "v", "h", "live", "t", "done", "n_live_runners")}
        o.sample(ctag_probs_for_step(cfg.seed, g, envs, N), g)
        assert ((o.action >= 0) & (o.action <= 4)).all()
        o.step()
        assert (o.x >= 0).all() and (o.x <= L).all() and (o.y >= 0).all() and (o.y <= L).all()
        assert (o.v >= 0).all() and (o.v <= vmax[None, :]).all()
        assert (o.h >= 0).all() and (o.h < cfg.num_headings).all()
        assert (o.live[:, :N_tag] == 1).all() and (o.live <= before["live"]).all()
        frozen = before["live"] == 0
        for n in ("x", "y", "v", "h"):
            assert np.array_equal(getattr(o, n)[frozen], before[n][frozen])
        # a step is never longer than the speed before clamping could be: at most the top speed
        dist = np.hypot(o.x.astype(np.float64) - before["x"], o.y.astype(np.float64) - before["y"])
        assert (dist <= vmax[None, :] + 1e-5).all()  # (positions near 20 carry 2e-6 of rounding)
        tags = before["live"].sum(axis=1) - o.live.sum(axis=1)
        assert np.array_equal(tags, o.tags_step) and np.array_equal(o.n_live_runners, before["n_live_runners"] - tags)
        assert np.array_equal(o.n_live_runners, o.live[:, N_tag:].sum(axis=1))
        assert np.allclose(o.reward[:, :N_tag].sum(axis=1), tags * cfg.tag_reward)
        assert np.allclose(o.reward[:, N_tag:].sum(axis=1), tags * cfg.tag_penalty)
        assert np.array_equal(o.t, before["t"] + 1)
        assert np.array_equal(o.done, ((o.n_live_runners == 0) | (o.t >= cfg.episode_length)).astype(np.int32))
        # rows: own features, and neighbour slots in order of distance, all of live agents
        assert np.array_equal(o.obs[..., 6], o.live.astype(np.float32))
        assert np.array_equal(o.obs[..., 2], o.v)
        K = cfg.obs_k
        slots = o.obs[..., 8:].reshape(envs, N, K, 6)
        d = np.hypot(slots[..., 0].astype(np.float64), slots[..., 1].astype(np.float64))
        used = slots[..., 5] == 1
        assert ((np.diff(d, axis=2) >= -1e-7) | ~used[..., 1:]).all()
        n_used = used.sum(axis=2)
        assert np.array_equal(n_used, np.where(o.live == 1, np.minimum(K, o.live.sum(axis=1)[:, None] - 1), 0))
        total_tags += int(tags.sum())
        o.reset(ctag_oracle.RESET_DONE)
    assert total_tags > 0


def test_env_slices_reproduce_the_whole():
    cfg = CTAG_CONFIGS["ctag_10x5"]
    whole = ctag_oracle.CTagOracle(**cfg.kwargs())
    kw = cfg.kwargs()
    kw["num_envs"] = 4
    part = ctag_oracle.CTagOracle(env_offset=3, **kw)
    whole.reset()
    part.reset()
    for g in range(130):
        whole.iterate(ctag_probs_for_step(cfg.seed, g, 10, 5), g)
        part.iterate(ctag_probs_for_step(cfg.seed, g, 10, 5, 3, 7), g)
    for name in ("x", "y", "v", "h", "live", "action", "reward", "obs", "t", "done", "n_live_runners", "tags_step"):
        assert np.array_equal(getattr(whole, name)[3:7], getattr(part, name)), name
