"""Pins for the oracle's sampler: closed forms and distribution."""
import numpy as np

import pyref
from oracle import tag_oracle
from workloads import probs_for_step


def test_inverse_cdf_closed_forms(oracle_lib):
    p = np.array([0.1, 0.2, 0.3, 0.4, 0.0], dtype=np.float32)
    assert oracle_lib.sample_from_u(p, 0.05) == 0
    assert oracle_lib.sample_from_u(p, float(np.float32(0.1))) == 1  # strict "<": u equal to the first partial sum
    assert oracle_lib.sample_from_u(p, 0.29) == 1
    assert oracle_lib.sample_from_u(p, 0.95) == 3
    assert oracle_lib.sample_from_u(p, 0.0) == 0
    # partial sums that stay below u fall through to the last action
    assert oracle_lib.sample_from_u(np.array([0.1, 0.1, 0.1, 0.1, 0.1], dtype=np.float32), 0.9) == 4
    # a zero-probability action is never chosen while the sums reach u
    q = np.array([0.0, 0.5, 0.0, 0.5, 0.0], dtype=np.float32)
    assert oracle_lib.sample_from_u(q, 0.0) == 1
    assert oracle_lib.sample_from_u(q, 0.5) == 3
    # NaN probabilities never satisfy the comparison
    assert oracle_lib.sample_from_u(np.full(5, np.nan, dtype=np.float32), 0.3) == 4


def test_partial_sums_are_float32_left_to_right(oracle_lib):
    # (2^-24 + 1) rounds to 1 in float32 when added in this order, so u = 1 - 2^-24 < 1 picks
    # action 1; a float64 or reordered sum would behave differently on the reversed vector.
    tiny = np.float32(2.0 ** -25)
    p = np.array([tiny, 1.0, 0.0, 0.0, 0.0], dtype=np.float32)
    u = float(np.float32(1.0) - np.float32(2.0 ** -24))
    assert oracle_lib.sample_from_u(p, u) == 1
    a, b, c = np.float32(0.5), np.float32(2.0 ** -25), np.float32(2.0 ** -25)
    # 0.5 + 2^-25 rounds back to 0.5, twice: the running float32 sum never exceeds 0.5,
    # whereas float64 accumulation would reach 0.5 + 2^-24 > u.
    p = np.array([a, b, c, 0.0, 0.25], dtype=np.float32)
    u = 0.5
    assert oracle_lib.sample_from_u(p, u) == 4


def test_one_hot_probabilities_pick_that_action(oracle_lib):
    o = tag_oracle.TagOracle(3, 6, 2, 8, 10, seed=5)
    o.reset()
    probs = np.zeros((3, 6, 5), dtype=np.float32)
    want = np.arange(18).reshape(3, 6) % 5
    for e in range(3):
        for i in range(6):
            probs[e, i, want[e, i]] = 1.0
    for g in range(4):
        o.sample(probs, g)
        assert np.array_equal(o.action, want)


def test_sample_matches_python_statement_and_uses_env_offset(oracle_lib):
    E, N, seed = 4, 7, 42
    o = tag_oracle.TagOracle(E, N, 2, 9, 10, seed=seed)
    o.reset()
    for g in (0, 1, 2**32 + 3):
        probs = probs_for_step(seed, g % 1000, E, N)
        o.sample(probs, g)
        for e in range(E):
            for i in range(N):
                assert o.action[e, i] == pyref.sample_action(seed, e, i, g, probs[e, i])
        sh = tag_oracle.TagOracle(2, N, 2, 9, 10, seed=seed, env_offset=2)
        sh.reset()
        sh.sample(probs[2:4], g)
        assert np.array_equal(sh.action, o.action[2:4])


def test_frequencies_follow_the_probabilities(oracle_lib):
    E, N = 50, 40
    p = np.array([0.05, 0.15, 0.4, 0.3, 0.1], dtype=np.float32)
    probs = np.broadcast_to(p, (E, N, 5)).copy()
    o = tag_oracle.TagOracle(E, N, 1, 10, 10, seed=99)
    o.reset()
    counts = np.zeros(5)
    steps = 500
    for g in range(steps):
        o.sample(probs, g)
        counts += np.bincount(o.action.ravel(), minlength=5)
    n = E * N * steps  # 1e6 draws
    chi2 = ((counts - n * p) ** 2 / (n * p)).sum()
    assert chi2 < 30  # 4 degrees of freedom; P(chi2 > 30) ~ 5e-6
