"""Runs the hand traces of ``tests/golden/tag_hand_traces.json`` against a backend.

A backend offers: ``make(config) -> env`` with ``env.set_start(list of (x, y))`` (puts the
single env in that start state through the reset-of-done-envs path), ``env.step(actions)``,
``env.reset_done()`` and ``env.get(name) -> numpy array`` for the state arrays of env 0.
"""
import json
import os

import numpy as np

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "tag_hand_traces.json")


def load_traces():
    with open(GOLDEN) as f:
        return json.load(f)["traces"]


def _value(v):
    if isinstance(v, str):
        a, b = v.split("/")
        return np.float32(int(a)) / np.float32(int(b))
    return np.float32(v)


def _check(env, expect, where):
    for name, want in expect.items():
        if name == "pos":
            got = np.stack([env.get("pos_x"), env.get("pos_y")], axis=-1)
            assert got.tolist() == want, f"{where}: pos {got.tolist()} != {want}"
        elif name in ("obs", "reward"):
            want_arr = np.array([[_value(v) for v in row] for row in want] if name == "obs"
                                else [_value(v) for v in want], dtype=np.float32)
            got = env.get(name)
            assert got.shape == want_arr.shape, f"{where}: {name} shape {got.shape}"
            assert np.abs(got.astype(np.float64) - want_arr.astype(np.float64)).max() <= env.float_tol, \
                f"{where}: {name}\n{got}\n!=\n{want_arr}"
        else:
            got = env.get(name)
            want_arr = np.array(want, dtype=np.int32).reshape(got.shape)
            assert np.array_equal(got, want_arr), f"{where}: {name} {got.tolist()} != {want}"


def run_trace(backend_make, trace):
    env = backend_make(trace["config"])
    env.set_start(trace["start"])
    if "expect_after_reset" in trace:
        _check(env, trace["expect_after_reset"], trace["name"] + " / after reset")
    for n, ev in enumerate(trace["events"]):
        if "actions" in ev:
            env.step(ev["actions"])
        elif ev.get("reset_done"):
            env.reset_done()
        _check(env, ev.get("expect", {}), f"{trace['name']} / event {n}")
