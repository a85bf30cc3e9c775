"""Runs the hand traces of ``tests/golden/ctag_hand_traces.json`` (continuous Tag) against a backend.

A backend offers ``make(config) -> env`` with ``env.set_start(rows of [x0, y0, h0])`` (puts the
single env in that start state through the reset-of-done-envs path), ``env.step(actions)`` with
rows of [acceleration level, turn level], ``env.reset_done()`` and ``env.get(name)`` for the state
arrays of env 0; ``env.float_tol`` bounds the difference allowed on ``obs``.
"""
import json
import os
import struct

import numpy as np

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "ctag_hand_traces.json")
EXACT_FLOATS = ("x", "y", "v", "reward")


def load_traces():
    with open(GOLDEN) as f:
        return json.load(f)["traces"]


def _value(v):
    if isinstance(v, str):
        if v.startswith("0x"):
            return np.frombuffer(struct.pack("<I", int(v, 16)), dtype=np.float32)[0]
        a, b = v.split("/")
        return np.float32(float(a)) / np.float32(float(b))
    return np.float32(v)


def _check(env, expect, where):
    for name, want in expect.items():
        got = env.get(name)
        if name == "obs":
            want_arr = np.array([[_value(v) for v in row] for row in want], dtype=np.float32)
            assert got.shape == want_arr.shape, f"{where}: obs shape {got.shape} != {want_arr.shape}"
            err = np.abs(got.astype(np.float64) - want_arr.astype(np.float64)).max()
            assert err <= env.float_tol, f"{where}: obs\n{got}\n!=\n{want_arr}"
        elif name in EXACT_FLOATS:
            want_arr = np.array([_value(v) for v in want], dtype=np.float32)
            assert np.array_equal(got, want_arr), f"{where}: {name} {got.tolist()} != {want_arr.tolist()}"
        else:
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
