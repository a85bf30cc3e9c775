"""ctypes front end of the C++ continuous-Tag oracle (``wdc_oracle.cpp``).

TEST INFRASTRUCTURE ONLY.  Holds the state arrays as numpy arrays and forwards
every call to the oracle library; no arithmetic of the method lives here.
"""
import ctypes

import numpy as np

from . import tag_oracle

RESET_ALL = 0
RESET_DONE = 1

_i32p = ctypes.POINTER(ctypes.c_int32)
_f32p = ctypes.POINTER(ctypes.c_float)


class _Config(ctypes.Structure):
    _fields_ = [
        ("num_envs", ctypes.c_int32),
        ("env_offset", ctypes.c_int32),
        ("num_agents", ctypes.c_int32),
        ("num_taggers", ctypes.c_int32),
        ("num_headings", ctypes.c_int32),
        ("episode_length", ctypes.c_int32),
        ("obs_k", ctypes.c_int32),
        ("world_size", ctypes.c_float),
        ("accel", ctypes.c_float),
        ("max_speed_tagger", ctypes.c_float),
        ("max_speed_runner", ctypes.c_float),
        ("tag_r2", ctypes.c_float),
        ("tag_reward", ctypes.c_float),
        ("tag_penalty", ctypes.c_float),
        ("seed", ctypes.c_uint64),
    ]


# (name, dtype, shape suffix after [E, N]) in the order of wdco_state
_AGENT_ARRAYS = (("x", np.float32), ("y", np.float32), ("v", np.float32), ("h", np.int32),
                 ("x0", np.float32), ("y0", np.float32), ("h0", np.int32), ("live", np.int32))
_STATE_ENV = ("t", "done", "n_live_runners", "tags_step")


class _State(ctypes.Structure):
    _fields_ = ([(n, _f32p if dt is np.float32 else _i32p) for n, dt in _AGENT_ARRAYS]
                + [("action", _i32p), ("reward", _f32p), ("obs", _f32p)]
                + [(n, _i32p) for n in _STATE_ENV])


_ready = False


def load():
    global _ready
    lib = tag_oracle.load()
    if not _ready:
        lib.wdco_obs_dim.argtypes = [ctypes.POINTER(_Config)]
        lib.wdco_obs_dim.restype = ctypes.c_int32
        lib.wdco_heading_table.argtypes = [ctypes.c_int32, _f32p, _f32p]
        lib.wdco_reset.argtypes = [ctypes.POINTER(_Config), ctypes.POINTER(_State), ctypes.c_int]
        lib.wdco_sample.argtypes = [ctypes.POINTER(_Config), ctypes.POINTER(_State), _f32p, ctypes.c_uint64]
        lib.wdco_step.argtypes = [ctypes.POINTER(_Config), ctypes.POINTER(_State)]
        lib.wdco_observe.argtypes = [ctypes.POINTER(_Config), ctypes.POINTER(_State), ctypes.c_int32]
        for name in ("wdco_heading_table", "wdco_reset", "wdco_sample", "wdco_step", "wdco_observe"):
            getattr(lib, name).restype = ctypes.c_int
        _ready = True
    return lib


def heading_table(num_headings):
    cx = np.zeros(num_headings, dtype=np.float32)
    cy = np.zeros(num_headings, dtype=np.float32)
    rc = load().wdco_heading_table(int(num_headings), cx.ctypes.data_as(_f32p), cy.ctypes.data_as(_f32p))
    if rc != 0:
        raise ValueError("invalid number of headings")
    return cx, cy


class CTagOracle:
    """State arrays of E continuous-Tag environments plus the calls that advance them."""

    def __init__(self, num_envs, num_agents, num_taggers, episode_length, seed=0, world_size=20.0,
                 num_headings=16, accel=0.25, max_speed_tagger=1.0, max_speed_runner=0.75, tag_r2=1.0,
                 obs_k=4, tag_reward=1.0, tag_penalty=-1.0, env_offset=0, _arrays=None):
        self.lib = load()
        self.cfg = _Config(num_envs, env_offset, num_agents, num_taggers, num_headings, episode_length, obs_k,
                           world_size, accel, max_speed_tagger, max_speed_runner, tag_r2, tag_reward,
                           tag_penalty, seed)
        D = 8 + 6 * obs_k
        self.E, self.N, self.D = num_envs, num_agents, D
        if _arrays is None:
            E, N = num_envs, num_agents
            _arrays = {n: np.zeros((E, N), dtype=dt) for n, dt in _AGENT_ARRAYS}
            _arrays["action"] = np.zeros((E, N, 2), dtype=np.int32)
            _arrays["reward"] = np.zeros((E, N), dtype=np.float32)
            _arrays["obs"] = np.zeros((E, N, D), dtype=np.float32)
            _arrays.update({n: np.zeros((E,), dtype=np.int32) for n in _STATE_ENV})
        self.arrays = _arrays
        for name, arr in _arrays.items():
            assert arr.flags["C_CONTIGUOUS"]
            setattr(self, name, arr)

        def ptr(n):
            a = _arrays[n]
            return a.ctypes.data_as(_f32p if a.dtype == np.float32 else _i32p)

        self.state = _State(*[ptr(n) for n, _ in _AGENT_ARRAYS], ptr("action"), ptr("reward"), ptr("obs"),
                            *[ptr(n) for n in _STATE_ENV])

    def shard(self, lo, hi):
        c = self.cfg
        return CTagOracle(hi - lo, c.num_agents, c.num_taggers, c.episode_length, seed=c.seed,
                          world_size=c.world_size, num_headings=c.num_headings, accel=c.accel,
                          max_speed_tagger=c.max_speed_tagger, max_speed_runner=c.max_speed_runner,
                          tag_r2=c.tag_r2, obs_k=c.obs_k, tag_reward=c.tag_reward, tag_penalty=c.tag_penalty,
                          env_offset=c.env_offset + lo, _arrays={n: a[lo:hi] for n, a in self.arrays.items()})

    def _check(self, rc, what):
        if rc != 0:
            raise RuntimeError(f"oracle {what} failed with {rc}")

    def reset(self, mode=RESET_ALL):
        self._check(self.lib.wdco_reset(ctypes.byref(self.cfg), ctypes.byref(self.state), mode), "reset")

    def sample(self, probs, g):
        probs = np.ascontiguousarray(probs, dtype=np.float32)
        assert probs.shape == (self.E, self.N, 2, 5)
        self._check(self.lib.wdco_sample(ctypes.byref(self.cfg), ctypes.byref(self.state),
                                         probs.ctypes.data_as(_f32p), int(g)), "sample")

    def step(self):
        self._check(self.lib.wdco_step(ctypes.byref(self.cfg), ctypes.byref(self.state)), "step")

    def observe(self, e):
        self._check(self.lib.wdco_observe(ctypes.byref(self.cfg), ctypes.byref(self.state), int(e)), "observe")

    def iterate(self, probs, g):
        """One roll-out iteration in the canonical order: sample, step, reset done envs."""
        self.sample(probs, g)
        self.step()
        self.reset(RESET_DONE)
