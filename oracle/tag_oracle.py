"""ctypes front end of the C++ Tag oracle (``wd_oracle.cpp``).

TEST INFRASTRUCTURE ONLY.  Holds the state arrays as numpy arrays and forwards
every call to the oracle library; no arithmetic of the method lives here.
"""
import ctypes
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

from . import build as _build

RESET_ALL = 0
RESET_DONE = 1

_i32p = ctypes.POINTER(ctypes.c_int32)
_f32p = ctypes.POINTER(ctypes.c_float)
_u32p = ctypes.POINTER(ctypes.c_uint32)


class _Config(ctypes.Structure):
    _fields_ = [
        ("num_envs", ctypes.c_int32),
        ("env_offset", ctypes.c_int32),
        ("num_agents", ctypes.c_int32),
        ("num_taggers", ctypes.c_int32),
        ("grid_size", ctypes.c_int32),
        ("episode_length", ctypes.c_int32),
        ("tag_r2", ctypes.c_int32),
        ("obs_mode", ctypes.c_int32),
        ("obs_k", ctypes.c_int32),
        ("tag_reward", ctypes.c_float),
        ("tag_penalty", ctypes.c_float),
        ("seed", ctypes.c_uint64),
    ]


_STATE_I32 = ("pos_x", "pos_y", "pos_x0", "pos_y0", "live", "action")
_STATE_ENV = ("t", "done", "n_live_runners", "tags_step")


class _State(ctypes.Structure):
    _fields_ = (
        [(n, _i32p) for n in _STATE_I32]
        + [("reward", _f32p), ("obs", _f32p)]
        + [(n, _i32p) for n in _STATE_ENV]
    )


_lib = None


def load():
    """Load (building it first if it is missing or stale) the oracle library."""
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(_build.build(force=False))
        lib.wdo_philox4x32_10.argtypes = [_u32p, _u32p, _u32p]
        lib.wdo_philox4x32_10.restype = None
        lib.wdo_random_block.argtypes = [ctypes.c_uint64, ctypes.c_uint32, ctypes.c_uint32,
                                         ctypes.c_uint64, ctypes.c_uint32, _u32p]
        lib.wdo_random_block.restype = None
        lib.wdo_uniform_from_word.argtypes = [ctypes.c_uint32]
        lib.wdo_uniform_from_word.restype = ctypes.c_float
        lib.wdo_sample_from_u.argtypes = [_f32p, ctypes.c_int32, ctypes.c_float]
        lib.wdo_sample_from_u.restype = ctypes.c_int32
        lib.wdo_obs_dim.argtypes = [ctypes.POINTER(_Config)]
        lib.wdo_obs_dim.restype = ctypes.c_int32
        for name in ("wdo_reset",):
            getattr(lib, name).argtypes = [ctypes.POINTER(_Config), ctypes.POINTER(_State), ctypes.c_int]
        lib.wdo_sample.argtypes = [ctypes.POINTER(_Config), ctypes.POINTER(_State), _f32p, ctypes.c_uint64]
        lib.wdo_step.argtypes = [ctypes.POINTER(_Config), ctypes.POINTER(_State)]
        lib.wdo_observe.argtypes = [ctypes.POINTER(_Config), ctypes.POINTER(_State), ctypes.c_int32]
        for name in ("wdo_reset", "wdo_sample", "wdo_step", "wdo_observe"):
            getattr(lib, name).restype = ctypes.c_int
        _lib = lib
    return _lib


def philox4x32_10(ctr, key):
    c = (ctypes.c_uint32 * 4)(*[int(v) & 0xFFFFFFFF for v in ctr])
    k = (ctypes.c_uint32 * 2)(*[int(v) & 0xFFFFFFFF for v in key])
    out = (ctypes.c_uint32 * 4)()
    load().wdo_philox4x32_10(c, k, out)
    return [int(v) for v in out]


def random_block(seed, env, agent, g, stream):
    out = (ctypes.c_uint32 * 4)()
    load().wdo_random_block(int(seed), int(env), int(agent), int(g), int(stream), out)
    return [int(v) for v in out]


def uniform_from_word(w):
    return float(load().wdo_uniform_from_word(int(w) & 0xFFFFFFFF))


def sample_from_u(p, u):
    p = np.ascontiguousarray(p, dtype=np.float32)
    return int(load().wdo_sample_from_u(p.ctypes.data_as(_f32p), int(p.size), ctypes.c_float(u)))


class TagOracle:
    """State arrays of E environments plus the calls that advance them.

    ``env_offset`` is the global id of local env 0: an oracle built on a slice of
    the envs reproduces exactly those envs of the full run.
    """

    def __init__(self, num_envs, num_agents, num_taggers, grid_size, episode_length,
                 seed=0, tag_r2=2, obs_mode=0, obs_k=4, tag_reward=1.0, tag_penalty=-1.0,
                 env_offset=0, _arrays=None):
        self.lib = load()
        self.cfg = _Config(num_envs, env_offset, num_agents, num_taggers, grid_size,
                           episode_length, tag_r2, obs_mode, obs_k, tag_reward, tag_penalty, seed)
        D = self.lib.wdo_obs_dim(ctypes.byref(self.cfg))
        if D < 0:
            raise ValueError("invalid Tag configuration")
        self.E, self.N, self.D = num_envs, num_agents, D
        if _arrays is None:
            E, N = num_envs, num_agents
            _arrays = {n: np.zeros((E, N), dtype=np.int32) for n in _STATE_I32}
            _arrays["reward"] = np.zeros((E, N), dtype=np.float32)
            _arrays["obs"] = np.zeros((E, N, D), dtype=np.float32)
            _arrays.update({n: np.zeros((E,), dtype=np.int32) for n in _STATE_ENV})
        self.arrays = _arrays
        for name, arr in _arrays.items():
            assert arr.flags["C_CONTIGUOUS"]
            setattr(self, name, arr)
        self.state = _State(
            *[_arrays[n].ctypes.data_as(_i32p) for n in _STATE_I32],
            _arrays["reward"].ctypes.data_as(_f32p), _arrays["obs"].ctypes.data_as(_f32p),
            *[_arrays[n].ctypes.data_as(_i32p) for n in _STATE_ENV])

    # -- env-sliced views, sharing memory with this oracle --------------------
    def shard(self, lo, hi):
        c = self.cfg
        return TagOracle(hi - lo, c.num_agents, c.num_taggers, c.grid_size, c.episode_length,
                         seed=c.seed, tag_r2=c.tag_r2, obs_mode=c.obs_mode, obs_k=c.obs_k,
                         tag_reward=c.tag_reward, tag_penalty=c.tag_penalty,
                         env_offset=c.env_offset + lo,
                         _arrays={n: a[lo:hi] for n, a in self.arrays.items()})

    def _check(self, rc, what):
        if rc != 0:
            raise RuntimeError(f"oracle {what} failed with {rc}")

    def reset(self, mode=RESET_ALL):
        self._check(self.lib.wdo_reset(ctypes.byref(self.cfg), ctypes.byref(self.state), mode), "reset")

    def sample(self, probs, g):
        probs = np.ascontiguousarray(probs, dtype=np.float32)
        assert probs.shape == (self.E, self.N, 5)
        self._check(self.lib.wdo_sample(ctypes.byref(self.cfg), ctypes.byref(self.state),
                                        probs.ctypes.data_as(_f32p), int(g)), "sample")

    def step(self):
        self._check(self.lib.wdo_step(ctypes.byref(self.cfg), ctypes.byref(self.state)), "step")

    def observe(self, e):
        self._check(self.lib.wdo_observe(ctypes.byref(self.cfg), ctypes.byref(self.state), int(e)), "observe")

    def iterate(self, probs, g):
        """One roll-out iteration in the canonical order: sample, step, reset done envs."""
        self.sample(probs, g)
        self.step()
        self.reset(RESET_DONE)


def run_sharded(oracle, fn, threads=None):
    """Apply ``fn(shard)`` to disjoint env slices of ``oracle``, one thread per slice.

    Envs are independent and the random blocks are keyed by global env id, so the
    result equals ``fn(oracle)``; each thread runs the single-threaded oracle.
    Returns the number of threads used.
    """
    threads = max(1, min(int(threads or (os.cpu_count() or 1)), oracle.E))
    bounds = np.linspace(0, oracle.E, threads + 1).astype(int)
    shards = [oracle.shard(int(a), int(b)) for a, b in zip(bounds[:-1], bounds[1:]) if b > a]
    with ThreadPoolExecutor(max_workers=len(shards)) as pool:
        list(pool.map(fn, shards))
    return len(shards)
