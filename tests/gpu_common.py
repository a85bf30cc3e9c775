"""Helpers of the GPU parity tests: build the HIP path and the oracle on the same
configuration and compare their state arrays element by element."""
import numpy as np

INT_ARRAYS = ("pos_x", "pos_y", "pos_x0", "pos_y0", "live", "action", "t", "done", "n_live_runners", "tags_step")
FLOAT_ARRAYS = ("reward", "obs")
FLOAT_TOL = 1e-6  # absolute, float32 rewards and observations (spec tolerance)


def make_gpu(kw):
    import torch
    import paper_2108_13976_amd as wd

    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return wd.TagEnvs(**kw)


def make_oracle(kw, env_lo=0, env_hi=None):
    from oracle import tag_oracle

    kw = dict(kw)
    E = kw["num_envs"]
    env_hi = E if env_hi is None else env_hi
    base = kw.pop("env_offset", 0)
    kw["num_envs"] = env_hi - env_lo
    return tag_oracle.TagOracle(env_offset=base + env_lo, **kw)


def assert_equal_state(gpu_state, oracle, where, env_lo=0, env_hi=None, names=None):
    """Bit-exact on integer arrays, <= FLOAT_TOL absolute on float arrays."""
    env_hi = env_lo + oracle.E if env_hi is None else env_hi
    for n in (names or INT_ARRAYS + FLOAT_ARRAYS):
        got = gpu_state[n][env_lo:env_hi]
        want = getattr(oracle, n)
        assert got.shape == want.shape, f"{where}: {n} shape {got.shape} vs {want.shape}"
        if n in INT_ARRAYS:
            if not np.array_equal(got, want):
                bad = np.argwhere(got != want)
                raise AssertionError(f"{where}: {n} differs at {len(bad)} places, first {bad[:5].tolist()}: "
                                     f"gpu {got[tuple(bad[0])]} oracle {want[tuple(bad[0])]}")
        else:
            err = np.abs(got.astype(np.float64) - want.astype(np.float64))
            if not (err <= FLOAT_TOL).all():
                bad = np.argwhere(err > FLOAT_TOL)
                raise AssertionError(f"{where}: {n} off by up to {err.max():.3g} at {len(bad)} places, first "
                                     f"{bad[:5].tolist()}: gpu {got[tuple(bad[0])]} oracle {want[tuple(bad[0])]}")


def upload(probs, device):
    import torch

    return torch.from_numpy(np.ascontiguousarray(probs)).to(device)
