"""wd_iterate_static: the entry point that allocates nothing (its large-env work tables live in a static
device array) against wd_iterate on a handle, through the C ABI, element by element."""
import numpy as np
import pytest

import paper_2108_13976_amd as wd
from paper_2108_13976_amd import binding
from workloads import probs_for_step

from gpu_common import FLOAT_ARRAYS, INT_ARRAYS, upload

pytestmark = pytest.mark.gpu

# large-env layout (work tables in device memory): few envs of many agents; the second, smaller one runs
# after the first on the same static array
LARGE = dict(num_envs=6, num_agents=2000, num_taggers=150, grid_size=300, episode_length=6, seed=11)
SMALLER = dict(num_envs=3, num_agents=700, num_taggers=60, grid_size=120, episode_length=5, seed=12)
# small layout (no work tables at all)
PLAIN = dict(num_envs=40, num_agents=90, num_taggers=9, grid_size=30, episode_length=7, seed=13)
# envs that fit a wave (the kernel with a wave per env; no work tables either)
WAVE = dict(num_envs=33, num_agents=20, num_taggers=4, grid_size=9, episode_length=6, seed=14)


def run_both(kw, iterations):
    """The same iterations through a handle (wd_iterate) and through wd_iterate_static on a copy of the state."""
    import torch

    a = wd.TagEnvs(device="cuda:0", **kw)
    b = wd.TagEnvs(device="cuda:0", **kw)  # only its buffers and config are used
    a.reset(wd.WD_RESET_ALL)
    a.torch_stream.synchronize()
    for n in binding.BUFFER_NAMES:
        b.tensors[n].copy_(a.tensors[n])
    for g in range(iterations):
        probs = upload(probs_for_step(kw["seed"], g, kw["num_envs"], kw["num_agents"]), a.device)
        a.iterate(probs)
        wd.wd_iterate_static(b.cfg, b.bufs, probs.data_ptr(), g)
        torch.cuda.synchronize()
        got, want = {n: t.cpu().numpy() for n, t in b.tensors.items()}, a.to_host()
        for n in INT_ARRAYS:
            assert np.array_equal(got[n], want[n]), f"iteration {g}: {n}"
        for n in FLOAT_ARRAYS:
            assert np.abs(got[n].astype(np.float64) - want[n].astype(np.float64)).max() <= 1e-6, f"iteration {g}: {n}"
    a.close()
    b.close()


def test_static_entry_point_equals_wd_iterate_two_calls_in_a_row():
    # crosses episode ends (T = 6, 5), so resets of done envs are inside
    run_both(LARGE, 14)
    run_both(SMALLER, 12)  # smaller input on the same static array, which still holds the first run's tables
    run_both(PLAIN, 16)
    run_both(WAVE, 14)
