"""The five Tag workloads, three continuous-Tag workloads and the stand-in policy output.

The paper benchmarks its discrete Tag environment (Sec. 5.1) with 5 to 1000 agents
and up to 2000 environments (Sec. 5.3); its environment source and trained policies
are not available, so these seeded synthetic inputs stand in: start positions are
drawn by the method itself from the seed, and the per-agent action probabilities a
policy network would produce are float32 softmax of 5 i.i.d. N(0,1) logits, redrawn
every step.
"""
from dataclasses import dataclass, asdict

import numpy as np

NUM_ACTIONS = 5


@dataclass(frozen=True)
class TagConfig:
    name: str
    num_envs: int
    num_agents: int
    num_taggers: int
    grid_size: int
    episode_length: int
    seed: int
    tag_r2: int = 2
    obs_mode: int = 0
    obs_k: int = 4
    tag_reward: float = 1.0
    tag_penalty: float = -1.0

    def kwargs(self):
        d = asdict(self)
        d.pop("name")
        return d

    @property
    def obs_dim(self):
        return 5 + 4 * (self.obs_k if self.obs_mode == 0 else self.num_agents)


CONFIGS = {
    "tag_10x5": TagConfig("tag_10x5", 10, 5, 1, 20, 100, 0),
    "tag_100x50": TagConfig("tag_100x50", 100, 50, 10, 50, 500, 1),
    "tag_2000x1000": TagConfig("tag_2000x1000", 2000, 1000, 100, 100, 500, 2),
    "tag_20000x100": TagConfig("tag_20000x100", 20000, 100, 10, 40, 200, 3),
    "tag_10x8192": TagConfig("tag_10x8192", 10, 8192, 512, 512, 200, 4),
}


@dataclass(frozen=True)
class CTagConfig:
    """Continuous Tag (paper Sec. 5.1, second variant): sizes and the constants this build chose."""
    name: str
    num_envs: int
    num_agents: int
    num_taggers: int
    episode_length: int
    seed: int
    world_size: float = 20.0
    num_headings: int = 16
    accel: float = 0.25
    max_speed_tagger: float = 1.0
    max_speed_runner: float = 0.75
    tag_r2: float = 1.0
    obs_k: int = 4
    tag_reward: float = 1.0
    tag_penalty: float = -1.0

    def kwargs(self):
        d = asdict(self)
        d.pop("name")
        return d

    @property
    def obs_dim(self):
        return 8 + 6 * self.obs_k


# 2000 x 5 is the shape of the paper's continuous-Tag throughput figure (Sec. 5.3); 5 taggers and
# 100 runners on a 20 x 20 world is the shape of its snapshot figure
CTAG_CONFIGS = {
    "ctag_10x5": CTagConfig("ctag_10x5", 10, 5, 1, 100, 10),
    "ctag_2000x5": CTagConfig("ctag_2000x5", 2000, 5, 1, 500, 11),
    "ctag_2000x105": CTagConfig("ctag_2000x105", 2000, 105, 5, 500, 12),
}


def ctag_probs_for_step(seed, g, num_envs, num_agents, env_lo=0, env_hi=None):
    """Host probabilities [E, N, 2, 5] float32 for global step ``g`` of a continuous-Tag workload:
    one softmax per agent and action category (acceleration, turn)."""
    flat = probs_for_step(seed, g, num_envs, 2 * num_agents, env_lo, env_hi)
    return flat.reshape(flat.shape[0], num_agents, 2, NUM_ACTIONS)


def _softmax32(logits):
    z = logits - logits.max(axis=-1, keepdims=True)
    ez = np.exp(z, dtype=np.float32)
    return (ez / ez.sum(axis=-1, keepdims=True, dtype=np.float32)).astype(np.float32)


_ENV_BLOCK = 64  # envs drawn from one generator


def probs_for_step(seed, g, num_envs, num_agents, env_lo=0, env_hi=None):
    """Host probabilities [E, N, 5] float32 for global step ``g``.

    Each block of 64 envs depends only on (seed, g, block id), so any env slice of
    the full workload can be produced on its own and equals that slice of the whole.
    """
    env_hi = num_envs if env_hi is None else env_hi
    out = np.empty((env_hi - env_lo, num_agents, NUM_ACTIONS), dtype=np.float32)
    for b in range(env_lo // _ENV_BLOCK, (env_hi + _ENV_BLOCK - 1) // _ENV_BLOCK):
        rng = np.random.Generator(np.random.Philox(key=[int(seed) & (2**64 - 1), (int(g) << 32) | b]))
        block = _softmax32(rng.standard_normal((_ENV_BLOCK, num_agents, NUM_ACTIONS), dtype=np.float32))
        lo, hi = max(env_lo, b * _ENV_BLOCK), min(env_hi, (b + 1) * _ENV_BLOCK)
        out[lo - env_lo:hi - env_lo] = block[lo - b * _ENV_BLOCK:hi - b * _ENV_BLOCK]
    return out


def device_probs_ring(seed, ring_len, num_envs, num_agents, device):
    """A ring of ``ring_len`` steps of probabilities generated on the device.

    Same distribution as :func:`probs_for_step` (not the same bits); used where the
    probabilities only have to be resident before a timed region starts.
    """
    import torch

    gen = torch.Generator(device=device)
    gen.manual_seed(int(seed))
    logits = torch.randn((ring_len, num_envs, num_agents, NUM_ACTIONS), generator=gen,
                         device=device, dtype=torch.float32)
    return torch.softmax(logits, dim=-1).contiguous()
