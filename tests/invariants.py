"""Invariants of the Tag rules that hold at any size; shared by oracle and GPU tests.

They follow from the paper's prose (Sec. 5.1: positions on the grid, one cell per move,
tagged runners leave, one reward per tag, termination rule) and the observation layout.
"""
import numpy as np


def check_step_invariants(cfg, before, after, float_tol=0.0):
    """``before``/``after``: dicts of numpy arrays around ONE step (no reset in between).
    ``cfg``: object with num_agents, num_taggers, grid_size, episode_length, obs_k, tag_reward,
    tag_penalty."""
    N, n_tag, G, T = cfg.num_agents, cfg.num_taggers, cfg.grid_size, cfg.episode_length
    stepped = before["done"] == 0
    x0, y0, x1, y1 = before["pos_x"], before["pos_y"], after["pos_x"], after["pos_y"]
    assert (x1 >= 0).all() and (x1 < G).all() and (y1 >= 0).all() and (y1 < G).all()
    disp = np.abs(x1 - x0) + np.abs(y1 - y0)
    assert (disp <= 1).all()
    assert (disp[before["live"] == 0] == 0).all()          # agents out of play do not move
    assert (disp[~stepped] == 0).all()                      # done envs are frozen
    assert (after["live"][:, :n_tag] == 1).all()            # taggers always live
    assert (after["live"] <= before["live"]).all()          # nobody comes back within an episode
    assert np.array_equal(after["n_live_runners"], after["live"][:, n_tag:].sum(axis=1))
    tags = before["n_live_runners"] - after["n_live_runners"]
    assert np.array_equal(tags[stepped], after["tags_step"][stepped])
    assert (tags[~stepped] == 0).all()
    r = after["reward"].astype(np.float64)
    assert np.allclose(r[stepped][:, :n_tag].sum(axis=1), after["tags_step"][stepped] * cfg.tag_reward)
    assert np.allclose(r[stepped][:, n_tag:].sum(axis=1), after["tags_step"][stepped] * cfg.tag_penalty)
    newly = (before["live"] == 1) & (after["live"] == 0)
    assert (after["reward"][newly] == np.float32(cfg.tag_penalty)).all()
    assert (after["t"][stepped] == before["t"][stepped] + 1).all()
    assert (after["t"] <= T).all()
    want_done = (after["n_live_runners"] == 0) | (after["t"] >= T)
    assert np.array_equal(after["done"][stepped] == 1, want_done[stepped])
    check_obs_invariants(cfg, after, float_tol)


def check_obs_invariants(cfg, s, float_tol=0.0):
    """Observation rows against the state they were computed from (partial mode)."""
    N, n_tag, G, T, K = cfg.num_agents, cfg.num_taggers, cfg.grid_size, cfg.episode_length, cfg.obs_k
    obs = s["obs"]
    E = obs.shape[0]
    assert np.abs(obs).max() <= 1.0
    def close(a, b):
        return (np.abs(a.astype(np.float64) - b.astype(np.float64)) <= float_tol).all()

    assert close(obs[..., 0], (s["pos_x"].astype(np.float32) / np.float32(G)))
    assert close(obs[..., 1], (s["pos_y"].astype(np.float32) / np.float32(G)))
    assert np.array_equal(obs[..., 2], np.broadcast_to((np.arange(N) < n_tag).astype(np.float32), (E, N)))
    assert np.array_equal(obs[..., 3], s["live"].astype(np.float32))
    assert close(obs[..., 4], np.broadcast_to((s["t"].astype(np.float32) / np.float32(T))[:, None], (E, N)))
    if K == 0:
        return
    slots = obs[..., 5:].reshape(E, N, K, 4)
    valid = slots[..., 3]
    assert set(np.unique(valid)).issubset({0.0, 1.0})
    n_live = s["live"].sum(axis=1)
    want_valid = np.where(s["live"] == 1, np.minimum(K, n_live[:, None] - 1), 0)
    assert np.array_equal(valid.sum(axis=-1).astype(np.int64), want_valid)
    assert (np.diff(valid, axis=-1) <= 0).all()              # valid slots come first
    assert (slots[valid == 0] == 0).all()
    # distances do not decrease along the slots
    dx = np.rint(slots[..., 0].astype(np.float64) * G)
    dy = np.rint(slots[..., 1].astype(np.float64) * G)
    d2 = np.where(valid == 1, dx * dx + dy * dy, 1e18)
    assert (np.diff(d2, axis=-1) >= 0).all()
