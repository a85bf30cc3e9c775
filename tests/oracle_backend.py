"""Backend over the C++ oracle for the hand-trace runner."""
import numpy as np

from oracle import tag_oracle


class OracleTraceEnv:
    float_tol = 0.0  # the oracle must hit the hand-computed float32 values exactly

    def __init__(self, config):
        c = dict(config)
        self.o = tag_oracle.TagOracle(1, c["num_agents"], c["num_taggers"], c["grid_size"], c["episode_length"],
                                      seed=0, tag_r2=c["tag_r2"], obs_k=c["obs_k"], obs_mode=c.get("obs_mode", 0))
        self.o.reset(tag_oracle.RESET_ALL)

    def set_start(self, start):
        start = np.array(start, dtype=np.int32)
        self.o.pos_x0[0], self.o.pos_y0[0] = start[:, 0], start[:, 1]
        self.o.done[0] = 1
        self.o.reset(tag_oracle.RESET_DONE)

    def step(self, actions):
        self.o.action[0] = np.array(actions, dtype=np.int32)
        self.o.step()

    def reset_done(self):
        self.o.reset(tag_oracle.RESET_DONE)

    def get(self, name):
        return getattr(self.o, name)[0].copy()


class CTagOracleTraceEnv:
    """Backend over the continuous-Tag oracle for ``ctrace_runner``."""
    float_tol = 0.0  # the oracle must hit the hand-computed float32 values exactly

    def __init__(self, config):
        from oracle import ctag_oracle
        self.mod = ctag_oracle
        c = dict(config)
        self.o = ctag_oracle.CTagOracle(1, c["num_agents"], c["num_taggers"], c["episode_length"], seed=0,
                                        world_size=c["world_size"], num_headings=c["num_headings"],
                                        accel=c["accel"], max_speed_tagger=c["max_speed_tagger"],
                                        max_speed_runner=c["max_speed_runner"], tag_r2=c["tag_r2"],
                                        obs_k=c["obs_k"])
        self.o.reset(ctag_oracle.RESET_ALL)

    def set_start(self, start):
        self.o.x0[0] = np.array([r[0] for r in start], dtype=np.float32)
        self.o.y0[0] = np.array([r[1] for r in start], dtype=np.float32)
        self.o.h0[0] = np.array([r[2] for r in start], dtype=np.int32)
        self.o.done[0] = 1
        self.o.reset(self.mod.RESET_DONE)

    def step(self, actions):
        self.o.action[0] = np.array(actions, dtype=np.int32)
        self.o.step()

    def reset_done(self):
        self.o.reset(self.mod.RESET_DONE)

    def get(self, name):
        return getattr(self.o, name)[0].copy()
