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
