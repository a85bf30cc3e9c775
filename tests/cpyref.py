"""An independent pure-Python statement of continuous Tag (readings C1-C14), one env at a time,
every float32 operation written out with numpy float32 scalars.  Used to cross-check the C++ oracle
on tiny configurations; it shares nothing with it but the pinned random-block and sampler routines.
"""
import math

import numpy as np

from oracle import tag_oracle

F = np.float32


def heading_table(H):
    """C5 by its geometric meaning: directions at multiples of 360/H degrees, built from the first
    octant by reflection about the diagonal and quarter turns."""
    q = H // 4
    out = []
    for h in range(H):
        k, r = divmod(h, q)
        mirrored = 2 * r > q
        rr = q - r if mirrored else r
        c, s = F(math.cos(2.0 * math.pi * rr / H)), F(math.sin(2.0 * math.pi * rr / H))
        if 2 * rr == q:
            s = c
        if mirrored:
            c, s = s, c
        for _ in range(k):  # a quarter turn to the left: (c, s) -> (-s, c)
            c, s = F(-s), c
        out.append((c + F(0.0), s + F(0.0)))  # -0 + 0 = +0
    return out


class PyCTagEnv:
    def __init__(self, env_id, N, N_tag, T, seed, L=20.0, H=16, accel=0.25, vmax_t=1.0, vmax_r=0.75, tag_r2=1.0,
                 K=4, tag_reward=1.0, tag_penalty=-1.0):
        self.env_id, self.N, self.N_tag, self.T, self.seed = env_id, N, N_tag, T, seed
        self.L, self.H, self.accel, self.vmax = F(L), H, F(accel), (F(vmax_t), F(vmax_r))
        self.tag_r2, self.K, self.tag_reward, self.tag_penalty = F(tag_r2), K, F(tag_reward), F(tag_penalty)
        self.table = heading_table(H)
        self.start = []
        for i in range(N):
            w = tag_oracle.random_block(seed, env_id, i, 0, 3)
            u0, u1 = F(w[0] >> 8) * F(2.0 ** -24), F(w[1] >> 8) * F(2.0 ** -24)
            self.start.append((u0 * self.L, u1 * self.L, (w[2] * H) >> 32))
        self.reward = [F(0.0)] * N
        self.action = [(0, 0)] * N
        self.restore()

    def restore(self):
        self.x = [s[0] for s in self.start]
        self.y = [s[1] for s in self.start]
        self.h = [s[2] for s in self.start]
        self.v = [F(0.0)] * self.N
        self.live = [1] * self.N
        self.t, self.done, self.n_live, self.tags_step = 0, 0, self.N - self.N_tag, 0

    def sample(self, probs, g):
        self.action = []
        for i in range(self.N):
            w = tag_oracle.random_block(self.seed, self.env_id, i, g, 2)
            self.action.append(tuple(tag_oracle.sample_from_u(probs[i][c], float(F(w[c] >> 8) * F(2.0 ** -24)))
                                     for c in range(2)))

    def d2(self, a, b):
        dx, dy = self.x[a] - self.x[b], self.y[a] - self.y[b]
        return F(dx * dx) + F(dy * dy)

    def step(self):
        if self.done:
            return
        for i in range(self.N):
            if not self.live[i]:
                continue
            s_acc, s_turn = self.action[i][0] - 2, self.action[i][1] - 2
            self.h[i] = (self.h[i] + s_turn) % self.H
            v = self.v[i] + F(F(s_acc) * self.accel)
            vmax = self.vmax[0] if i < self.N_tag else self.vmax[1]
            v = F(0.0) if v < 0 else v
            v = vmax if v > vmax else v
            c, s = self.table[self.h[i]]
            x, y = self.x[i] + F(v * c), self.y[i] + F(v * s)
            cx_, cy_ = min(max(x, F(0.0)), self.L), min(max(y, F(0.0)), self.L)
            if cx_ != x or cy_ != y:
                v = F(0.0)
            self.x[i], self.y[i], self.v[i] = cx_, cy_, v
        credits, tagged = [0] * self.N_tag, []
        if self.tag_r2 >= 0:
            for r in range(self.N_tag, self.N):
                if self.live[r]:
                    best = min((self.d2(r, t), t) for t in range(self.N_tag))
                    if best[0] <= self.tag_r2:
                        tagged.append(r)
                        credits[best[1]] += 1
        for r in tagged:
            self.live[r] = 0
        self.reward = [F(credits[i]) * self.tag_reward if i < self.N_tag else
                       (self.tag_penalty if i in tagged else F(0.0)) for i in range(self.N)]
        self.t += 1
        self.n_live -= len(tagged)
        self.tags_step = len(tagged)
        self.done = int(self.n_live == 0 or self.t >= self.T)

    def reset_if_done(self):
        if self.done:
            self.restore()

    def obs(self):
        rows = []
        for i in range(self.N):
            c, s = self.table[self.h[i]]
            row = [self.x[i] / self.L, self.y[i] / self.L, self.v[i], c, s, F(i < self.N_tag), F(self.live[i]),
                   F(self.t) / F(self.T)]
            near = sorted((self.d2(j, i), j) for j in range(self.N) if j != i and self.live[j]) if self.live[i] else []
            for k in range(self.K):
                if k < len(near):
                    j = near[k][1]
                    cj, sj = self.table[self.h[j]]
                    row += [(self.x[j] - self.x[i]) / self.L, (self.y[j] - self.y[i]) / self.L,
                            F(self.v[j] * cj), F(self.v[j] * sj), F(j < self.N_tag), F(1.0)]
                else:
                    row += [F(0.0)] * 6
            rows.append(row)
        return np.array(rows, dtype=np.float32)
