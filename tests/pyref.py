"""An independent, pure-Python statement of the Tag rules for tiny inputs.

Written from the rules text (paper Sec. 5.1 plus this build's readings of what it
leaves open), in a different style from the C++ oracle (per-agent records, tagger-side
bookkeeping, full sorts, exact integer arithmetic; big-int Philox), so that a slip in
either shows up as a disagreement.  Only the tests import it.
"""
import numpy as np

M0, M1 = 0xD2511F53, 0xCD9E8D57
W0, W1 = 0x9E3779B9, 0xBB67AE85
MASK = 0xFFFFFFFF


def philox4x32_10(ctr, key):
    c = [int(v) & MASK for v in ctr]
    k = [int(v) & MASK for v in key]
    for _ in range(10):
        p0, p1 = M0 * c[0], M1 * c[2]
        c = [((p1 >> 32) ^ c[1] ^ k[0]) & MASK, p1 & MASK, ((p0 >> 32) ^ c[3] ^ k[1]) & MASK, p0 & MASK]
        k = [(k[0] + W0) & MASK, (k[1] + W1) & MASK]
    return c


def random_block(seed, env, index, g, stream):
    return philox4x32_10([env, index, g & MASK, (stream & 0xFF) | ((g >> 32) << 8)], [seed & MASK, seed >> 32])


def start_position(seed, env, agent, G):
    w = random_block(seed, env, agent, 0, 1)
    return (w[0] * G) >> 32, (w[1] * G) >> 32


def sample_action(seed, env, agent, g, p):
    w = random_block(seed, env, agent // 4, g, 0)  # four consecutive agents share a block
    u = np.float32(w[agent % 4] >> 8) * np.float32(2.0 ** -24)
    c = np.float32(0.0)
    for a in range(len(p)):
        c = np.float32(c + np.float32(p[a]))
        if u < c:
            return a
    return len(p) - 1


DELTA = {0: (0, 0), 1: (0, 1), 2: (0, -1), 3: (-1, 0), 4: (1, 0)}


def f32div(a, b):
    return np.float32(a) / np.float32(b)


class PyTagEnv:
    """One environment."""

    def __init__(self, start, num_taggers, G, T, K, tag_r2, tag_reward=1.0, tag_penalty=-1.0, obs_mode=0):
        self.start = [tuple(p) for p in start]
        self.N, self.n_tag, self.G, self.T, self.K = len(start), num_taggers, G, T, K
        self.tag_r2, self.tag_reward, self.tag_penalty, self.obs_mode = tag_r2, tag_reward, tag_penalty, obs_mode
        self.reward = [np.float32(0)] * self.N
        self.restore()

    def restore(self):
        self.pos = list(self.start)
        self.live = [True] * self.N
        self.t, self.done, self.tags_step = 0, False, 0
        self.n_live_runners = self.N - self.n_tag

    def step(self, actions):
        if self.done:
            return
        G = self.G
        for i in range(self.N):
            if self.live[i]:
                dx, dy = DELTA.get(int(actions[i]), (0, 0))
                x, y = self.pos[i]
                self.pos[i] = (min(G - 1, max(0, x + dx)), min(G - 1, max(0, y + dy)))
        # tagger-side bookkeeping: every tagger lists the runners in its range, then each
        # such runner picks among the taggers that listed it
        claims = {}
        if self.tag_r2 >= 0:
            for q in range(self.n_tag):
                for r in range(self.n_tag, self.N):
                    if not self.live[r]:
                        continue
                    d2 = (self.pos[q][0] - self.pos[r][0]) ** 2 + (self.pos[q][1] - self.pos[r][1]) ** 2
                    if d2 <= self.tag_r2:
                        claims.setdefault(r, []).append((d2, q))
        credits = [0] * self.n_tag
        for r, lst in claims.items():
            credits[sorted(lst)[0][1]] += 1
            self.live[r] = False
        self.reward = [np.float32(credits[i]) * np.float32(self.tag_reward) if i < self.n_tag
                       else (np.float32(self.tag_penalty) if i in claims else np.float32(0)) for i in range(self.N)]
        self.t += 1
        self.tags_step = len(claims)
        self.n_live_runners -= len(claims)
        self.done = self.n_live_runners == 0 or self.t >= self.T

    def obs_row(self, i):
        G = self.G
        x, y = self.pos[i]
        row = [f32div(x, G), f32div(y, G), np.float32(i < self.n_tag), np.float32(self.live[i]), f32div(self.t, self.T)]
        if self.obs_mode == 1:
            for j in range(self.N):
                if self.live[i] and self.live[j]:
                    row += [f32div(self.pos[j][0] - x, G), f32div(self.pos[j][1] - y, G), np.float32(j < self.n_tag), np.float32(1)]
                else:
                    row += [np.float32(0)] * 4
            return row
        ranked = []
        if self.live[i]:
            ranked = sorted(((self.pos[j][0] - x) ** 2 + (self.pos[j][1] - y) ** 2, j)
                            for j in range(self.N) if j != i and self.live[j])
        for k in range(self.K):
            if k < len(ranked):
                j = ranked[k][1]
                row += [f32div(self.pos[j][0] - x, G), f32div(self.pos[j][1] - y, G), np.float32(j < self.n_tag), np.float32(1)]
            else:
                row += [np.float32(0)] * 4
        return row

    def obs(self):
        return np.array([self.obs_row(i) for i in range(self.N)], dtype=np.float32)
