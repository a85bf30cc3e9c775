/*
 * wdc_oracle.cpp — CPU oracle for the batched continuous Tag roll-out path.
 *
 * TEST INFRASTRUCTURE ONLY (see wdc_oracle.h).  Plain, single-threaded, written for
 * reading: each environment on its own, each phase of a step over all agents before
 * the next phase starts, each pairwise quantity by its definition.
 *
 * The paper (Sec. 5.1, continuous variant of Tag) says what kind of world this is and
 * nothing about its numbers; the readings C1..C14 below fix the rest.  They were
 * written down before this file and are frozen with it.
 *
 *  C1  world [0, L]^2; per agent x, y, v >= 0 (float32), heading index h in [0, H),
 *      live; agents 0..N_tag-1 are taggers.
 *  C2  start state from the random block of (seed, env, agent, g = 0, stream 3):
 *      x0 = u(w0) * L, y0 = u(w1) * L, h0 = mulhi(w2, H), v0 = 0; saved at the first
 *      reset, restored (not redrawn) at every reset of an env.
 *  C3  two action categories per agent, acceleration (c = 0) and turn (c = 1), five
 *      levels each, drawn by inverse CDF from probs[e][i][c][0..4] with words 0 and 1
 *      of the block of (seed, env, agent, g, stream 2); level l means the signed step
 *      s = l - 2.  Every agent draws, in play or not.
 *  C4  h <- (h + s_turn) mod H.
 *  C5  heading table: first octant from double-precision cos / sin rounded to
 *      float32, the rest by the symmetries of the square; zeros are +0.
 *  C6  v <- v + float(s_acc) * accel; v <- 0 if v < 0; v <- vmax if v > vmax;
 *      vmax by kind (tagger / runner).
 *  C7  x' = x + v * cx[h], y' = y + v * cy[h]: product rounded, then the add.
 *  C8  x', y' clamped to [0, L]; a clamped agent stops (v <- 0).
 *  C9  an agent that is not live keeps its state, cannot be tagged, is not seen.
 *  C10 after all moves a live runner is tagged iff min over taggers of
 *      d2 = dx * dx + dy * dy (dx = x_r - x_t, dy = y_r - y_t, float32) <= tag_r2;
 *      tag_r2 < 0 disables; the credit goes to the smallest (d2, tagger index).
 *  C11 rewards, clock, end of episode, frozen done envs and reset as in the discrete
 *      variant.
 *  C12 row, D = 8 + 6 K: [x/L, y/L, v, cx[h], cy[h], is_tagger, live, t/T] then per
 *      k-th nearest other live agent j by (d2, j):
 *      [(xj - x)/L, (yj - y)/L, vj * cx[hj], vj * cy[hj], is_tagger_j, 1];
 *      zeros when fewer; zero slots for an agent that is not live.
 *  C13 all of the above in float32, each operation rounded on its own.
 *  C14 iteration = sample, step, reset of done envs.
 */
#include "wdc_oracle.h"

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <utility>
#include <vector>

#include "wd_oracle.h"

namespace {

constexpr uint32_t kStreamActionC = 2;  // C3
constexpr uint32_t kStreamInitC = 3;    // C2

bool config_ok(const wdco_config* c) {
  if (!c) return false;
  if (c->num_envs < 0 || c->num_agents < 2) return false;
  if (c->num_taggers < 1 || c->num_taggers > c->num_agents - 1) return false;
  if (c->num_headings < 4 || c->num_headings % 4 != 0 || c->num_headings > 4096) return false;
  if (c->episode_length < 1) return false;
  if (c->obs_k < 0 || c->obs_k > c->num_agents - 1) return false;
  if (!(c->world_size > 0.0f)) return false;
  return true;
}

bool state_ok(const wdco_state* s) {
  return s && s->x && s->y && s->v && s->h && s->x0 && s->y0 && s->h0 && s->live && s->action && s->reward &&
         s->obs && s->t && s->done && s->n_live_runners && s->tags_step;
}

// C10: squared distance in float32, each operation rounded.
inline float squared_distance(float xa, float ya, float xb, float yb) {
  const float dx = xa - xb;
  const float dy = ya - yb;
  const float dx2 = dx * dx;
  const float dy2 = dy * dy;
  return dx2 + dy2;
}

inline float plus_zero(float v) { return v == 0.0f ? 0.0f : v; }

void restore_env(const wdco_config* c, const wdco_state* s, int32_t e) {
  const int32_t N = c->num_agents;
  for (int32_t i = 0; i < N; ++i) {
    const int64_t a = int64_t(e) * N + i;
    s->x[a] = s->x0[a];
    s->y[a] = s->y0[a];
    s->h[a] = s->h0[a];
    s->v[a] = 0.0f;
    s->live[a] = 1;
  }
  s->t[e] = 0;
  s->n_live_runners[e] = N - c->num_taggers;
  s->tags_step[e] = 0;
  s->done[e] = 0;
  wdco_observe(c, s, e);
}

}  // namespace

extern "C" {

int32_t wdco_obs_dim(const wdco_config* cfg) { return 8 + 6 * cfg->obs_k; }

// C5.  Quarter turn q = H / 4.  Inside a quadrant the index r in [0, q) is in the first
// octant when 2 r <= q and is the mirror image about 45 degrees of q - r otherwise; the
// quadrant number turns the pair by that many right angles.
int wdco_heading_table(int32_t H, float* cx, float* cy) {
  if (H < 4 || H % 4 != 0 || !cx || !cy) return -1;
  const int32_t q = H / 4;
  const double two_pi = 6.283185307179586476925286766559;
  auto octant = [&](int32_t r, float* c, float* s) {  // 2 r <= q
    const double angle = two_pi * double(r) / double(H);
    *c = static_cast<float>(std::cos(angle));
    *s = static_cast<float>(std::sin(angle));
    if (2 * r == q) *s = *c;  // 45 degrees: equal components
  };
  for (int32_t h = 0; h < H; ++h) {
    const int32_t k = h / q, r = h % q;
    float c, s;
    if (2 * r <= q) {
      octant(r, &c, &s);
    } else {
      octant(q - r, &s, &c);
    }
    float rx, ry;
    switch (k) {
      case 0: rx = c; ry = s; break;
      case 1: rx = -s; ry = c; break;
      case 2: rx = -c; ry = -s; break;
      default: rx = s; ry = -c; break;
    }
    cx[h] = plus_zero(rx);
    cy[h] = plus_zero(ry);
  }
  return 0;
}

int wdco_reset(const wdco_config* c, const wdco_state* s, int mode) {
  if (!config_ok(c) || !state_ok(s)) return -1;
  if (mode != WDCO_RESET_ALL && mode != WDCO_RESET_DONE) return -1;
  const int32_t N = c->num_agents;
  if (mode == WDCO_RESET_ALL) {
    for (int32_t e = 0; e < c->num_envs; ++e) {
      for (int32_t i = 0; i < N; ++i) {
        uint32_t w[4];
        wdo_random_block(c->seed, uint32_t(c->env_offset + e), uint32_t(i), 0, kStreamInitC, w);  // C2
        const int64_t a = int64_t(e) * N + i;
        s->x0[a] = wdo_uniform_from_word(w[0]) * c->world_size;
        s->y0[a] = wdo_uniform_from_word(w[1]) * c->world_size;
        s->h0[a] = int32_t((uint64_t(w[2]) * uint64_t(c->num_headings)) >> 32);
      }
    }
  }
  for (int32_t e = 0; e < c->num_envs; ++e)
    if (mode == WDCO_RESET_ALL || s->done[e] == 1) restore_env(c, s, e);
  return 0;
}

int wdco_sample(const wdco_config* c, const wdco_state* s, const float* probs, uint64_t g) {
  if (!config_ok(c) || !state_ok(s) || !probs) return -1;
  const int32_t N = c->num_agents;
  for (int32_t e = 0; e < c->num_envs; ++e) {
    for (int32_t i = 0; i < N; ++i) {
      uint32_t w[4];
      wdo_random_block(c->seed, uint32_t(c->env_offset + e), uint32_t(i), g, kStreamActionC, w);  // C3
      const int64_t a = int64_t(e) * N + i;
      for (int32_t cat = 0; cat < 2; ++cat)
        s->action[2 * a + cat] = wdo_sample_from_u(probs + (2 * a + cat) * 5, 5, wdo_uniform_from_word(w[cat]));
    }
  }
  return 0;
}

int wdco_step(const wdco_config* c, const wdco_state* s) {
  if (!config_ok(c) || !state_ok(s)) return -1;
  const int32_t N = c->num_agents, N_tag = c->num_taggers, H = c->num_headings;
  const float L = c->world_size;
  std::vector<float> cx(H), cy(H);
  wdco_heading_table(H, cx.data(), cy.data());
  std::vector<int32_t> credits(N_tag), tagged_now(N);
  for (int32_t e = 0; e < c->num_envs; ++e) {
    if (s->done[e] == 1) continue;  // C11 (R6)
    const int64_t base = int64_t(e) * N;
    // C4, C6, C7, C8: every live agent turns, changes speed, moves
    for (int32_t i = 0; i < N; ++i) {
      const int64_t a = base + i;
      if (s->live[a] != 1) continue;  // C9
      const int32_t s_acc = s->action[2 * a] - 2, s_turn = s->action[2 * a + 1] - 2;
      int32_t h = (s->h[a] + s_turn) % H;
      if (h < 0) h += H;
      const float vmax = i < N_tag ? c->max_speed_tagger : c->max_speed_runner;
      const float dv = static_cast<float>(s_acc) * c->accel;
      float v = s->v[a] + dv;
      if (v < 0.0f) v = 0.0f;
      if (v > vmax) v = vmax;
      const float step_x = v * cx[h];
      const float step_y = v * cy[h];
      float x = s->x[a] + step_x;
      float y = s->y[a] + step_y;
      bool clamped = false;
      if (x < 0.0f) { x = 0.0f; clamped = true; }
      if (x > L) { x = L; clamped = true; }
      if (y < 0.0f) { y = 0.0f; clamped = true; }
      if (y > L) { y = L; clamped = true; }
      if (clamped) v = 0.0f;
      s->x[a] = x;
      s->y[a] = y;
      s->v[a] = v;
      s->h[a] = h;
    }
    // C10: tag check on the moved positions
    std::fill(credits.begin(), credits.end(), 0);
    std::fill(tagged_now.begin(), tagged_now.end(), 0);
    int32_t tags = 0;
    if (c->tag_r2 >= 0.0f) {
      for (int32_t r = N_tag; r < N; ++r) {
        if (s->live[base + r] != 1) continue;
        int32_t best_t = -1;
        float best_d2 = 0.0f;
        for (int32_t t = 0; t < N_tag; ++t) {
          const float d2 = squared_distance(s->x[base + r], s->y[base + r], s->x[base + t], s->y[base + t]);
          if (best_t < 0 || d2 < best_d2) {  // strict: equal distances keep the smaller index
            best_t = t;
            best_d2 = d2;
          }
        }
        if (best_d2 <= c->tag_r2) {
          tagged_now[r] = 1;
          ++credits[best_t];
          ++tags;
        }
      }
    }
    for (int32_t r = N_tag; r < N; ++r)
      if (tagged_now[r]) s->live[base + r] = 0;
    // C11: rewards, clock, end of episode
    for (int32_t i = 0; i < N; ++i) {
      float rew = 0.0f;
      if (i < N_tag)
        rew = static_cast<float>(credits[i]) * c->tag_reward;
      else if (tagged_now[i])
        rew = c->tag_penalty;
      s->reward[base + i] = rew;
    }
    s->t[e] += 1;
    s->n_live_runners[e] -= tags;
    s->tags_step[e] = tags;
    s->done[e] = (s->n_live_runners[e] == 0 || s->t[e] >= c->episode_length) ? 1 : 0;
    wdco_observe(c, s, e);
  }
  return 0;
}

// C12.
int wdco_observe(const wdco_config* c, const wdco_state* s, int32_t e) {
  if (!config_ok(c) || !state_ok(s) || e < 0 || e >= c->num_envs) return -1;
  const int32_t N = c->num_agents, N_tag = c->num_taggers, K = c->obs_k, H = c->num_headings;
  const int32_t D = wdco_obs_dim(c);
  const float L = c->world_size;
  std::vector<float> cx(H), cy(H);
  wdco_heading_table(H, cx.data(), cy.data());
  const int64_t base = int64_t(e) * N;
  const float t_feature = static_cast<float>(s->t[e]) / static_cast<float>(c->episode_length);
  std::vector<std::pair<float, int32_t>> others;
  for (int32_t i = 0; i < N; ++i) {
    float* row = s->obs + (base + i) * D;
    std::fill(row, row + D, 0.0f);
    const float x = s->x[base + i], y = s->y[base + i];
    row[0] = x / L;
    row[1] = y / L;
    row[2] = s->v[base + i];
    row[3] = cx[s->h[base + i]];
    row[4] = cy[s->h[base + i]];
    row[5] = i < N_tag ? 1.0f : 0.0f;
    row[6] = s->live[base + i] == 1 ? 1.0f : 0.0f;
    row[7] = t_feature;
    if (s->live[base + i] != 1) continue;
    others.clear();
    for (int32_t j = 0; j < N; ++j)
      if (j != i && s->live[base + j] == 1)
        others.emplace_back(squared_distance(s->x[base + j], s->y[base + j], x, y), j);
    std::sort(others.begin(), others.end());  // by (d2, j)
    for (int32_t k = 0; k < K && k < int32_t(others.size()); ++k) {
      const int32_t j = others[k].second;
      float* slot = row + 8 + 6 * k;
      const float dx = s->x[base + j] - x;
      const float dy = s->y[base + j] - y;
      slot[0] = dx / L;
      slot[1] = dy / L;
      slot[2] = s->v[base + j] * cx[s->h[base + j]];
      slot[3] = s->v[base + j] * cy[s->h[base + j]];
      slot[4] = j < N_tag ? 1.0f : 0.0f;
      slot[5] = 1.0f;
    }
  }
  return 0;
}

}  // extern "C"
