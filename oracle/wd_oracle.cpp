/*
 * wd_oracle.cpp — CPU oracle for the batched discrete Tag roll-out path.
 *
 * TEST INFRASTRUCTURE ONLY (see wd_oracle.h).  Plain, single-threaded, written
 * for reading, not for speed: each environment is processed on its own, each
 * phase of a step over all agents before the next phase starts, each pairwise
 * quantity by its definition.
 *
 * The Tag rules of the paper (Sec. 5.1 "Benchmark Environments") are stated in
 * prose without constants.  The readings below (R1..R17) fix what the paper
 * leaves open; each is marked where it is implemented.
 *
 *  R1  agents 0..N_tag-1 are taggers, the rest runners, in every env.
 *  R2  start positions are uniform on the grid, from the random block of
 *      (seed, env, agent, g = 0, stream 1): x0 = mulhi(w0, G), y0 = mulhi(w1, G).
 *  R3  agents do not block each other; a cell may hold any number of agents.
 *  R4  sampling is by inverse CDF in float32, accumulated left to right, with a
 *      strict "u < c" test and the last action as the fall-through.
 *  R5  random numbers are Philox4x32-10 blocks, key = (seed lo, seed hi),
 *      counter = (env, index, g lo, stream | g hi << 8).  A block has four words: for
 *      sampling (stream 0) the index is agent / 4 and agent i draws from word i mod 4,
 *      so no word of a block is thrown away; for start positions (stream 1) the index
 *      is the agent and words 0 and 1 give x and y.
 *  R6  an env whose done flag is set is not stepped at all.
 *  R7  actions: 0 stay, 1 up (y+1), 2 down (y-1), 3 left (x-1), 4 right (x+1);
 *      any other value is treated as stay.
 *  R8  coordinates are clamped to [0, G-1]: a move into a wall is a stay.
 *  R9  agents that are not live do not move, cannot be tagged, are not seen by
 *      others and get reward 0.  Taggers are always live.
 *  R10 after all moves, a live runner is tagged iff some tagger is at squared
 *      Euclidean distance <= tag_r2 (integers); tag_r2 < 0 disables tagging.
 *  R11 one credit per tag, to the in-range tagger with the smallest
 *      (squared distance, tagger index).
 *  R12 rewards: tagger = credits * tag_reward (one float multiply); runner tagged
 *      on this step = tag_penalty; everyone else 0.  No other reward terms.
 *  R13 t += 1; n_live_runners -= tags; tags_step = tags;
 *      done = (n_live_runners == 0 || t >= T).
 *  R14 observation row (partial mode), D = 5 + 4K floats, from the state after
 *      move and tag and the incremented t:
 *        [x/G, y/G, is_tagger, live, t/T] then for the k-th nearest other live
 *        agent j by (squared distance, j): [(xj-x)/G, (yj-y)/G, is_tagger_j, 1],
 *        zeros when there are fewer than k+1 such agents; an agent that is not
 *        live has zeros in all neighbour slots.  Each quotient is one int->float
 *        conversion of the integer numerator followed by one float32 divide.
 *  R15 full mode, D = 5 + 4N: slot j (index order, self included) holds
 *        [(xj-x)/G, (yj-y)/G, is_tagger_j, 1] if j is live, else zeros; an agent
 *        that is not live has zeros in all slots.
 *  R16 every tie is broken by index, so exactly one result is correct.
 *  R17 reset restores, it does not redraw: pos <- pos0, live <- 1, t <- 0,
 *      n_live_runners <- N_run, tags_step <- 0, done <- 0, obs <- observation of
 *      that state; reward and action are left as they are.
 */
#include "wd_oracle.h"

#include <algorithm>
#include <cstdint>
#include <utility>
#include <vector>

namespace {

constexpr uint32_t kStreamAction = 0;  // R5: stream ids
constexpr uint32_t kStreamInit = 1;

bool config_ok(const wdo_config* c) {
  if (!c) return false;
  if (c->num_envs < 0 || c->num_agents < 2) return false;
  if (c->num_taggers < 1 || c->num_taggers > c->num_agents - 1) return false;
  if (c->grid_size < 1 || c->grid_size > 32767) return false;
  if (c->episode_length < 1) return false;
  if (c->obs_mode != 0 && c->obs_mode != 1) return false;
  if (c->obs_mode == 0 && (c->obs_k < 0 || c->obs_k > c->num_agents - 1)) return false;
  return true;
}

bool state_ok(const wdo_state* s) {
  return s && s->pos_x && s->pos_y && s->pos_x0 && s->pos_y0 && s->live && s->action &&
         s->reward && s->obs && s->t && s->done && s->n_live_runners && s->tags_step;
}

inline int64_t squared_distance(int32_t xa, int32_t ya, int32_t xb, int32_t yb) {
  const int64_t dx = int64_t(xa) - int64_t(xb);
  const int64_t dy = int64_t(ya) - int64_t(yb);
  return dx * dx + dy * dy;
}

// One feature: integer numerator -> float32, then one float32 divide (R14).
inline float ratio(int32_t numerator, int32_t denominator) {
  return static_cast<float>(numerator) / static_cast<float>(denominator);
}

// R17: put local env e into its start state.
void restore_env(const wdo_config* c, const wdo_state* s, int32_t e) {
  const int32_t N = c->num_agents;
  for (int32_t i = 0; i < N; ++i) {
    const int64_t a = int64_t(e) * N + i;
    s->pos_x[a] = s->pos_x0[a];
    s->pos_y[a] = s->pos_y0[a];
    s->live[a] = 1;
  }
  s->t[e] = 0;
  s->n_live_runners[e] = N - c->num_taggers;
  s->tags_step[e] = 0;
  s->done[e] = 0;
  wdo_observe(c, s, e);
}

}  // namespace

extern "C" {

// Philox4x32-10 as published (Salmon et al., SC'11, Sec. 3.3 and the table of
// multipliers and Weyl key increments for the 4x32 variant): ten rounds; a round
// maps (c0,c1,c2,c3) to (hi(M1*c2)^c1^k0, lo(M1*c2), hi(M0*c0)^c3^k1, lo(M0*c0));
// the key is bumped by (W0, W1) between rounds.
void wdo_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  const uint64_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
  const uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int round = 0; round < 10; ++round) {
    const uint64_t p0 = M0 * c0;
    const uint64_t p1 = M1 * c2;
    const uint32_t n0 = uint32_t(p1 >> 32) ^ c1 ^ k0;
    const uint32_t n1 = uint32_t(p1);
    const uint32_t n2 = uint32_t(p0 >> 32) ^ c3 ^ k1;
    const uint32_t n3 = uint32_t(p0);
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    k0 += W0;
    k1 += W1;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// R5: how (seed, env, index, step, stream) become key and counter.
void wdo_random_block(uint64_t seed, uint32_t env, uint32_t index, uint64_t g,
                      uint32_t stream, uint32_t out[4]) {
  const uint32_t key[2] = {uint32_t(seed), uint32_t(seed >> 32)};
  const uint32_t ctr[4] = {env, index, uint32_t(g),
                           (stream & 0xFFu) | (uint32_t(g >> 32) << 8)};
  wdo_philox4x32_10(ctr, key, out);
}

// R4: 24 random bits -> a float32 in [0,1), exactly representable.
float wdo_uniform_from_word(uint32_t w) {
  return static_cast<float>(w >> 8) * (1.0f / 16777216.0f);
}

// R4: inverse CDF, float32 running sum, strict comparison, last action as fall-through.
int32_t wdo_sample_from_u(const float* p, int32_t num_actions, float u) {
  volatile float c = 0.0f;  // volatile: keep every partial sum rounded to float32
  for (int32_t a = 0; a < num_actions; ++a) {
    c = c + p[a];
    if (u < c) return a;
  }
  return num_actions - 1;
}

int32_t wdo_obs_dim(const wdo_config* c) {
  if (!config_ok(c)) return -1;
  return c->obs_mode == 0 ? 5 + 4 * c->obs_k : 5 + 4 * c->num_agents;
}

// R14 / R15.
int wdo_observe(const wdo_config* c, const wdo_state* s, int32_t e) {
  if (!config_ok(c) || !state_ok(s) || e < 0 || e >= c->num_envs) return -1;
  const int32_t N = c->num_agents, G = c->grid_size, T = c->episode_length;
  const int32_t D = wdo_obs_dim(c);
  const int32_t* x = s->pos_x + int64_t(e) * N;
  const int32_t* y = s->pos_y + int64_t(e) * N;
  const int32_t* live = s->live + int64_t(e) * N;
  std::vector<std::pair<int64_t, int32_t>> others;  // (squared distance, index)
  for (int32_t i = 0; i < N; ++i) {
    float* o = s->obs + (int64_t(e) * N + i) * D;
    o[0] = ratio(x[i], G);
    o[1] = ratio(y[i], G);
    o[2] = i < c->num_taggers ? 1.0f : 0.0f;  // R1
    o[3] = live[i] ? 1.0f : 0.0f;
    o[4] = ratio(s->t[e], T);
    for (int32_t d = 5; d < D; ++d) o[d] = 0.0f;
    if (!live[i]) continue;  // R9: no neighbours for an agent that left the game
    if (c->obs_mode == 1) {  // R15
      for (int32_t j = 0; j < N; ++j) {
        if (!live[j]) continue;
        float* slot = o + 5 + 4 * j;
        slot[0] = ratio(x[j] - x[i], G);
        slot[1] = ratio(y[j] - y[i], G);
        slot[2] = j < c->num_taggers ? 1.0f : 0.0f;
        slot[3] = 1.0f;
      }
      continue;
    }
    // R14: the K smallest (squared distance, index) among the other live agents.
    others.clear();
    for (int32_t j = 0; j < N; ++j)
      if (j != i && live[j]) others.emplace_back(squared_distance(x[i], y[i], x[j], y[j]), j);
    const size_t k_found = std::min<size_t>(size_t(c->obs_k), others.size());
    std::partial_sort(others.begin(), others.begin() + k_found, others.end());
    for (size_t k = 0; k < k_found; ++k) {
      const int32_t j = others[k].second;
      float* slot = o + 5 + 4 * k;
      slot[0] = ratio(x[j] - x[i], G);
      slot[1] = ratio(y[j] - y[i], G);
      slot[2] = j < c->num_taggers ? 1.0f : 0.0f;
      slot[3] = 1.0f;
    }
  }
  return 0;
}

int wdo_reset(const wdo_config* c, const wdo_state* s, int mode) {
  if (!config_ok(c) || !state_ok(s)) return -1;
  if (mode != WDO_RESET_ALL && mode != WDO_RESET_DONE) return -1;
  const int32_t E = c->num_envs, N = c->num_agents, G = c->grid_size;
  if (mode == WDO_RESET_ALL) {
    for (int32_t e = 0; e < E; ++e)
      for (int32_t i = 0; i < N; ++i) {  // R2
        uint32_t w[4];
        wdo_random_block(c->seed, uint32_t(c->env_offset + e), uint32_t(i), 0, kStreamInit, w);
        s->pos_x0[int64_t(e) * N + i] = int32_t((uint64_t(w[0]) * uint64_t(G)) >> 32);
        s->pos_y0[int64_t(e) * N + i] = int32_t((uint64_t(w[1]) * uint64_t(G)) >> 32);
      }
    for (int32_t e = 0; e < E; ++e) restore_env(c, s, e);
  } else {
    for (int32_t e = 0; e < E; ++e)
      if (s->done[e]) restore_env(c, s, e);
  }
  return 0;
}

int wdo_sample(const wdo_config* c, const wdo_state* s, const float* probs, uint64_t g) {
  if (!config_ok(c) || !state_ok(s) || !probs) return -1;
  const int32_t E = c->num_envs, N = c->num_agents, A = 5;
  for (int32_t e = 0; e < E; ++e)
    for (int32_t i = 0; i < N; ++i) {
      uint32_t w[4];  // R5: one block per four consecutive agents, one word each
      wdo_random_block(c->seed, uint32_t(c->env_offset + e), uint32_t(i) / 4u, g, kStreamAction, w);
      const float u = wdo_uniform_from_word(w[i % 4]);
      const int64_t a = int64_t(e) * N + i;
      s->action[a] = wdo_sample_from_u(probs + a * A, A, u);
    }
  return 0;
}

int wdo_step(const wdo_config* c, const wdo_state* s) {
  if (!config_ok(c) || !state_ok(s)) return -1;
  const int32_t E = c->num_envs, N = c->num_agents, N_tag = c->num_taggers;
  const int32_t G = c->grid_size, T = c->episode_length;
  std::vector<int32_t> credits(size_t(N_tag), 0);
  std::vector<char> tagged_now(size_t(N), 0);
  for (int32_t e = 0; e < E; ++e) {
    if (s->done[e]) continue;  // R6
    int32_t* x = s->pos_x + int64_t(e) * N;
    int32_t* y = s->pos_y + int64_t(e) * N;
    int32_t* live = s->live + int64_t(e) * N;
    const int32_t* action = s->action + int64_t(e) * N;
    float* reward = s->reward + int64_t(e) * N;

    // Move (R3, R7, R8, R9).
    for (int32_t i = 0; i < N; ++i) {
      if (!live[i]) continue;
      int32_t nx = x[i], ny = y[i];
      switch (action[i]) {
        case 1: ny += 1; break;
        case 2: ny -= 1; break;
        case 3: nx -= 1; break;
        case 4: nx += 1; break;
        default: break;
      }
      x[i] = std::min(std::max(nx, 0), G - 1);
      y[i] = std::min(std::max(ny, 0), G - 1);
    }

    // Tag (R10, R11): every live runner against every tagger, on the moved positions.
    std::fill(credits.begin(), credits.end(), 0);
    std::fill(tagged_now.begin(), tagged_now.end(), 0);
    int32_t tags = 0;
    for (int32_t r = N_tag; r < N; ++r) {
      if (!live[r] || c->tag_r2 < 0) continue;
      bool found = false;
      int64_t best_d2 = 0;
      int32_t best_tagger = -1;
      for (int32_t q = 0; q < N_tag; ++q) {
        const int64_t d2 = squared_distance(x[r], y[r], x[q], y[q]);
        if (d2 > int64_t(c->tag_r2)) continue;
        if (!found || d2 < best_d2) {  // ascending q, strict "<": smallest index wins ties
          found = true;
          best_d2 = d2;
          best_tagger = q;
        }
      }
      if (found) {
        tagged_now[size_t(r)] = 1;
        credits[size_t(best_tagger)] += 1;
        tags += 1;
      }
    }
    for (int32_t r = N_tag; r < N; ++r)
      if (tagged_now[size_t(r)]) live[r] = 0;

    // Rewards (R12).
    for (int32_t q = 0; q < N_tag; ++q) reward[q] = static_cast<float>(credits[size_t(q)]) * c->tag_reward;
    for (int32_t r = N_tag; r < N; ++r) reward[r] = tagged_now[size_t(r)] ? c->tag_penalty : 0.0f;

    // Time and termination (R13).
    s->t[e] += 1;
    s->n_live_runners[e] -= tags;
    s->tags_step[e] = tags;
    s->done[e] = (s->n_live_runners[e] == 0 || s->t[e] >= T) ? 1 : 0;

    // Observations (R14, R15).
    wdo_observe(c, s, e);
  }
  return 0;
}

}  // extern "C"
