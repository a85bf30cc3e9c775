// wdc.hip — continuous Tag: the C ABI of include/wdc.h and its kernels (gfx950).
//
// One thread per agent.  A workgroup of `bd` threads holds floor(bd / N) envs (these envs are
// small: the paper's own continuous-Tag runs have 5 to 45 agents per env); the moved positions
// and velocities of the workgroup's envs are staged in LDS, where the runner-side tag test and the
// brute-force K-nearest search read them.  Every float32 operation that feeds a comparison is
// written as its own statement and the file is compiled without contraction, so that the state is
// reproducible to the bit (arXiv 2108.13976, Sec. 5.1, continuous variant; the numbers are this
// build's reading, stated in wdc.h).
#include <hip/hip_runtime.h>

#include <cmath>
#include <new>
#include <string>
#include <utility>
#include <vector>

#include "../../include/wdc.h"
#include "wd_dev_common.h"

namespace wdc {

constexpr int kMaxThreads = 1024;      // one thread per agent, so also the largest env
constexpr int kMaxK = 8;
constexpr uint32_t kStreamActionC = 2;  // random streams of this variant (0 and 1 are the discrete variant's)
constexpr uint32_t kStreamInitC = 3;
enum Mode : int { kSample = 1, kStep = 2, kResetDone = 4, kResetAll = 8 };

struct Params {
  int32_t E, N, N_tag, H, T, K, D;
  int32_t envs_per_wg, threads;
  uint32_t env_offset, seed_lo, seed_hi;
  wd::FastDiv div_N;
  float L, inv_L, inv_T, accel, vmax_tagger, vmax_runner, tag_r2, tag_reward, tag_penalty;
  float *x, *y, *v;
  int32_t* h;
  float *x0, *y0;
  int32_t* h0;
  int32_t* live;
  int32_t* action;
  float* reward;
  float* obs;
  int32_t *t, *done, *n_live_runners, *tags_step;
  const float2* table;  // (cx, cy) per heading
};

namespace {

using wd::dev::philox_block;
using wd::dev::sample_action;

// start state of every agent (once per reset of all envs)
__global__ __launch_bounds__(256) void init_kernel(const Params p) {
  const int64_t a = int64_t(blockIdx.x) * 256 + threadIdx.x;
  if (a >= int64_t(p.E) * p.N) return;
  const uint32_t e = uint32_t(a / p.N), i = uint32_t(a - int64_t(e) * p.N);
  const wd::dev::Block4 r = philox_block(p.env_offset + e, i, 0u, kStreamInitC, p.seed_lo, p.seed_hi);
  const float u0 = static_cast<float>(r.w[0] >> 8) * (1.0f / 16777216.0f);
  const float u1 = static_cast<float>(r.w[1] >> 8) * (1.0f / 16777216.0f);
  p.x0[a] = u0 * p.L;
  p.y0[a] = u1 * p.L;
  p.h0[a] = int32_t(__umulhi(r.w[2], uint32_t(p.H)));
}

// heading index brought into [0, H): also keeps a caller's stray value from indexing outside the table
__device__ __forceinline__ int wrap_heading(int h, int H) {
  const int r = h % H;
  return r < 0 ? r + H : r;
}

__device__ __forceinline__ float squared_distance(float xa, float ya, float xb, float yb) {
  const float dx = xa - xb;
  const float dy = ya - yb;
  const float dx2 = dx * dx;
  const float dy2 = dy * dy;
  return dx2 + dy2;
}

// One live agent turns, changes speed, moves and meets the walls.
__device__ __forceinline__ void advance_agent(const Params& p, bool tagger, int lvl_acc, int lvl_turn, float& x, float& y,
                                              float& v, int& h, float2& dir) {
  h = wrap_heading(h + (lvl_turn - 2), p.H);
  dir = p.table[h];
  const float vmax = tagger ? p.vmax_tagger : p.vmax_runner;
  const float dv = static_cast<float>(lvl_acc - 2) * p.accel;
  v = v + dv;
  if (v < 0.0f) v = 0.0f;
  if (v > vmax) v = vmax;
  const float step_x = v * dir.x;
  const float step_y = v * dir.y;
  x = x + step_x;
  y = y + step_y;
  bool clamped = false;
  if (x < 0.0f) { x = 0.0f; clamped = true; }
  if (x > p.L) { x = p.L; clamped = true; }
  if (y < 0.0f) { y = 0.0f; clamped = true; }
  if (y > p.L) { y = p.L; clamped = true; }
  if (clamped) v = 0.0f;
}

// An agent's ten probabilities (five per action category) as five 8-byte pieces.
struct Probs10 {
  float2 q[5];
};
__device__ __forceinline__ Probs10 load_probs(const float* __restrict__ probs, int64_t a) {
  const float2* pr = reinterpret_cast<const float2*>(probs + a * 10);
  Probs10 r;
#pragma unroll
  for (int k = 0; k < 5; ++k) r.q[k] = pr[k];
  return r;
}

// The two levels of an agent's action from its ten probabilities and one random block.
__device__ __forceinline__ int2 draw_levels(const Params& p, const Probs10& pr, int e, int i, uint32_t g_lo,
                                            uint32_t g_hi) {
  const wd::dev::Block4 r = philox_block(p.env_offset + uint32_t(e), uint32_t(i), g_lo, kStreamActionC | (g_hi << 8),
                                         p.seed_lo, p.seed_hi);
  const int lvl_acc = sample_action(pr.q[0].x, pr.q[0].y, pr.q[1].x, pr.q[1].y, r.w[0]);   // probabilities 0..3 of category 0
  const int lvl_turn = sample_action(pr.q[2].y, pr.q[3].x, pr.q[3].y, pr.q[4].x, r.w[1]);  // 5..8 = 0..3 of category 1
  return make_int2(lvl_acc, lvl_turn);
}

// The nearest tagger of a runner at (x, y) by (d2, index): true if it is in range.
__device__ __forceinline__ bool tagger_in_range(const Params& p, const float* s_x, const float* s_y, int first, float x,
                                                float y, int* tagger_out) {
  int best_t = 0;
  float best_d2 = squared_distance(x, y, s_x[first], s_y[first]);
  for (int t = 1; t < p.N_tag; ++t) {
    const float d2 = squared_distance(x, y, s_x[first + t], s_y[first + t]);
    if (d2 < best_d2) {
      best_d2 = d2;
      best_t = t;
    }
  }
  *tagger_out = best_t;
  return best_d2 <= p.tag_r2;
}

// The observation row of agent i of the env whose agents sit in LDS slots first .. first + N - 1.
template <int KT>
__device__ __forceinline__ void write_row(const Params& p, float* row, const float* s_x, const float* s_y,
                                          const float* s_vx, const float* s_vy, const int32_t* s_live, int first, int i,
                                          float x, float y, float v, float2 dir, bool tagger, int live, int t_out) {
  const int K = p.K;
  uint64_t keys[KT];
#pragma unroll
  for (int k = 0; k < KT; ++k) keys[k] = ~0ull;
  if (live == 1 && K > 0) {
    for (int j = 0; j < p.N; ++j) {
      if (j == i || s_live[first + j] != 1) continue;
      const float d2 = squared_distance(s_x[first + j], s_y[first + j], x, y);
      uint64_t key = (uint64_t(__float_as_uint(d2)) << 32) | uint32_t(j);  // d2 >= +0: its bits order like its value
#pragma unroll
      for (int k = 0; k < KT; ++k) {
        if (k < K && key < keys[k]) {
          const uint64_t tmp = keys[k];
          keys[k] = key;
          key = tmp;
        }
      }
    }
  }
  float2* row2 = reinterpret_cast<float2*>(row);  // D is even and the buffer 256-byte aligned: 8-byte pieces
  row2[0] = make_float2(x * p.inv_L, y * p.inv_L);
  row2[1] = make_float2(v, dir.x);
  row2[2] = make_float2(dir.y, tagger ? 1.0f : 0.0f);
  row2[3] = make_float2(live == 1 ? 1.0f : 0.0f, static_cast<float>(t_out) * p.inv_T);
#pragma unroll
  for (int k = 0; k < KT; ++k) {
    if (k < K) {
      float2 s0 = make_float2(0.0f, 0.0f), s1 = s0, s2 = s0;
      if (keys[k] != ~0ull) {
        const int j = int(uint32_t(keys[k]));
        const float dx = s_x[first + j] - x;
        const float dy = s_y[first + j] - y;
        s0 = make_float2(dx * p.inv_L, dy * p.inv_L);
        s1 = make_float2(s_vx[first + j], s_vy[first + j]);
        s2 = make_float2(j < p.N_tag ? 1.0f : 0.0f, 1.0f);
      }
      row2[4 + 3 * k] = s0;
      row2[5 + 3 * k] = s1;
      row2[6 + 3 * k] = s2;
    }
  }
}

// KT: length of the register list of nearest keys (4 or 8, at least K)
template <int KT>
__global__ __launch_bounds__(kMaxThreads) void env_kernel(const Params p, const int mode, const float* __restrict__ probs,
                                                           const uint32_t g_lo, const uint32_t g_hi) {
  // per local agent slot: moved position, velocity components, live flag, credits (taggers)
  // (dynamic LDS: 26 bytes per thread of the workgroup, see lds_bytes)
  extern __shared__ __align__(16) unsigned char smem[];
  float* const s_x = reinterpret_cast<float*>(smem);
  float* const s_y = s_x + p.threads;
  float* const s_vx = s_y + p.threads;
  float* const s_vy = s_vx + p.threads;
  int32_t* const s_live = reinterpret_cast<int32_t*>(s_vy + p.threads);
  int32_t* const s_credits = s_live + p.threads;
  int32_t* const s_tags = s_credits + p.threads;  // per env of the workgroup: at most threads / 2
  const int tid = threadIdx.x;
  const int el = int(wd::dev::fastdiv(uint32_t(tid), p.div_N));  // env of the workgroup
  const int i = tid - el * p.N;                                  // agent
  const int e = blockIdx.x * p.envs_per_wg + el;
  const bool valid = el < p.envs_per_wg && e < p.E;
  const int first = el * p.N;  // slot of the env's agent 0
  const int64_t a = int64_t(valid ? e : 0) * p.N + i;
  const bool tagger = i < p.N_tag;

  // ---- sampler: two draws per agent from one random block ------------------------------------
  int lvl_acc = 2, lvl_turn = 2;
  if (mode & kSample) {
    if (valid) {
      const int2 lv = draw_levels(p, load_probs(probs, a), e, i, g_lo, g_hi);
      lvl_acc = lv.x;
      lvl_turn = lv.y;
      *reinterpret_cast<int2*>(p.action + 2 * a) = lv;
    }
    if (mode == kSample) return;
  } else if ((mode & kStep) && valid) {
    const int2 act = *reinterpret_cast<const int2*>(p.action + 2 * a);
    lvl_acc = act.x;
    lvl_turn = act.y;
  }

  int done_in = 0, t_in = 0, nlr_in = 0;
  if (valid) {
    done_in = p.done[e];
    t_in = p.t[e];
    nlr_in = p.n_live_runners[e];
  }
  const bool step_act = (mode & kStep) && valid && !done_in;
  bool new_rows = false;
  int t_out = t_in;
  bool done_now = done_in != 0;
  float x = 0.0f, y = 0.0f, v = 0.0f;
  int h = 0, live = 0;
  float2 dir = make_float2(1.0f, 0.0f);

  if (mode & kStep) {
    if (step_act) {
      x = p.x[a];
      y = p.y[a];
      v = p.v[a];
      h = p.h[a];
      live = p.live[a];
      if (live == 1) {
        advance_agent(p, tagger, lvl_acc, lvl_turn, x, y, v, h, dir);
        p.x[a] = x;
        p.y[a] = y;
        p.v[a] = v;
        p.h[a] = h;
      } else {
        dir = p.table[wrap_heading(h, p.H)];
      }
      s_x[tid] = x;
      s_y[tid] = y;
      s_vx[tid] = v * dir.x;
      s_vy[tid] = v * dir.y;
      s_live[tid] = live;
      s_credits[tid] = 0;
      if (i == 0) s_tags[el] = 0;
    }
    __syncthreads();
    // ---- tag test from the runner's side: nearest tagger by (d2, index) ------------------------
    bool tagged_now = false;
    if (step_act && !tagger && live == 1 && p.tag_r2 >= 0.0f) {
      int best_t;
      if (tagger_in_range(p, s_x, s_y, first, x, y, &best_t)) {
        tagged_now = true;
        live = 0;
        s_live[tid] = 0;  // (the loops above read taggers only, and taggers stay live)
        p.live[a] = 0;
        atomicAdd(&s_credits[first + best_t], 1);
        atomicAdd(&s_tags[el], 1);
      }
    }
    __syncthreads();
    // ---- rewards, clock, end of episode ---------------------------------------------------------
    if (step_act) {
      float rew = 0.0f;
      if (tagger)
        rew = static_cast<float>(s_credits[tid]) * p.tag_reward;
      else if (tagged_now)
        rew = p.tag_penalty;
      p.reward[a] = rew;
      const int tags = s_tags[el];
      const int nlr = nlr_in - tags;
      t_out = t_in + 1;
      done_now = nlr == 0 || t_out >= p.T;
      if (i == 0) {
        p.t[e] = t_out;
        p.n_live_runners[e] = nlr;
        p.tags_step[e] = tags;
        p.done[e] = done_now ? 1 : 0;
      }
      new_rows = true;
    }
  }

  // ---- reset: envs that are done (or all) go back to their start state ---------------------------
  if (mode & (kResetDone | kResetAll)) {
    if (valid && ((mode & kResetAll) || done_now)) {
      x = p.x0[a];
      y = p.y0[a];
      h = wrap_heading(p.h0[a], p.H);
      v = 0.0f;
      live = 1;
      dir = p.table[h];
      p.x[a] = x;
      p.y[a] = y;
      p.h[a] = h;
      p.v[a] = v;
      p.live[a] = 1;
      t_out = 0;
      if (i == 0) {
        p.t[e] = 0;
        p.n_live_runners[e] = p.N - p.N_tag;
        p.tags_step[e] = 0;
        p.done[e] = 0;
      }
      s_x[tid] = x;
      s_y[tid] = y;
      s_vx[tid] = v * dir.x;
      s_vy[tid] = v * dir.y;
      s_live[tid] = 1;
      new_rows = true;
    }
  }
  __syncthreads();

  // ---- observation rows ---------------------------------------------------------------------------
  if (!new_rows) return;
  write_row<KT>(p, p.obs + a * p.D, s_x, s_y, s_vx, s_vy, s_live, first, i, x, y, v, dir, tagger, live, t_out);
}

// Several roll-out iterations in one launch (envs never interact, and an env's agents share a
// workgroup, so no synchronisation beyond the workgroup is needed).  Between the iterations an
// agent's state stays in its thread's registers and the env's clock, live count and done flag in
// every one of its threads; iteration s draws with step g0 + s from ring entry (ring_pos + s) mod
// ring_len and writes action, reward and rows to slice s of the roll-out arrays (to the in-place
// arrays where a roll-out array is not given, and always in the last iteration); the done flags
// recorded are those before the reset.  The state arrays are written once, at the end.
struct Roll {
  int32_t steps, ring_len, ring_pos, pad;
  int32_t* action;
  float* reward;
  int32_t* done;
  float* obs;
  const float* ring;
  uint64_t g0;
};

template <int KT>
__global__ __launch_bounds__(kMaxThreads) void rollout_kernel(const Params p, const Roll roll) {
  extern __shared__ __align__(16) unsigned char smem[];
  float* const s_x = reinterpret_cast<float*>(smem);
  float* const s_y = s_x + p.threads;
  float* const s_vx = s_y + p.threads;
  float* const s_vy = s_vx + p.threads;
  int32_t* const s_live = reinterpret_cast<int32_t*>(s_vy + p.threads);
  int32_t* const s_credits = s_live + p.threads;
  int32_t* const s_tags = s_credits + p.threads;
  const int tid = threadIdx.x;
  const int el = int(wd::dev::fastdiv(uint32_t(tid), p.div_N));
  const int i = tid - el * p.N;
  const int e = blockIdx.x * p.envs_per_wg + el;
  const bool valid = el < p.envs_per_wg && e < p.E;
  const int first = el * p.N;
  const int64_t a = int64_t(valid ? e : 0) * p.N + i;
  const bool tagger = i < p.N_tag;
  const int64_t EN = int64_t(p.E) * p.N;

  float x = 0.0f, y = 0.0f, v = 0.0f;
  int h = 0, live = 0, t = 0, nlr = 0, tags_last = 0;
  bool done = false;
  if (valid) {
    x = p.x[a];
    y = p.y[a];
    v = p.v[a];
    h = wrap_heading(p.h[a], p.H);
    live = p.live[a];
    t = p.t[e];
    nlr = p.n_live_runners[e];
    tags_last = p.tags_step[e];
    done = p.done[e] != 0;
  }
  float2 dir = p.table[h];

  for (int s = 0; s < roll.steps; ++s) {
    const bool last = s + 1 == roll.steps;
    const uint64_t g = roll.g0 + uint64_t(s);
    const float* probs = roll.ring + int64_t((roll.ring_pos + s) % roll.ring_len) * EN * 10;
    int32_t* const action_out = (roll.action && !last) ? roll.action + int64_t(s) * 2 * EN : p.action;
    float* const reward_out = (roll.reward && !last) ? roll.reward + int64_t(s) * EN : p.reward;
    float* const obs_out = (roll.obs && !last) ? roll.obs + int64_t(s) * EN * p.D : p.obs;
    int2 lv = make_int2(2, 2);
    if (valid) {
      lv = draw_levels(p, load_probs(probs, a), e, i, uint32_t(g), uint32_t(g >> 32));
      *reinterpret_cast<int2*>(action_out + 2 * a) = lv;
    }
    const bool step_act = valid && !done;
    bool new_rows = false;
    if (step_act) {
      if (live == 1) advance_agent(p, tagger, lv.x, lv.y, x, y, v, h, dir);
      s_x[tid] = x;
      s_y[tid] = y;
      s_vx[tid] = v * dir.x;
      s_vy[tid] = v * dir.y;
      s_live[tid] = live;
      s_credits[tid] = 0;
      if (i == 0) s_tags[el] = 0;
    }
    __syncthreads();
    bool tagged_now = false;
    if (step_act && !tagger && live == 1 && p.tag_r2 >= 0.0f) {
      int best_t;
      if (tagger_in_range(p, s_x, s_y, first, x, y, &best_t)) {
        tagged_now = true;
        live = 0;
        s_live[tid] = 0;
        atomicAdd(&s_credits[first + best_t], 1);
        atomicAdd(&s_tags[el], 1);
      }
    }
    __syncthreads();
    if (step_act) {
      float rew = 0.0f;
      if (tagger)
        rew = static_cast<float>(s_credits[tid]) * p.tag_reward;
      else if (tagged_now)
        rew = p.tag_penalty;
      reward_out[a] = rew;
      tags_last = s_tags[el];
      nlr -= tags_last;
      t += 1;
      done = nlr == 0 || t >= p.T;
      new_rows = true;
    }
    if (roll.done && valid && i == 0) roll.done[int64_t(s) * p.E + e] = done ? 1 : 0;  // the flag before the reset
    if (valid && done) {  // back to the start state
      x = p.x0[a];
      y = p.y0[a];
      h = wrap_heading(p.h0[a], p.H);
      v = 0.0f;
      live = 1;
      dir = p.table[h];
      t = 0;
      nlr = p.N - p.N_tag;
      tags_last = 0;
      done = false;
      s_x[tid] = x;
      s_y[tid] = y;
      s_vx[tid] = v * dir.x;
      s_vy[tid] = v * dir.y;
      s_live[tid] = 1;
      new_rows = true;
    }
    __syncthreads();
    if (new_rows)
      write_row<KT>(p, obs_out + a * p.D, s_x, s_y, s_vx, s_vy, s_live, first, i, x, y, v, dir, tagger, live, t);
    __syncthreads();  // the rows are read out of LDS before the next iteration overwrites it
  }
  if (valid) {
    p.x[a] = x;
    p.y[a] = y;
    p.v[a] = v;
    p.h[a] = h;
    p.live[a] = live;
    if (i == 0) {
      p.t[e] = t;
      p.n_live_runners[e] = nlr;
      p.tags_step[e] = tags_last;
      p.done[e] = done ? 1 : 0;
    }
  }
}

}  // namespace
}  // namespace wdc

// ------------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------------
struct wdc_handle {
  wdc_config cfg;
  wdc_buffers bufs;
  wdc::Params params;
  hipStream_t stream;
  uint64_t g;
  bool started;
  void* table;
  std::string last_error;
};

namespace {

int check_config(const wdc_config* c) {
  if (!c) return WD_E_NULL;
  if (c->struct_size != sizeof(wdc_config)) return WD_E_CONFIG;
  if (c->num_envs < 1 || c->env_offset < 0) return WD_E_CONFIG;
  if (c->num_agents < 2 || c->num_agents > wdc::kMaxThreads) return WD_E_CONFIG;
  if (c->num_taggers < 1 || c->num_taggers > c->num_agents - 1) return WD_E_CONFIG;
  if (c->num_headings < 4 || c->num_headings > 4096 || c->num_headings % 4 != 0) return WD_E_CONFIG;
  if (c->episode_length < 1) return WD_E_CONFIG;
  if (c->obs_k < 0 || c->obs_k > wdc::kMaxK || c->obs_k > c->num_agents - 1) return WD_E_CONFIG;
  if (!(c->world_size > 0.0f) || std::isinf(c->world_size)) return WD_E_CONFIG;
  const float fields[] = {c->accel, c->max_speed_tagger, c->max_speed_runner, c->tag_r2, c->tag_reward, c->tag_penalty};
  for (float f : fields)
    if (!(f == f) || std::isinf(f)) return WD_E_CONFIG;
  if (c->accel < 0.0f || c->max_speed_tagger < 0.0f || c->max_speed_runner < 0.0f) return WD_E_CONFIG;
  if (int64_t(c->num_envs) * c->num_agents > int64_t(INT32_MAX) / 2) return WD_E_CONFIG;
  return WD_OK;
}

// The heading table: the first octant from double-precision cos / sin rounded to float32, the
// rest by reflection about the diagonal and by quarter turns; zeros are +0.
std::vector<float2> heading_table(int H) {
  std::vector<float2> t(H);
  const int quarter = H / 4;
  const double pi = 3.14159265358979323846;
  for (int h = 0; h < H; ++h) {
    const int turns = h / quarter;
    int r = h % quarter;
    const bool reflect = 2 * r > quarter;
    if (reflect) r = quarter - r;
    const double angle = 2.0 * pi * double(r) / double(H);
    float c = float(std::cos(angle)), s = float(std::sin(angle));
    if (2 * r == quarter) s = c;
    if (reflect) std::swap(c, s);
    for (int k = 0; k < turns; ++k) {  // a quarter turn to the left
      const float old_c = c;
      c = -s;
      s = old_c;
    }
    t[h] = make_float2(c + 0.0f, s + 0.0f);  // (-0) + 0 = +0
  }
  return t;
}

bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

int fail_hip(wdc_handle* h, hipError_t err, const char* what) {
  h->last_error = std::string(what) + ": " + hipGetErrorString(err);
  return WD_E_HIP;
}

// four float and two int arrays of one element per thread, one int per env of the workgroup
size_t lds_bytes(const wdc::Params& p) { return size_t(p.threads) * 24 + size_t(p.threads / 2) * 4; }

int launch(wdc_handle* h, int mode, const float* probs) {
  const wdc::Params& p = h->params;
  const int groups = (p.E + p.envs_per_wg - 1) / p.envs_per_wg;
  if (p.K <= 4)
    hipLaunchKernelGGL(wdc::env_kernel<4>, dim3(groups), dim3(p.threads), lds_bytes(p), h->stream, p, mode, probs,
                       uint32_t(h->g), uint32_t(h->g >> 32));
  else
    hipLaunchKernelGGL(wdc::env_kernel<wdc::kMaxK>, dim3(groups), dim3(p.threads), lds_bytes(p), h->stream, p, mode, probs,
                       uint32_t(h->g), uint32_t(h->g >> 32));
  const hipError_t err = hipGetLastError();
  if (err != hipSuccess) return fail_hip(h, err, "env_kernel launch");
  return WD_OK;
}

}  // namespace

extern "C" {

int wdc_query_layout(const wdc_config* cfg, wdc_layout* out) {
  if (!cfg || !out) return WD_E_NULL;
  const int rc = check_config(cfg);
  if (rc != WD_OK) return rc;
  const int64_t EN = int64_t(cfg->num_envs) * cfg->num_agents;
  out->obs_dim = 8 + 6 * cfg->obs_k;
  out->agent_elems = EN;
  out->action_elems = 2 * EN;
  out->obs_elems = EN * out->obs_dim;
  out->env_elems = cfg->num_envs;
  out->probs_elems = 10 * EN;
  // 40 probabilities, 20 state read, 20 state written, 8 actions, 4 reward, 4 D row; 24 per env
  out->bytes_per_iteration = EN * (40 + 20 + 20 + 8 + 4 + 4 * int64_t(out->obs_dim)) + 24 * int64_t(cfg->num_envs);
  return WD_OK;
}

int wdc_create(const wdc_config* cfg, const wdc_buffers* bufs, wdc_handle** out) {
  if (!cfg || !bufs || !out) return WD_E_NULL;
  *out = nullptr;
  const int rc = check_config(cfg);
  if (rc != WD_OK) return rc;
  const void* ptrs[] = {bufs->x, bufs->y, bufs->v, bufs->h, bufs->x0, bufs->y0, bufs->h0, bufs->live,
                        bufs->action, bufs->reward, bufs->obs, bufs->t, bufs->done, bufs->n_live_runners,
                        bufs->tags_step};
  for (const void* q : ptrs) {
    if (!q) return WD_E_NULL;
    if (!aligned(q, 256)) return WD_E_ALIGN;
  }
  wdc_handle* h = new (std::nothrow) wdc_handle();
  if (!h) return WD_E_HIP;
  h->cfg = *cfg;
  h->bufs = *bufs;
  h->stream = static_cast<hipStream_t>(cfg->stream);
  h->g = 0;
  h->started = false;
  h->table = nullptr;
  wdc::Params& p = h->params;
  p.E = cfg->num_envs;
  p.N = cfg->num_agents;
  p.N_tag = cfg->num_taggers;
  p.H = cfg->num_headings;
  p.T = cfg->episode_length;
  p.K = cfg->obs_k;
  p.D = 8 + 6 * cfg->obs_k;
  // (envs that fit a wave, in a batch of at most a quarter of a million agents: workgroups of one wave,
  // whose barriers cost nothing and which spread over more compute units)
  p.threads = (p.N <= 64 && int64_t(p.E) * p.N <= 262144) ? 64 : (p.N <= 256 ? 256 : (p.N + 63) / 64 * 64);
  p.envs_per_wg = p.threads / p.N;
  p.env_offset = uint32_t(cfg->env_offset);
  p.seed_lo = uint32_t(cfg->seed);
  p.seed_hi = uint32_t(cfg->seed >> 32);
  p.div_N = wd::make_fastdiv(uint32_t(p.N));
  p.L = cfg->world_size;
  p.inv_L = float(1.0 / double(cfg->world_size));
  p.inv_T = float(1.0 / double(cfg->episode_length));
  p.accel = cfg->accel;
  p.vmax_tagger = cfg->max_speed_tagger;
  p.vmax_runner = cfg->max_speed_runner;
  p.tag_r2 = cfg->tag_r2;
  p.tag_reward = cfg->tag_reward;
  p.tag_penalty = cfg->tag_penalty;
  p.x = bufs->x; p.y = bufs->y; p.v = bufs->v; p.h = bufs->h;
  p.x0 = bufs->x0; p.y0 = bufs->y0; p.h0 = bufs->h0;
  p.live = bufs->live; p.action = bufs->action; p.reward = bufs->reward; p.obs = bufs->obs;
  p.t = bufs->t; p.done = bufs->done; p.n_live_runners = bufs->n_live_runners; p.tags_step = bufs->tags_step;
  const std::vector<float2> table = heading_table(p.H);
  hipError_t err = hipMalloc(&h->table, sizeof(float2) * table.size());
  if (err == hipSuccess) err = hipMemcpy(h->table, table.data(), sizeof(float2) * table.size(), hipMemcpyHostToDevice);
  if (err != hipSuccess) {
    if (h->table) (void)hipFree(h->table);
    delete h;
    return WD_E_HIP;
  }
  p.table = static_cast<const float2*>(h->table);
  *out = h;
  return WD_OK;
}

int wdc_reset(wdc_handle* h, int mode) {
  if (!h) return WD_E_NULL;
  if (mode != WD_RESET_ALL && mode != WD_RESET_DONE) return WD_E_CONFIG;
  if (mode == WD_RESET_DONE) {
    if (!h->started) return WD_E_STATE;
    return launch(h, wdc::kResetDone, nullptr);
  }
  const int64_t agents = int64_t(h->params.E) * h->params.N;
  hipLaunchKernelGGL(wdc::init_kernel, dim3(uint32_t((agents + 255) / 256)), dim3(256), 0, h->stream, h->params);
  const hipError_t err = hipGetLastError();
  if (err != hipSuccess) return fail_hip(h, err, "init_kernel launch");
  h->g = 0;
  const int rc = launch(h, wdc::kResetAll, nullptr);
  if (rc == WD_OK) h->started = true;
  return rc;
}

int wdc_sample(wdc_handle* h, const float* probs) {
  if (!h || !probs) return WD_E_NULL;
  if (!aligned(probs, 8)) return WD_E_ALIGN;
  if (!h->started) return WD_E_STATE;
  return launch(h, wdc::kSample, probs);
}

int wdc_step(wdc_handle* h) {
  if (!h) return WD_E_NULL;
  if (!h->started) return WD_E_STATE;
  const int rc = launch(h, wdc::kStep, nullptr);
  if (rc == WD_OK) ++h->g;
  return rc;
}

int wdc_iterate(wdc_handle* h, const float* probs) {
  if (!h || !probs) return WD_E_NULL;
  if (!aligned(probs, 8)) return WD_E_ALIGN;
  if (!h->started) return WD_E_STATE;
  const int rc = launch(h, wdc::kSample | wdc::kStep | wdc::kResetDone, probs);
  if (rc == WD_OK) ++h->g;
  return rc;
}

int wdc_rollout(wdc_handle* h, const float* probs_ring, int ring_len, int k, const wdc_rollout_buffers* out) {
  if (!h || !probs_ring) return WD_E_NULL;
  if (ring_len < 1 || k < 1) return WD_E_CONFIG;
  if (!aligned(probs_ring, 8)) return WD_E_ALIGN;
  if (out) {
    const void* ptrs[] = {out->action, out->reward, out->done, out->obs};
    for (const void* q : ptrs)
      if (!aligned(q, 8)) return WD_E_ALIGN;
  }
  if (!h->started) return WD_E_STATE;
  const wdc::Params& p = h->params;
  wdc::Roll roll = {};
  roll.steps = k;
  roll.ring_len = ring_len;
  roll.ring_pos = int32_t(h->g % uint64_t(ring_len));
  roll.ring = probs_ring;
  roll.g0 = h->g;
  if (out) {
    roll.action = out->action;
    roll.reward = out->reward;
    roll.done = out->done;
    roll.obs = out->obs;
  }
  const int groups = (p.E + p.envs_per_wg - 1) / p.envs_per_wg;
  if (p.K <= 4)
    hipLaunchKernelGGL(wdc::rollout_kernel<4>, dim3(groups), dim3(p.threads), lds_bytes(p), h->stream, p, roll);
  else
    hipLaunchKernelGGL(wdc::rollout_kernel<wdc::kMaxK>, dim3(groups), dim3(p.threads), lds_bytes(p), h->stream, p, roll);
  hipError_t err = hipGetLastError();
  if (err != hipSuccess) return fail_hip(h, err, "rollout_kernel launch");
  if (out) {  // the last iteration wrote the in-place arrays: its slices are copies of them
    const int64_t EN = int64_t(p.E) * p.N, last = int64_t(k - 1);
    if (out->action && err == hipSuccess)
      err = hipMemcpyAsync(out->action + last * 2 * EN, h->bufs.action, size_t(2 * EN) * 4, hipMemcpyDeviceToDevice, h->stream);
    if (out->reward && err == hipSuccess)
      err = hipMemcpyAsync(out->reward + last * EN, h->bufs.reward, size_t(EN) * 4, hipMemcpyDeviceToDevice, h->stream);
    if (out->obs && err == hipSuccess)
      err = hipMemcpyAsync(out->obs + last * EN * p.D, h->bufs.obs, size_t(EN * p.D) * 4, hipMemcpyDeviceToDevice, h->stream);
    if (err != hipSuccess) return fail_hip(h, err, "copy of the last roll-out slice");
  }
  h->g += uint64_t(k);
  return WD_OK;
}

int wdc_get_step(const wdc_handle* h, uint64_t* g) {
  if (!h || !g) return WD_E_NULL;
  *g = h->g;
  return WD_OK;
}

int wdc_set_step(wdc_handle* h, uint64_t g) {
  if (!h) return WD_E_NULL;
  h->g = g;
  return WD_OK;
}

int wdc_destroy(wdc_handle* h) {
  if (!h) return WD_OK;
  if (h->table) (void)hipFree(h->table);
  delete h;
  return WD_OK;
}

const char* wdc_last_error(const wdc_handle* h) { return h ? h->last_error.c_str() : ""; }

}  // extern "C"
