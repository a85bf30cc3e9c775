// wd_api.hip — host side of libwd: the C ABI of include/wd.h, configuration checks,
// launch geometry and LDS map, and the calls into the launchers of wd_kernels.hip.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstring>
#include <new>
#include <string>

#include "../../include/wd.h"
#include "wd_internal.h"

struct wd_handle {
  wd_config cfg;
  wd_buffers bufs;
  wd::Params params;
  hipStream_t stream;
  uint64_t g;          // global step: RNG step index
  bool started;        // wd_reset(WD_RESET_ALL) has run
  bool rows_valid;     // bufs.obs holds the rows this library wrote for the current state
  void* scratch;       // device memory of the large-env tables (NULL for the small layout)
  int spread_parity;   // spread form of the large-env pair: the set of accumulators the next stepping call uses
  // roll-outs of the large-env layout: a second stream for the observation kernels, a second
  // table image and two events per image (created by the first such roll-out, freed by wd_destroy)
  hipStream_t obs_stream;
  hipEvent_t tables_ready[2], rows_done[2];
  void* second_image;
  bool pipe_ready;
  std::string last_error;
};

namespace {

// LDS of one gfx950 compute unit, less the 256 bytes of static LDS the env kernels carry (the
// workgroup votes of __syncthreads_and / __syncthreads_or): what a launch may ask for dynamically
constexpr int64_t kLdsLimitBytes = 160 * 1024 - 256;
constexpr int kMaxAgents = 32768;
constexpr int kMaxGrid = 32767;
// spread form of the large-env pair: while its observation kernel has a compute unit per workgroup to spare
constexpr int kSpreadMaxWorkgroups = 192;
constexpr int kSpreadMinAgents = 1024;
// envs: one round of waves on the chip (256 compute units x 32 waves).  Measured, us per wd_iterate, wave per env / general
// kernel: 8192 envs x 50 agents 22.6 / 27.7, 8192 x 32 16.3 / 23.1; beyond one round 20000 x 16 20.5 / 26.4, but 20000 x 50
// 46.9 / 41.3, 20000 x 64 58.1 / 39.0 and 50000 x 5 38.5 / 32.8 (a wave for five agents)
constexpr int kWaveEnvsMaxBatch = 8192;

int bits_for(uint32_t v) {  // bits needed to hold values 0..v
  int b = 1;
  while ((uint64_t(1) << b) <= v) ++b;
  return b;
}

uint32_t pow2_ceil(uint32_t v) {
  uint32_t r = 1;
  while (r < v) r <<= 1;
  return r;
}

int32_t isqrt64(int64_t v) {
  int64_t r = int64_t(std::sqrt(double(v)));
  while (r * r > v) --r;
  while ((r + 1) * (r + 1) <= v) ++r;
  return int32_t(r);
}

int64_t align16(int64_t v) { return (v + 15) & ~int64_t(15); }

int check_config(const wd_config* c) {
  if (!c) return WD_E_NULL;
  if (c->struct_size != sizeof(wd_config)) return WD_E_CONFIG;
  if (c->num_envs < 1 || c->env_offset < 0) return WD_E_CONFIG;
  if (int64_t(c->num_envs) + int64_t(c->env_offset) > int64_t(INT32_MAX)) return WD_E_CONFIG;
  if (c->num_agents < 2 || c->num_agents > kMaxAgents) return WD_E_CONFIG;
  if (c->num_taggers < 1 || c->num_taggers > c->num_agents - 1) return WD_E_CONFIG;
  if (c->grid_size < 1 || c->grid_size > kMaxGrid) return WD_E_CONFIG;
  if (c->num_actions != wd::kNumActions) return WD_E_CONFIG;
  if (c->episode_length < 1) return WD_E_CONFIG;
  if (c->obs_mode != WD_OBS_PARTIAL && c->obs_mode != WD_OBS_FULL) return WD_E_CONFIG;
  if (c->obs_mode == WD_OBS_PARTIAL && (c->obs_k < 0 || c->obs_k > c->num_agents - 1)) return WD_E_CONFIG;
  if (!(c->tag_reward == c->tag_reward) || !(c->tag_penalty == c->tag_penalty)) return WD_E_CONFIG;  // NaN
  if (int64_t(c->num_envs) * c->num_agents > int64_t(INT32_MAX)) return WD_E_CONFIG;
  return WD_OK;
}

int32_t obs_dim(const wd_config* c) {
  return c->obs_mode == WD_OBS_PARTIAL ? 5 + 4 * c->obs_k : 5 + 4 * c->num_agents;
}

bool aligned256(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 255u) == 0; }

// probs is read with aligned 16-byte loads when N % 4 == 0, else with loads that need 4-byte alignment
bool probs_aligned(const wd::Params& p, const void* probs) {
  return (reinterpret_cast<uintptr_t>(probs) & (p.vec4 ? 15u : 3u)) == 0;
}

// LDS map of the strip variant: per team a kept part (positions by index, scalars, strip edges),
// an X part (the padded strip-sorted list and the table of bin starts) that the row staging area
// overlays once the neighbour search is done, and a Y part (slots, tag keys, credits) that the
// retry queue and the neighbour lists overlay once the rewards are out.  The columns are as narrow
// as the table's share of LDS allows without costing the launch a workgroup per CU.
bool plan_strip_layout(const wd_config& c, wd::Params* p) {
  const int N = c.num_agents, G = c.grid_size, K = p->K;
  const int64_t NPAD = p->NPAD;
  const int tpw = p->teams_per_wg;
  // strips about 1.5 expected K-th-neighbour distances tall: G / R = 1.5 G sqrt(K / (pi n))
  p->strip_scale = float(std::sqrt(3.14159265358979 / double(K)) / 1.5);
  // the own window overhangs the list by up to its half width, and the window of a neighbouring strip then sits beyond it
  p->pad_l = wd::strip_pad(K);
  p->pad_r = wd::strip_pad(K);
  const int64_t slots = NPAD + p->pad_l + p->pad_r;
  const int r_want = std::min<int64_t>(G, int64_t(std::ceil(double(p->strip_scale) * std::sqrt(double(N)))) + 1);
  const int64_t waves = p->wg_size / wd::kWaveSize;
  int srl = 5;  // rows per wave and flush of the staging area: 32, or 16 if an env does not fit otherwise
  const int64_t nbr_bytes = align16((K == 4 && N < 1024) ? 5 * NPAD : 2 * NPAD * K);
  const int64_t retry_bytes = align16(2 * NPAD);
  auto layout = [&](int cshift, bool commit) -> int64_t {
    const int64_t stage = waves * (int64_t(1) << srl) * p->D * 4;
    const int C = ((G - 1) >> cshift) + 1;
    const int64_t entries = int64_t(r_want) * C + 1;
    int64_t off = 0;
    auto take = [&off](int64_t bytes) {
      const int64_t at = off;
      off = align16(off + bytes);
      return int32_t(at);
    };
    const int32_t o_pl = take(4 * NPAD), o_misc = take(128), o_edges = take(2 * (r_want + 2));
    const int64_t keep = off;
    off = 0;
    const int32_t o_sorted = take(4 * slots), o_id = take(2 * slots), o_t = take(2 * (entries + 1));
    const int64_t x_stride = off;
    off = 0;
    const int32_t o_slot = take(2 * NPAD), o_best = take(4 * NPAD), o_credits = take(4ll * c.num_taggers);
    const int64_t y_tables = off;
    const int64_t x_area = x_stride * tpw;
    int64_t x_span, y_stride;
    if (tpw == 1) {
      x_span = x_area;
      y_stride = align16(std::max<int64_t>(std::max<int64_t>(y_tables, retry_bytes + nbr_bytes), stage + nbr_bytes - x_area));
    } else {
      x_span = std::max<int64_t>(x_area, stage);
      y_stride = align16(std::max<int64_t>(y_tables, retry_bytes + nbr_bytes));
    }
    const int64_t total = keep * tpw + x_span + y_stride * tpw;
    if (commit) {
      p->cshift = cshift;
      p->strip_C = C;
      p->strip_rmax = r_want;
      p->off_pl = o_pl;
      p->off_misc = o_misc;
      p->off_edges = o_edges;
      p->keep_stride = int32_t(keep);
      p->off_sorted = o_sorted + 4 * p->pad_l;
      p->off_sorted_id = o_id + 2 * p->pad_l;
      p->off_starts = o_t;
      p->x_stride = int32_t(x_stride);
      p->off_slot = o_slot;
      p->off_best = o_best;
      p->off_credits = o_credits;
      p->off_counts = 0;
      p->off_retry = 0;
      p->compact_nbr = (K == 4 && N < 1024) ? 1 : 0;
      p->stage_rows_log2 = srl;
      p->y_stride = int32_t(y_stride);
      p->off_nbr = int32_t(y_stride - nbr_bytes);
      p->x_base = int32_t(keep * tpw);
      p->y_base = int32_t(p->x_base + x_span);
      p->lds_bytes = int32_t(std::min<int64_t>(total, INT32_MAX));
      p->g_stride_image = p->y_base;
    }
    return total;
  };
  // the share of LDS that keeps as many workgroups on a CU as the coarsest columns would
  int64_t total_min = layout(15, false);
  if (total_min > kLdsLimitBytes) {
    srl = 4;
    total_min = layout(15, false);
  }
  if (total_min > kLdsLimitBytes) return false;
  const int64_t by_threads = std::max<int64_t>(1, 2048 / p->wg_size);
  const int64_t wgs = std::max<int64_t>(1, std::min<int64_t>(by_threads, kLdsLimitBytes / total_min));
  const int64_t budget = kLdsLimitBytes / wgs;
  int cshift = 0;
  while (cshift < 15 && layout(cshift, false) > budget) ++cshift;
  layout(cshift, true);
  return true;
}

// Launch geometry and LDS map of the env-per-team kernels.  Returns false if an env does
// not fit one workgroup's LDS.
// (`big_tables_in_lds`: a large env also keeps slots, tag keys and credits in LDS when they fit)
bool plan_env_kernels(const wd_config& c, wd::Params* p, bool big, bool big_tables_in_lds = false) {
  const int N = c.num_agents, G = c.grid_size;
  p->NG = (N + 3) / 4;
  p->big = big ? 1 : 0;
  int ts_log2 = 3;
  while ((1 << ts_log2) < p->NG && ts_log2 < 8) ++ts_log2;
  // A batch that cannot fill the chip is bound by the latency of one workgroup's chain of
  // phases, not by throughput: give each env more lanes (fewer search rounds per lane) and each
  // workgroup fewer envs (fewer row chunks per wave) while that still shortens the chain.
  while (!big && ts_log2 < 8) {
    const int ts_now = 1 << ts_log2, tpw_now = 256 / ts_now;
    const int64_t waves_if_doubled = int64_t(c.num_envs) * std::max(1, 2 * ts_now / wd::kWaveSize);
    const int64_t rows_per_wg = int64_t(std::min(tpw_now, c.num_envs)) * N;
    // 8192 wave slots on the chip: beyond that, wider teams only add rounds of workgroups
    // (and up to a whole wave per team in any case: the strip search serves the teams of a wave one
    // after the other; a batch of at most one workgroup per CU gets a workgroup per env, whose
    // kernel variant keeps everything that depends on the team in scalar registers:
    // 10 envs x 5 agents 13.1 -> 11.7 us per iteration, 11.6 -> 8.1 inside a roll-out)
    const int min_width = c.num_envs <= 256 ? 256 : wd::kWaveSize;
    if (waves_if_doubled > 8192 || (rows_per_wg <= 64 && N <= ts_now && ts_now >= min_width)) break;
    ++ts_log2;
  }
  p->wg_size = 256;
  // An env of more than 1024 agents takes more LDS than lets eight 256-thread workgroups share
  // a CU: wider workgroups keep the CU's wave slots filled.  Measured at E = 2000, us per
  // iteration with 256 / 512 / 1024 threads: N = 1100 105 / 92 / -, N = 2000 249 / 218 / -,
  // N = 3000 443 / 338 / 462, N = 3500 840 / 586 / 526, N = 4000 887 / 644 / 584.
  if (!big && N > 1024) {
    ts_log2 = N > 3072 ? 10 : 9;
    p->wg_size = 1 << ts_log2;
  }
  if (big) {  // one env per 1024-thread workgroup
    ts_log2 = 10;
    p->wg_size = wd::kBigEnvWorkgroupSize;
  }
  const int ts = 1 << ts_log2;
  p->ts_log2 = ts_log2;
  p->teams_per_wg = p->wg_size / ts;
  p->gpt = (p->NG + ts - 1) / ts;
  p->NPAD = (4 * p->NG + 7) / 8 * 8;
  p->vec4 = (N % 4 == 0) ? 1 : 0;
  uint32_t nb_cap = pow2_ceil(uint32_t(N)) / 2;
  if (nb_cap > 4096u) nb_cap = 4096u;
  if (nb_cap < uint32_t(ts)) nb_cap = uint32_t(ts);
  if (nb_cap < 16u) nb_cap = 16u;
  p->nb_cap = int32_t(nb_cap);
  p->scan_chunk = int32_t(nb_cap) / ts;
  // buckets are 65536 / mul cells wide; the table holds nbx^2 <= nb_cap of them
  uint32_t side = 1;
  while ((side + 1) * (side + 1) <= nb_cap) ++side;
  // largest mul with ((G - 1) * mul >> 16) + 1 <= side
  uint32_t mul_max = 65536u;
  if (G > 1) mul_max = uint32_t(std::min<uint64_t>(65536u, ((uint64_t(side) << 16) - 1) / uint64_t(G - 1)));
  p->bucket_mul_max = mul_max;
  p->bucket_scale = float(65536.0 / double(G));
  // target live agents per bucket: about 5 in an env of a hundred agents, 2.2 from five hundred on
  // (with every agent of the headline shape in play: 80.2 us per iteration at 1.5 .. 2.0, where the
  // size of the bucket table sets the width, 78.2 at 2.2, 78.9 at 2.6, 80.9 at 3.0)
  p->lambda_c = 47.0f;
  p->lambda_min = 2.2f;
  p->lambda_max = 5.0f;
  if (ts >= N) {  // a lane per agent: one search round, so fewer, fuller buckets shorten the chain
    p->lambda_c = 70.0f;
    p->lambda_max = 8.0f;
  }
  if (p->K > 4) {  // more neighbours wanted: the 3x3 block of the first pass has to hold more agents
    const float ks = float(p->K) / 4.0f;
    p->lambda_c *= ks;
    p->lambda_min *= ks;
    p->lambda_max *= ks;
  }
  p->div_N = wd::make_fastdiv(uint32_t(N));
  p->div_NG = wd::make_fastdiv(uint32_t(p->NG));

  // (distance, index) keys and bucket entries: 32 bits when they fit, else 64
  p->idx_bits = bits_for(uint32_t(N - 1));
  p->xy_bits = bits_for(uint32_t(G - 1));
  const uint64_t d2max = 2ull * uint64_t(G - 1) * uint64_t(G - 1);
  // 32-bit form: live keys stay below 2^31, and a dead mark (x + dead_dx) exists that puts the
  // squared distance of a marked entry from any grid cell into [2^(31-ib), 2^(32-ib))
  bool narrow = false;
  p->dead_dx = 0;
  if (p->idx_bits <= 16) {
    const uint64_t band = 1ull << (31 - p->idx_bits);
    uint64_t lo = uint64_t(std::sqrt(double(band)));
    while (lo * lo < band) ++lo;
    const uint64_t shift = lo + uint64_t(G - 1);
    const uint64_t far = shift + uint64_t(G - 1);
    if (d2max + 1 <= band && far <= 32767 && far * far + uint64_t(G - 1) * uint64_t(G - 1) < 2 * band) {
      narrow = true;
      p->dead_dx = int32_t(shift);
    }
  }
  // The variants with 32-bit keys and K = 1 .. 8 compiled in (small layout) sort by strip and keep the
  // positions of that list scaled by 2^h per axis (2 h >= idx_bits), so that the squared length of a
  // packed 16-bit difference is the key's distance part where it belongs; an entry out of play has y
  // field 0x7FFF.  That needs room in 16 bits: the keys of such entries, at least (32767 - A)^2 with
  // A = (G - 1) << h, must lie above every key of a live pair, below 2 A^2 + 2^(2 h).  Larger grids
  // take 64-bit keys and the bucket rings.
  if (narrow && !big && c.obs_mode == WD_OBS_PARTIAL && p->K >= 1 && p->K <= wd::kMaxRegisterK) {
    const int h = (p->idx_bits + 1) / 2;
    const int64_t A = int64_t(G - 1) << h;
    const int64_t dead_min = A < 32767 ? (32767 - A) * (32767 - A) : 0;
    if (A < 32767 && 2 * A * A + (int64_t(1) << (2 * h)) <= dead_min) {
      p->pos_shift = h;
      p->key_shift = 2 * h;
      p->dead_key_min = uint32_t(dead_min);
    } else {
      narrow = false;
    }
  }
  // Else, in the large-env layout: keys that need all 32 bits, the dead mark moved into bit 15
  // of the index array.  Else 64-bit keys.
  const bool flagged32 = !narrow && big && p->idx_bits <= 15 && G <= 32767 &&
                         p->idx_bits + bits_for(uint32_t(d2max)) <= 32 &&
                         ((d2max << p->idx_bits) | uint64_t(N - 1)) < 0xFFFFFFFFull;  // all ones = "none"
  if (flagged32) narrow = true;  // the same table layout as the 31-bit form
  p->wide = flagged32 ? 2 : (narrow ? 0 : 1);
  const int key_bytes = narrow ? 4 : 8;
  const bool register_path = c.obs_mode == WD_OBS_PARTIAL && p->K <= wd::kMaxRegisterK2;
  // The variants with 32-bit keys and K compiled in (small layout) sort by strip and column
  // instead of by square bucket (wd_dev_strips.h).
  p->strips = (!big && p->wide == 0 && c.obs_mode == WD_OBS_PARTIAL && p->K >= 1 && p->K <= wd::kMaxRegisterK) ? 1 : 0;
  if (p->strips) return plan_strip_layout(c, p);

  int64_t off = 0;
  auto take = [&off](int64_t bytes) {
    const int64_t at = off;
    off = align16(off + bytes);
    return int32_t(at);
  };
  const int64_t NPAD = p->NPAD;
  const int tpw = p->teams_per_wg;
  p->off_pl = take(4 * NPAD);
  p->off_misc = take(128);
  p->off_edges = take(2 * (side + 2));
  p->keep_stride = int32_t(off);
  off = 0;
  p->off_sorted = take((narrow ? 4 : 8) * (NPAD + 4));
  p->off_sorted_id = take(narrow ? 2 * (NPAD + 4) : 0);
  p->off_starts = take(2ll * (nb_cap + 4));
  p->x_stride = int32_t(off);
  off = 0;
  p->big_lds_tables = (big && big_tables_in_lds) ? 1 : 0;
  if (!big || big_tables_in_lds) {
    p->off_slot = take(2 * NPAD);
    p->off_best = take(key_bytes * NPAD);
    p->off_credits = take(4ll * c.num_taggers);
  }
  p->off_counts = take(4ll * nb_cap);
  // slots of the second search pass: over slot[] (not needed any more by then), which the
  // neighbour lists therefore must not overlay; a large env has no slot[] in LDS
  p->off_retry = 0;  // (a large env searches in its observation kernel, which needs no second pass)
  const int64_t retry_bytes = (big || !register_path) ? 0 : align16(2 * NPAD);
  const int64_t y_tables = off;
  // neighbour lists: K 16-bit ids per agent, or 40 bits per agent when K = 4 and ids fit 10 bits
  p->compact_nbr = (!big && narrow && p->K == 4 && N < 1024) ? 1 : 0;
  const int64_t nbr_bytes = (!register_path || big) ? 0 : align16(p->compact_nbr ? 5 * NPAD : 2 * NPAD * p->K);
  // per-env strides of the tables a large env keeps in device memory
  p->g_stride_agents = NPAD;
  p->g_stride_credits = (c.num_taggers + 3) / 4 * 4;
  // observation kernel of a large env: about one search per thread
  p->big_slices = std::max(1, std::min(64, (N + wd::kBigObsWorkgroupSize - 1) / wd::kBigObsWorkgroupSize));
  // The staging area of the rows (32 or 16 rows per wave and flush) overlays the X parts and,
  // in a one-team workgroup, the head of the Y part in front of the neighbour lists.
  const int64_t x_area = int64_t(p->x_stride) * tpw;
  const int64_t waves = p->wg_size / wd::kWaveSize;
  const int64_t stage32 = register_path ? waves * 32 * p->D * 4 : 0;
  const int64_t stage16 = register_path ? waves * 16 * p->D * 4 : 0;
  auto plan_with = [&](int64_t stage, int64_t* x_span, int64_t* y_stride) {
    if (tpw == 1) {
      *x_span = x_area;
      *y_stride = align16(std::max<int64_t>(std::max<int64_t>(y_tables, retry_bytes + nbr_bytes), stage + nbr_bytes - x_area));
    } else {
      *x_span = std::max<int64_t>(x_area, stage);
      *y_stride = align16(std::max<int64_t>(y_tables, retry_bytes + nbr_bytes));
    }
    return p->keep_stride * int64_t(tpw) + *x_span + *y_stride * tpw;
  };
  int64_t xs32, ys32, xs16, ys16;
  const int64_t total32 = plan_with(stage32, &xs32, &ys32);
  const int64_t total16 = plan_with(stage16, &xs16, &ys16);
  // 32 rows: whole 64-row chunks then leave through the path without bounds tests, which is
  // worth more than the workgroup per CU that the larger staging area can cost (measured at 100
  // agents per env: 6 workgroups per CU with 32 rows beat 7 with 16); 16 rows only if 32 do not fit
  const bool use32 = total32 <= kLdsLimitBytes;
  (void)total16;
  p->stage_rows_log2 = use32 ? 5 : 4;
  const int64_t x_span = use32 ? xs32 : xs16;
  p->y_stride = int32_t(use32 ? ys32 : ys16);
  p->off_nbr = int32_t(p->y_stride - nbr_bytes);
  p->x_base = p->keep_stride * tpw;
  p->y_base = int32_t(p->x_base + x_span);
  const int64_t total = int64_t(p->y_base) + int64_t(p->y_stride) * tpw;
  p->lds_bytes = int32_t(std::min<int64_t>(total, INT32_MAX));
  p->g_stride_image = p->y_base;  // kept part + sorted part, a multiple of 16 bytes
  return total <= kLdsLimitBytes;
}

// Spread form of the large-env pair.  The pair's first kernel runs one workgroup per env, so a
// batch of a few envs leaves most of the chip idle through seven phases of one workgroup's
// latency; the spread form gives every 512 agents a workgroup for the move and the tag check
// and lets every slice of the second kernel build the env's tables itself.  It pays while the
// batch has far fewer slices than the chip has compute units.  Measured, us per iteration, one
// workgroup per env -> spread (K = 4, a tenth of the agents taggers): 10 envs x 500 agents
// 21.4 -> 21.5, 10 x 2000 24.8 -> 23.8, 10 x 8192 35.9 -> 29.1, 32 x 2000 25.5 -> 25.2,
// 64 x 2000 27.2 -> 27.8, 64 x 4096 35.7 -> 47.2, 128 x 2000 31.3 -> 41.9.
void plan_spread(const wd_config& c, wd::Params* p) {
  p->big_spread = 0;
  if (!p->big || c.num_taggers > wd::kSpreadMaxTaggers || c.num_agents < kSpreadMinAgents ||
      int64_t(c.num_envs) * p->big_slices > kSpreadMaxWorkgroups)
    return;
  p->big_spread = 1;
  // The second kernel's slices: as many as the chip has compute units for, down to 256 agents each (every
  // slice sorts the whole env, so narrower slices only shorten the search and the row stores:
  // tag_10x8192 with 12 / 16 / 20 / 25 slices per env: 30.6 / 28.6 / 28.2 / 28.0 us per iteration).
  p->big_slices = std::max<int64_t>(p->big_slices, std::min<int64_t>(std::min<int64_t>(64, c.num_agents / 256), 250 / c.num_envs));
  p->spread_slices = (p->NG + wd::kSpreadMoveThreads - 1) / wd::kSpreadMoveThreads;
  // coarse cells of the taggers' table: at least a tag radius wide, so that a runner looks at no
  // more than three per axis, and at most kSpreadTagSide per grid side
  const int64_t width = std::max<int64_t>(std::max<int64_t>(p->tag_rad, 1),
                                          (c.grid_size + wd::kSpreadTagSide - 1) / wd::kSpreadTagSide);
  p->tag_mul = uint32_t(std::max<int64_t>(1, 65536 / width));
  p->tag_nbx = int32_t((uint64_t(c.grid_size - 1) * p->tag_mul) >> 16) + 1;
  p->acc_credits = 0;
  p->acc_tags = int32_t(p->g_stride_credits);
  p->g_stride_acc = (p->acc_tags + 1 + 3) / 4 * 4;
}

int fill_params(const wd_config& c, const wd_buffers& b, wd::Params* p) {
  std::memset(p, 0, sizeof(*p));
  p->E = c.num_envs;
  p->N = c.num_agents;
  p->N_tag = c.num_taggers;
  p->G = c.grid_size;
  p->T = c.episode_length;
  const int64_t d2max = 2ll * int64_t(c.grid_size - 1) * int64_t(c.grid_size - 1);
  p->tag_r2 = c.tag_r2 < 0 ? -1 : int32_t(std::min<int64_t>(c.tag_r2, d2max));  // beyond d2max everything is in range
  p->tag_rad = c.tag_r2 < 0 ? 0 : isqrt64(p->tag_r2);
  p->K = c.obs_mode == WD_OBS_PARTIAL ? c.obs_k : 0;
  p->D = obs_dim(&c);
  p->obs_mode = c.obs_mode;
  p->env_offset = uint32_t(c.env_offset);
  p->seed_lo = uint32_t(c.seed);
  p->seed_hi = uint32_t(c.seed >> 32);
  p->tag_reward = c.tag_reward;
  p->tag_penalty = c.tag_penalty;
  p->inv_G = float(1.0 / double(c.grid_size));
  p->inv_T = float(1.0 / double(c.episode_length));
  p->pos_x = b.pos_x;
  p->pos_y = b.pos_y;
  p->pos_x0 = b.pos_x0;
  p->pos_y0 = b.pos_y0;
  p->live = b.live;
  p->action = b.action;
  p->reward = b.reward;
  p->obs = b.obs;
  p->t = b.t;
  p->done = b.done;
  p->n_live_runners = b.n_live_runners;
  p->tags_step = b.tags_step;
  // Two layouts serve an env: one workgroup with every table in LDS, or the large-env pair of
  // kernels (a 1024-thread workgroup for the step, then the neighbour search spread over many
  // workgroups).  The pair costs a second launch and a round trip of the tables through device
  // memory, but puts a whole chip on the search of a few envs, so it wins while the batch is too
  // small to fill the chip with one workgroup per env.  Measured crossovers (partial
  // observations, K = 4, us per iteration one workgroup -> pair): E = 10: N = 500 26 -> 22,
  // N = 2000 64 -> 26, N = 6000 158 -> 36; E = 320: N = 1000 39 -> 45, N = 2000 82 -> 66,
  // N = 4000 133 -> 114; E = 640: N = 2000 92 -> 106, N = 4000 215 -> 226, N = 6000 306 -> 381.
  const bool pair_serves = c.obs_mode == WD_OBS_PARTIAL && p->K <= wd::kMaxRegisterK2;
  const int64_t pair_up_to = c.num_agents <= 1024 ? 3ll * c.num_agents / 10 : 450;  // envs
  const bool prefer_pair = pair_serves && c.num_agents >= 384 && c.num_envs <= pair_up_to;
  const wd::Params filled = *p;
  bool planned = prefer_pair && plan_env_kernels(c, p, true, true);
  if (!planned && prefer_pair) {
    *p = filled;
    planned = plan_env_kernels(c, p, true);
  }
  if (!planned) {
    *p = filled;
    planned = plan_env_kernels(c, p, false);
  }
  if (!planned && !prefer_pair) {
    *p = filled;
    planned = plan_env_kernels(c, p, true, true);
    if (!planned) {
      *p = filled;
      planned = plan_env_kernels(c, p, true);
    }
  }
  if (!planned || !wd::env_kernel_available(*p)) return WD_E_UNSUPPORTED;
  plan_spread(c, p);
  // Envs that fit a wave, in a batch that cannot fill the chip anyway: a wave per env, a lane per agent
  // (keys of 32 bits: squared distance << 6 | index).
  p->wave_envs = (!p->big && c.num_agents <= wd::kWaveSize && c.num_envs <= kWaveEnvsMaxBatch &&
                  c.obs_mode == WD_OBS_PARTIAL && p->K <= wd::kMaxRegisterK2 && c.grid_size <= 4096)
                     ? 1
                     : 0;
  return WD_OK;
}

int hip_failed(wd_handle* h, hipError_t err, const char* what) {
  h->last_error = std::string(what) + ": " + hipGetErrorString(err);
  return WD_E_HIP;
}

// Work tables of the large-env layout (slots, tag keys, credits and the table image of every env):
// total bytes, and the pointers into one block of that size.
int64_t place_big_tables(wd::Params* p, int64_t E, unsigned char* base) {
  const int64_t key_bytes = p->wide == 1 ? 8 : 4;
  const int64_t slot_b = align16(2 * p->g_stride_agents * E), best_b = align16(key_bytes * p->g_stride_agents * E);
  const int64_t cred_b = align16(4 * p->g_stride_credits * E), image_b = p->big_spread ? 0 : p->g_stride_image * E;
  // spread form: packed positions, the envs' scalars and the two sets of accumulators
  const int64_t pl_b = p->big_spread ? align16(4 * p->g_stride_agents * E) : 0;
  const int64_t env_b = p->big_spread ? 16 * E : 0;
  const int64_t acc_b = p->big_spread ? 2 * 4 * p->g_stride_acc * E : 0;
  if (base) {
    p->g_best = base;
    p->g_credits = reinterpret_cast<int32_t*>(base + best_b);
    p->g_slot = reinterpret_cast<uint16_t*>(base + best_b + cred_b);
    p->g_image = base + best_b + cred_b + slot_b;
    unsigned char* at = p->g_image + image_b;
    p->g_pl = reinterpret_cast<uint32_t*>(at);
    p->g_env = reinterpret_cast<int32_t*>(at + pl_b);
    p->g_acc = reinterpret_cast<uint32_t*>(at + pl_b + env_b);
  }
  return slot_b + best_b + cred_b + image_b + pl_b + env_b + acc_b;
}

// What a roll-out of the large-env layout needs to run the observation kernel of one iteration
// beside the step kernel of the next: a stream of default priority, events, a second table image.
int ensure_pipe(wd_handle* h) {
  if (h->pipe_ready) return WD_OK;
  hipError_t err = hipStreamCreateWithFlags(&h->obs_stream, hipStreamNonBlocking);
  if (err != hipSuccess) return hip_failed(h, err, "stream for the observation kernels");
  for (int b = 0; b < 2 && err == hipSuccess; ++b) {
    err = hipEventCreateWithFlags(&h->tables_ready[b], hipEventDisableTiming);
    if (err == hipSuccess) err = hipEventCreateWithFlags(&h->rows_done[b], hipEventDisableTiming);
  }
  if (err == hipSuccess) err = hipMalloc(&h->second_image, size_t(h->params.g_stride_image) * size_t(h->params.E));
  if (err != hipSuccess) return hip_failed(h, err, "events and second table image of a roll-out");
  h->pipe_ready = true;
  return WD_OK;
}

// The work tables of wd_iterate_static: one array per device, held until the process ends.
constexpr size_t kStaticScratchBytes = size_t(WD_STATIC_SCRATCH_BYTES);
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each device, once asked for

}  // namespace

extern "C" {

int wd_query_layout(const wd_config* cfg, wd_layout* out) {
  if (!cfg || !out) return WD_E_NULL;
  const int rc = check_config(cfg);
  if (rc != WD_OK) return rc;
  const int64_t E = cfg->num_envs, N = cfg->num_agents, D = obs_dim(cfg);
  out->obs_dim = int32_t(D);
  out->per_agent_elems = E * N;
  out->obs_elems = E * N * D;
  out->per_env_elems = E;
  out->probs_elems = E * N * wd::kNumActions;
  out->bytes_per_iteration = E * N * (4 * wd::kNumActions + 36 + 4 * D) + 24 * E;
  return WD_OK;
}

int wd_create(const wd_config* cfg, const wd_buffers* bufs, wd_handle** out) {
  if (!cfg || !bufs || !out) return WD_E_NULL;
  *out = nullptr;
  int rc = check_config(cfg);
  if (rc != WD_OK) return rc;
  const void* ptrs[] = {bufs->pos_x, bufs->pos_y, bufs->pos_x0, bufs->pos_y0, bufs->live, bufs->action,
                        bufs->reward, bufs->obs, bufs->t, bufs->done, bufs->n_live_runners, bufs->tags_step};
  for (const void* ptr : ptrs)
    if (!ptr) return WD_E_NULL;
  for (const void* ptr : ptrs)
    if (!aligned256(ptr)) return WD_E_ALIGN;
  wd::Params params;
  rc = fill_params(*cfg, *bufs, &params);
  if (rc != WD_OK) return rc;
  wd_handle* h = new (std::nothrow) wd_handle();
  if (!h) return WD_E_NULL;
  h->scratch = nullptr;
  if (params.big) {
    // large envs: slots, tag keys, credits and the table image of every env, in one allocation
    if (hipMalloc(&h->scratch, size_t(place_big_tables(&params, cfg->num_envs, nullptr))) != hipSuccess) {
      (void)hipGetLastError();
      delete h;
      return WD_E_HIP;
    }
    place_big_tables(&params, cfg->num_envs, static_cast<unsigned char*>(h->scratch));
    if (params.big_spread &&  // both sets of accumulators start clear
        hipMemset(params.g_acc, 0, size_t(2 * 4 * params.g_stride_acc) * size_t(cfg->num_envs)) != hipSuccess) {
      (void)hipGetLastError();
      (void)hipFree(h->scratch);
      delete h;
      return WD_E_HIP;
    }
  }
  h->spread_parity = 0;
  h->cfg = *cfg;
  h->bufs = *bufs;
  h->params = params;
  h->stream = static_cast<hipStream_t>(cfg->stream);
  h->g = 0;
  h->started = false;
  h->rows_valid = false;
  h->obs_stream = nullptr;
  h->second_image = nullptr;
  h->pipe_ready = false;
  *out = h;
  return WD_OK;
}

int wd_reset(wd_handle* h, int mode) {
  if (!h) return WD_E_NULL;
  if (mode != WD_RESET_ALL && mode != WD_RESET_DONE) return WD_E_CONFIG;
  if (mode == WD_RESET_DONE && !h->started) return WD_E_STATE;
  hipError_t err;
  if (mode == WD_RESET_ALL) {
    err = wd::launch_init_start_positions(h->params, h->stream);
    if (err != hipSuccess) return hip_failed(h, err, "start-position kernel");
    err = wd::launch_env_kernel(h->params, wd::kModeResetAll, nullptr, 0, h->stream);
    if (err != hipSuccess) return hip_failed(h, err, "reset kernel");
    h->g = 0;
    h->started = true;
    h->rows_valid = true;
    return WD_OK;
  }
  err = wd::launch_env_kernel(h->params, wd::kModeResetDone, nullptr, 0, h->stream);
  if (err != hipSuccess) return hip_failed(h, err, "reset kernel");
  return WD_OK;
}

int wd_sample(wd_handle* h, const float* probs) {
  if (!h || !probs) return WD_E_NULL;
  if (!probs_aligned(h->params, probs)) return WD_E_ALIGN;
  if (!h->started) return WD_E_STATE;
  const hipError_t err = wd::launch_sample(h->params, probs, h->g, h->stream);
  if (err != hipSuccess) return hip_failed(h, err, "sample kernel");
  return WD_OK;
}

int wd_step(wd_handle* h) {
  if (!h) return WD_E_NULL;
  if (!h->started) return WD_E_STATE;
  wd::Params q = h->params;
  q.rows_kept = h->rows_valid ? 1 : 0;
  q.spread_parity = h->spread_parity;
  const hipError_t err = wd::launch_env_kernel(q, wd::kModeStep, nullptr, h->g, h->stream);
  if (err != hipSuccess) return hip_failed(h, err, "step kernel");
  h->spread_parity ^= 1;
  h->rows_valid = true;
  h->g += 1;
  return WD_OK;
}

int wd_iterate(wd_handle* h, const float* probs) {
  if (!h || !probs) return WD_E_NULL;
  if (!probs_aligned(h->params, probs)) return WD_E_ALIGN;
  if (!h->started) return WD_E_STATE;
  wd::Params q = h->params;
  q.rows_kept = h->rows_valid ? 1 : 0;
  q.spread_parity = h->spread_parity;
  const hipError_t err = wd::launch_env_kernel(q, wd::kModeIterate, probs, h->g, h->stream);
  if (err != hipSuccess) return hip_failed(h, err, "iterate kernel");
  h->spread_parity ^= 1;
  h->rows_valid = true;
  h->g += 1;
  return WD_OK;
}

int wd_iterate_static(const wd_config* cfg, const wd_buffers* bufs, const float* probs, uint64_t g) {
  if (!cfg || !bufs || !probs) return WD_E_NULL;
  int rc = check_config(cfg);
  if (rc != WD_OK) return rc;
  const void* ptrs[] = {bufs->pos_x, bufs->pos_y, bufs->pos_x0, bufs->pos_y0, bufs->live, bufs->action,
                        bufs->reward, bufs->obs, bufs->t, bufs->done, bufs->n_live_runners, bufs->tags_step};
  for (const void* ptr : ptrs)
    if (!ptr) return WD_E_NULL;
  for (const void* ptr : ptrs)
    if (!aligned256(ptr)) return WD_E_ALIGN;
  wd::Params params;
  rc = fill_params(*cfg, *bufs, &params);
  if (rc != WD_OK) return rc;
  if (!probs_aligned(params, probs)) return WD_E_ALIGN;
  params.big_spread = 0;  // (its accumulators have to start clear; the pair with one workgroup per env needs nothing of the kind)
  if (params.big) {
    if (size_t(place_big_tables(&params, cfg->num_envs, nullptr)) > kStaticScratchBytes) return WD_E_SCRATCH;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
      (void)hipGetLastError();
      return WD_E_HIP;
    }
    if (!g_scratch_ptr[dev]) {  // this device's copy of the array, at its own address
      void* ptr = nullptr;
      if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
        (void)hipGetLastError();
        return WD_E_HIP;
      }
      g_scratch_ptr[dev] = ptr;
    }
    // (nothing in the tables has to start at zero: the kernels write every entry before they read it)
    place_big_tables(&params, cfg->num_envs, static_cast<unsigned char*>(g_scratch_ptr[dev]));
  }
  params.rows_kept = 0;  // no handle, so nothing is known about what `obs` holds: every row is written whole
  if (wd::launch_env_kernel(params, wd::kModeIterate, probs, g, static_cast<hipStream_t>(cfg->stream)) != hipSuccess) {
    (void)hipGetLastError();
    return WD_E_HIP;
  }
  return WD_OK;
}

int wd_rollout(wd_handle* h, const float* probs_ring, int ring_len, int k, const wd_rollout_buffers* out) {
  if (!h || !probs_ring) return WD_E_NULL;
  if (ring_len < 1 || k < 1) return WD_E_CONFIG;
  if (!probs_aligned(h->params, probs_ring)) return WD_E_ALIGN;
  if (out) {
    const void* ptrs[] = {out->action, out->reward, out->done, out->obs};
    for (const void* ptr : ptrs)
      if (reinterpret_cast<uintptr_t>(ptr) & 15u) return WD_E_ALIGN;
  }
  if (!h->started) return WD_E_STATE;
  // recorded observations go to slices that hold nothing yet, and the in-place rows that the last
  // iteration then meets date from before the call: every row is written whole
  const int rows_kept = (h->rows_valid && !(out && out->obs)) ? 1 : 0;
  if (!wd::rollout_available(h->params)) {
    // Configurations without a multi-step kernel (large-env layout, full observations,
    // K > 8): the same results from one launch of the iteration kernels per iteration,
    // outputs redirected to the slices, the last slice copied from the in-place buffers.
    // In the large-env layout the observation kernel of iteration s runs on a second stream beside
    // the step kernel of iteration s + 1 (which needs the state, not the rows): two table images
    // in turn, an image rewritten only once the observation kernel that read it has finished.
    const bool piped = h->params.big && !h->params.big_spread && k > 1;
    if (piped) {
      const int rc = ensure_pipe(h);
      if (rc != WD_OK) return rc;
    }
    const int64_t EN = int64_t(h->cfg.num_envs) * h->cfg.num_agents, D = h->params.D;
    for (int s = 0; s < k; ++s) {
      wd::Params q = h->params;
      q.rows_kept = rows_kept;
      q.spread_parity = h->spread_parity;
      wd::ObsPipe pipe = {};
      if (piped) {
        const int b = s & 1;
        if (b) q.g_image = static_cast<unsigned char*>(h->second_image);
        if (s >= 2) {
          const hipError_t werr = hipStreamWaitEvent(h->stream, h->rows_done[b], 0);
          if (werr != hipSuccess) return hip_failed(h, werr, "wait for a table image");
        }
        pipe.stream = h->obs_stream;
        pipe.tables_ready = h->tables_ready[b];
        pipe.rows_done = h->rows_done[b];
      }
      if (out && s + 1 < k) {
        if (out->action) q.action = out->action + int64_t(s) * EN;
        if (out->reward) q.reward = out->reward + int64_t(s) * EN;
        if (out->obs) q.obs = out->obs + int64_t(s) * EN * D;
      }
      q.done_log = (out && out->done) ? out->done + int64_t(s) * h->cfg.num_envs : nullptr;
      const float* probs = probs_ring + int64_t((h->g + uint64_t(s)) % uint64_t(ring_len)) * EN * wd::kNumActions;
      const hipError_t err = wd::launch_env_kernel(q, wd::kModeIterate, probs, h->g + uint64_t(s), h->stream,
                                                   piped ? &pipe : nullptr);
      if (err != hipSuccess) return hip_failed(h, err, "iteration kernel of a roll-out");
      h->spread_parity ^= 1;
    }
    if (piped) {  // what follows on the caller's stream sees every row
      const hipError_t werr = hipStreamWaitEvent(h->stream, h->rows_done[(k - 1) & 1], 0);
      if (werr != hipSuccess) return hip_failed(h, werr, "wait for the last observation kernel");
    }
    if (out) {
      const int64_t last = int64_t(k - 1) * EN;
      hipError_t err = hipSuccess;
      if (out->action && err == hipSuccess)
        err = hipMemcpyAsync(out->action + last, h->bufs.action, size_t(EN) * 4, hipMemcpyDeviceToDevice, h->stream);
      if (out->reward && err == hipSuccess)
        err = hipMemcpyAsync(out->reward + last, h->bufs.reward, size_t(EN) * 4, hipMemcpyDeviceToDevice, h->stream);
      if (out->obs && err == hipSuccess)
        err = hipMemcpyAsync(out->obs + last * D, h->bufs.obs, size_t(EN * D) * 4, hipMemcpyDeviceToDevice, h->stream);
      if (err != hipSuccess) return hip_failed(h, err, "copy of the last roll-out slice");
    }
    h->rows_valid = true;
    h->g += uint64_t(k);
    return WD_OK;
  }
  wd::Roll roll;
  std::memset(&roll, 0, sizeof(roll));
  roll.steps = k;
  roll.ring_len = ring_len;
  roll.ring_pos = int32_t(h->g % uint64_t(ring_len));
  if (out) {
    roll.action = out->action;
    roll.reward = out->reward;
    roll.done = out->done;
    roll.obs = out->obs;
  }
  wd::Params q = h->params;
  q.rows_kept = rows_kept;
  const hipError_t err = wd::launch_rollout(q, roll, probs_ring, h->g, h->stream);
  if (err != hipSuccess) return hip_failed(h, err, "rollout kernel");
  h->rows_valid = true;
  h->g += uint64_t(k);
  return WD_OK;
}

int wd_get_step(wd_handle* h, uint64_t* g) {
  if (!h || !g) return WD_E_NULL;
  *g = h->g;
  return WD_OK;
}

int wd_set_step(wd_handle* h, uint64_t g) {
  if (!h) return WD_E_NULL;
  h->g = g;
  h->rows_valid = false;  // a resumed run: the caller may have restored the state arrays without the observations
  return WD_OK;
}

int wd_invalidate_obs(wd_handle* h) {
  if (!h) return WD_E_NULL;
  h->rows_valid = false;
  return WD_OK;
}

int wd_destroy(wd_handle* h) {
  if (!h) return WD_E_NULL;
  if (h->scratch) (void)hipFree(h->scratch);
  if (h->pipe_ready) {
    (void)hipStreamSynchronize(h->obs_stream);
    (void)hipFree(h->second_image);
    for (int b = 0; b < 2; ++b) {
      (void)hipEventDestroy(h->tables_ready[b]);
      (void)hipEventDestroy(h->rows_done[b]);
    }
    (void)hipStreamDestroy(h->obs_stream);
  }
  delete h;
  return WD_OK;
}

const char* wd_strerror(int status) {
  switch (status) {
    case WD_OK: return "ok";
    case WD_E_NULL: return "a required pointer is NULL";
    case WD_E_CONFIG: return "configuration field out of range";
    case WD_E_ALIGN: return "device buffer not aligned as required";
    case WD_E_STATE: return "call before the first wd_reset(WD_RESET_ALL)";
    case WD_E_HIP: return "HIP call failed";
    case WD_E_UNSUPPORTED: return "configuration not covered by this build's kernels";
    case WD_E_SCRATCH: return "work tables of this configuration exceed the static scratch array of wd_iterate_static";
    default: return "unknown status";
  }
}

const char* wd_last_error(wd_handle* h) { return h ? h->last_error.c_str() : ""; }

}  // extern "C"
