// wd_kernels.hip — device code of libwd for gfx950 (wave64, 160 KB LDS per CU).
//
// Three services of the roll-out loop (arXiv 2108.13976, Sec. 4.4: sampler and reset
// kernels of the service layer, step kernel of the environment; Sec. 4.5 items 3-6),
// for the discrete Tag rules of Sec. 5.1.  The paper maps one thread block to an env
// and one thread to an agent; here a TEAM of 8..256 threads owns an env (several small
// envs share a 256-thread workgroup, a thread owns several agents of a large env), the
// env's positions are staged in LDS, the pairwise passes (tag check, K-nearest search)
// run over a bucket-sorted copy of the live agents instead of over all pairs, and
// observation rows leave through an LDS transpose so that HBM sees whole lines.
#include "wd_internal.h"

namespace wd {
namespace {

constexpr uint32_t kDeadBit = 0x80000000u;  // in a packed position: agent is out of play
constexpr uint32_t kNoNeighbour = 0xFFFFu;

// ----------------------------------------------------------------------------------
// Random numbers: Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11).  Ten rounds of
// two 32x32->64 multiplies and a word permutation, the key bumped by Weyl constants.
// ----------------------------------------------------------------------------------
struct Block4 {
  uint32_t w0, w1, w2, w3;
};

__device__ __forceinline__ Block4 philox_block(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                               uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int round = 0; round < 10; ++round) {
    const uint32_t hi_a = __umulhi(0xD2511F53u, c0), lo_a = 0xD2511F53u * c0;
    const uint32_t hi_b = __umulhi(0xCD9E8D57u, c2), lo_b = 0xCD9E8D57u * c2;
    c0 = hi_b ^ c1 ^ k0;
    c1 = lo_b;
    c2 = hi_a ^ c3 ^ k1;
    c3 = lo_a;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return Block4{c0, c1, c2, c3};
}

// Counter layout: (global env id, agent, g low word, stream | g high word << 8).
__device__ __forceinline__ Block4 random_block(const Params& p, uint32_t env_local, uint32_t agent,
                                               uint32_t g_lo, uint32_t g_hi, uint32_t stream) {
  return philox_block(p.env_offset + env_local, agent, g_lo, stream | (g_hi << 8), p.seed_lo, p.seed_hi);
}

__device__ __forceinline__ uint32_t fastdiv(uint32_t a, const FastDiv& f) {
  const uint32_t t = __umulhi(a, f.mul);
  return (t + ((a - t) >> f.sh1)) >> f.sh2;
}

// Inverse-CDF draw: float32 running sum left to right, strict "<", last action as fall-through.
__device__ __forceinline__ int32_t sample_action(const float* __restrict__ pr, uint32_t word) {
  const float u = static_cast<float>(word >> 8) * (1.0f / 16777216.0f);
  const float c0 = 0.0f + pr[0];
  const float c1 = c0 + pr[1];
  const float c2 = c1 + pr[2];
  const float c3 = c2 + pr[3];
  return (u < c0) ? 0 : (u < c1) ? 1 : (u < c2) ? 2 : (u < c3) ? 3 : 4;
}

// ----------------------------------------------------------------------------------
// Flat per-agent kernels
// ----------------------------------------------------------------------------------
__global__ __launch_bounds__(kWorkgroupSize) void sample_kernel(const Params p, const float* __restrict__ probs,
                                                                uint32_t g_lo, uint32_t g_hi) {
  const int64_t total = int64_t(p.E) * p.N;
  const int64_t a = int64_t(blockIdx.x) * kWorkgroupSize + threadIdx.x;
  if (a >= total) return;
  const uint32_t e = fastdiv(uint32_t(a), p.div_N);
  const uint32_t i = uint32_t(a) - e * uint32_t(p.N);
  const Block4 r = random_block(p, e, i, g_lo, g_hi, kStreamAction);
  p.action[a] = sample_action(probs + a * kNumActions, r.w0);
}

__global__ __launch_bounds__(kWorkgroupSize) void init_start_positions_kernel(const Params p) {
  const int64_t total = int64_t(p.E) * p.N;
  const int64_t a = int64_t(blockIdx.x) * kWorkgroupSize + threadIdx.x;
  if (a >= total) return;
  const uint32_t e = fastdiv(uint32_t(a), p.div_N);
  const uint32_t i = uint32_t(a) - e * uint32_t(p.N);
  const Block4 r = random_block(p, e, i, 0u, 0u, kStreamInit);
  p.pos_x0[a] = int32_t(__umulhi(r.w0, uint32_t(p.G)));
  p.pos_y0[a] = int32_t(__umulhi(r.w1, uint32_t(p.G)));
}

// ----------------------------------------------------------------------------------
// Team helpers
// ----------------------------------------------------------------------------------
template <typename KeyT>
struct KeyLimits {
  static constexpr KeyT kNone = ~KeyT(0);
};

// Exclusive prefix sum of one value per thread across a team of (1 << ts_log2) threads.
// Teams of up to one wave use lane shuffles; larger teams add per-wave totals through LDS
// (wave_totals: one int per wave of the team).  Contains a workgroup barrier when the team
// spans several waves, so every thread of the workgroup must call it.
__device__ __forceinline__ int team_exclusive_scan(int v, int lt, int ts_log2, int* wave_totals, int* total) {
  const int lane = threadIdx.x & (kWaveSize - 1);
  const int width = ts_log2 >= 6 ? kWaveSize : (1 << ts_log2);
  const int sub = lane & (width - 1);
  int incl = v;
  for (int d = 1; d < width; d <<= 1) {
    const int up = __shfl_up(incl, d, width);
    if (sub >= d) incl += up;
  }
  if (ts_log2 <= 6) {
    *total = __shfl(incl, width - 1, width);
    return incl - v;
  }
  const int waves = 1 << (ts_log2 - 6);
  const int my_wave = lt >> 6;
  if (lane == kWaveSize - 1) wave_totals[my_wave] = incl;
  __syncthreads();
  int before = 0, all = 0;
  for (int w = 0; w < waves; ++w) {
    const int wt = wave_totals[w];
    all += wt;
    if (w < my_wave) before += wt;
  }
  *total = all;
  return before + incl - v;
}

struct Buckets {
  int shift;  // a bucket is (1 << shift) cells wide
  int nbx;    // buckets per grid side
};

// Bucket width for `n_live` agents on a G x G grid: the smallest power of two that keeps
// the bucket count within nb_cap and the mean occupancy at or above lambda.  Any choice
// gives the same results; this one only trades search rings against candidates per ring.
__device__ __forceinline__ Buckets choose_buckets(const Params& p, int n_live) {
  int s = 0;
  for (; s < 15; ++s) {
    const int64_t nbx = (p.G + (1 << s) - 1) >> s;
    if (nbx * nbx <= p.nb_cap &&
        (int64_t(n_live) << (2 * s)) * p.lambda_den >= int64_t(p.lambda_num) * p.G * p.G)
      break;
  }
  Buckets b;
  b.shift = s;
  b.nbx = (p.G + (1 << s) - 1) >> s;
  return b;
}

__device__ __forceinline__ uint32_t pack_pos(int x, int y, bool is_live) {
  return uint32_t(x) | (uint32_t(y) << 16) | (is_live ? 0u : kDeadBit);
}
__device__ __forceinline__ int pos_x_of(uint32_t pl) { return int(pl & 0x7FFFu); }
__device__ __forceinline__ int pos_y_of(uint32_t pl) { return int((pl >> 16) & 0x7FFFu); }

// LDS views of one team's region.
template <typename KeyT>
struct TeamLds {
  uint32_t* pl;       // [N] packed position + dead bit, by agent index
  uint2* sorted;      // [N] (packed position, agent index) of live agents, grouped by bucket
  uint16_t* slot;     // [N] where agent i sits in `sorted`
  KeyT* best;         // [N] per runner: smallest (distance, tagger) key in range
  int32_t* credits;   // [N_tag]
  uint16_t* nbr;      // [N][K] neighbour indices
  uint32_t* counts;   // [nb_cap] bucket counts, then scatter cursors
  uint32_t* starts;   // [nb_cap + 1] bucket start offsets in `sorted`
  int32_t* misc;      // [0] tags this step, [1] t after the call, [2] rows to be written, [4..7] scan scratch
  __device__ __forceinline__ TeamLds(unsigned char* base, const Params& p)
      : pl(reinterpret_cast<uint32_t*>(base + p.off_pl)),
        sorted(reinterpret_cast<uint2*>(base + p.off_sorted)),
        slot(reinterpret_cast<uint16_t*>(base + p.off_slot)),
        best(reinterpret_cast<KeyT*>(base + p.off_best)),
        credits(reinterpret_cast<int32_t*>(base + p.off_credits)),
        nbr(reinterpret_cast<uint16_t*>(base + p.off_nbr)),
        counts(reinterpret_cast<uint32_t*>(base + p.off_counts)),
        starts(reinterpret_cast<uint32_t*>(base + p.off_starts)),
        misc(reinterpret_cast<int32_t*>(base + p.off_misc)) {}
};

// Counting sort of the team's live agents by bucket: counts -> starts -> sorted/slot.
// `act` marks teams that take part; every thread of the workgroup must call (barriers inside).
// Requires pl[] written and counts[] zeroed before the call (and a barrier after that).
template <typename KeyT>
__device__ __forceinline__ void build_buckets(const Params& p, const TeamLds<KeyT>& L, bool act, int lt, int ts,
                                              const Buckets bk) {
  if (act) {
    for (int k = 0; k < p.apt; ++k) {
      const int i = lt + k * ts;
      if (i < p.N) {
        const uint32_t v = L.pl[i];
        if (!(v & kDeadBit))
          atomicAdd(&L.counts[(pos_y_of(v) >> bk.shift) * bk.nbx + (pos_x_of(v) >> bk.shift)], 1u);
      }
    }
  }
  __syncthreads();
  int part = 0;
  const int j0 = lt * p.scan_chunk;
  if (act)
    for (int c = 0; c < p.scan_chunk; ++c) part += int(L.counts[j0 + c]);
  int total = 0;
  int run = team_exclusive_scan(part, lt, p.ts_log2, L.misc + 4, &total);
  if (act) {
    for (int c = 0; c < p.scan_chunk; ++c) {
      const int v = int(L.counts[j0 + c]);
      L.starts[j0 + c] = uint32_t(run);
      L.counts[j0 + c] = uint32_t(run);
      run += v;
    }
    if (lt == ts - 1) L.starts[p.nb_cap] = uint32_t(total);
  }
  __syncthreads();
  if (act) {
    for (int k = 0; k < p.apt; ++k) {
      const int i = lt + k * ts;
      if (i < p.N) {
        const uint32_t v = L.pl[i];
        if (!(v & kDeadBit)) {
          const uint32_t at =
              atomicAdd(&L.counts[(pos_y_of(v) >> bk.shift) * bk.nbx + (pos_x_of(v) >> bk.shift)], 1u);
          L.sorted[at] = make_uint2(v, uint32_t(i));
          L.slot[i] = uint16_t(at);
        }
      }
    }
  }
  __syncthreads();
}

// Sorted insertion of `key` into an ascending list of KT keys (the largest falls off).
template <typename KeyT, int KT>
__device__ __forceinline__ void insert_key(KeyT (&keys)[KT], KeyT key) {
#pragma unroll
  for (int k = KT - 1; k >= 1; --k) {
    const KeyT hi = keys[k - 1] > key ? keys[k - 1] : key;
    keys[k] = keys[k] < hi ? keys[k] : hi;
  }
  keys[0] = keys[0] < key ? keys[0] : key;
}

// The K smallest (squared distance, index) keys among the other live agents, exactly.
// Scans the (2r+1)^2 buckets around the agent's own; every agent outside that block is
// farther than r bucket widths in x or in y, so once the K-th key is below (r*B+1)^2 (or
// the block covers the grid) no unseen agent can enter the list; otherwise r doubles and
// the scan restarts.
template <typename KeyT, int KT>
__device__ __forceinline__ void nearest_keys(KeyT (&keys)[KT], int K, int x, int y, uint32_t self_slot,
                                             const Buckets bk, int idx_bits, const uint2* sorted,
                                             const uint32_t* starts) {
  const int bx = x >> bk.shift, by = y >> bk.shift, last = bk.nbx - 1;
  for (int r = 1;; r *= 2) {
#pragma unroll
    for (int k = 0; k < KT; ++k) keys[k] = KeyLimits<KeyT>::kNone;
    const int x0 = max(bx - r, 0), x1 = min(bx + r, last);
    const int y0 = max(by - r, 0), y1 = min(by + r, last);
    for (int row = y0; row <= y1; ++row) {
      const uint32_t q_end = starts[row * bk.nbx + x1 + 1];
      for (uint32_t q = starts[row * bk.nbx + x0]; q < q_end; ++q) {
        const uint2 ent = sorted[q];
        const int dx = pos_x_of(ent.x) - x, dy = pos_y_of(ent.x) - y;
        const uint32_t d2 = uint32_t(__mul24(dx, dx)) + uint32_t(__mul24(dy, dy));
        KeyT key = (KeyT(d2) << idx_bits) | KeyT(ent.y);
        if (q == self_slot || (ent.x & kDeadBit)) key = KeyLimits<KeyT>::kNone;
        insert_key<KeyT, KT>(keys, key);
      }
    }
    if (bx - r <= 0 && bx + r >= last && by - r <= 0 && by + r >= last) break;
    const uint64_t reach = uint64_t(r) * (uint64_t(1) << bk.shift) + 1;
    if (uint64_t(keys[K - 1]) < ((reach * reach) << idx_bits)) break;
  }
}

// ----------------------------------------------------------------------------------
// The env-per-team kernel: step, reset, or a whole iteration (sample + step + reset).
// KT > 0: K <= KT nearest neighbours kept in registers, rows leave through the LDS
// transpose.  KT == 0: any K, by repeated selection, rows written directly (slow path).
// ----------------------------------------------------------------------------------
template <typename KeyT, int KT>
__global__ __launch_bounds__(kWorkgroupSize) void env_kernel(const Params p, const int mode,
                                                             const float* __restrict__ probs, uint32_t g_lo,
                                                             uint32_t g_hi) {
  extern __shared__ __align__(16) unsigned char smem[];
  const int tid = threadIdx.x;
  const int ts = 1 << p.ts_log2;
  const int team = tid >> p.ts_log2;
  const int lt = tid & (ts - 1);
  const int e0 = blockIdx.x * p.teams_per_wg;
  const int e = e0 + team;
  const int N = p.N, N_tag = p.N_tag, G = p.G, K = p.K;
  const bool valid = e < p.E;
  const int64_t abase = int64_t(valid ? e : 0) * N;
  const TeamLds<KeyT> L(smem + team * p.team_stride, p);
  const KeyT idx_mask = (KeyT(1) << p.idx_bits) - 1;

  int done_in = 0, t_in = 0, nlr_in = 0;
  if (valid) {
    done_in = p.done[e];
    t_in = p.t[e];
    nlr_in = p.n_live_runners[e];
  }
  const bool stepping = (mode == kModeStep || mode == kModeIterate);
  const bool step_act = stepping && valid && !done_in;
  bool out_act = false;   // this team's env gets new observation rows
  int t_out = t_in;
  bool done_now = done_in != 0;
  Buckets bk = choose_buckets(p, nlr_in + N_tag);

  if (stepping) {
    // ---- sample (iterate mode) and move; stage positions in LDS -------------------
    for (int k = 0; k < p.apt; ++k) {
      const int i = lt + k * ts;
      if (valid && i < N) {
        int act = 0;
        if (mode == kModeIterate) {
          const Block4 r = random_block(p, uint32_t(e), uint32_t(i), g_lo, g_hi, kStreamAction);
          act = sample_action(probs + (abase + i) * kNumActions, r.w0);
          p.action[abase + i] = act;
        } else if (step_act) {
          act = p.action[abase + i];
        }
        if (step_act) {
          // positions are kept on the grid by every writer; the clamp only keeps a caller's
          // stray value from indexing outside the bucket table
          int x = min(max(p.pos_x[abase + i], 0), G - 1), y = min(max(p.pos_y[abase + i], 0), G - 1);
          const bool lv = p.live[abase + i] != 0;
          if (lv) {
            const int nx = min(max(x + (act == 4) - (act == 3), 0), G - 1);
            const int ny = min(max(y + (act == 1) - (act == 2), 0), G - 1);
            if (nx != x) p.pos_x[abase + i] = nx;
            if (ny != y) p.pos_y[abase + i] = ny;
            x = nx;
            y = ny;
          }
          L.pl[i] = pack_pos(x, y, lv);
          L.best[i] = KeyLimits<KeyT>::kNone;
        }
      }
    }
    if (step_act) {
      for (int j = lt; j < p.nb_cap; j += ts) L.counts[j] = 0u;
      for (int j = lt; j < N_tag; j += ts) L.credits[j] = 0;
      if (lt == 0) L.misc[0] = 0;
    }
    __syncthreads();
    build_buckets<KeyT>(p, L, step_act, lt, ts, bk);

    // ---- tag check, from the tagger's side: runners in range get the smallest
    //      (distance, tagger) key; min is order-independent, so the result is unique ----
    if (step_act && p.tag_r2 >= 0) {
      for (int k = 0; k < p.apt; ++k) {
        const int i = lt + k * ts;
        if (i < N_tag) {
          const uint32_t me = L.pl[i];
          const int x = pos_x_of(me), y = pos_y_of(me);
          const int bx0 = max(x - p.tag_rad, 0) >> bk.shift, bx1 = min(x + p.tag_rad, G - 1) >> bk.shift;
          const int by0 = max(y - p.tag_rad, 0) >> bk.shift, by1 = min(y + p.tag_rad, G - 1) >> bk.shift;
          for (int row = by0; row <= by1; ++row) {
            const uint32_t q_end = L.starts[row * bk.nbx + bx1 + 1];
            for (uint32_t q = L.starts[row * bk.nbx + bx0]; q < q_end; ++q) {
              const uint2 ent = L.sorted[q];
              if (int(ent.y) < N_tag) continue;
              const int dx = pos_x_of(ent.x) - x, dy = pos_y_of(ent.x) - y;
              const uint32_t d2 = uint32_t(__mul24(dx, dx)) + uint32_t(__mul24(dy, dy));
              if (d2 <= uint32_t(p.tag_r2)) atomicMin(&L.best[ent.y], (KeyT(d2) << p.idx_bits) | KeyT(i));
            }
          }
        }
      }
    }
    __syncthreads();
    // ---- runners: leave the game if tagged, credit the tagger, take the penalty ------
    if (step_act) {
      for (int k = 0; k < p.apt; ++k) {
        const int i = lt + k * ts;
        if (i >= N_tag && i < N) {
          const uint32_t me = L.pl[i];
          float rew = 0.0f;
          if (!(me & kDeadBit)) {
            const KeyT b = L.best[i];
            if (b != KeyLimits<KeyT>::kNone) {
              p.live[abase + i] = 0;
              L.pl[i] = me | kDeadBit;
              L.sorted[L.slot[i]].x = me | kDeadBit;
              rew = p.tag_penalty;
              atomicAdd(&L.credits[int(b & idx_mask)], 1);
              atomicAdd(&L.misc[0], 1);
            }
          }
          p.reward[abase + i] = rew;
        }
      }
    }
    __syncthreads();
    // ---- tagger rewards, env clock and termination ------------------------------------
    if (step_act) {
      for (int k = 0; k < p.apt; ++k) {
        const int i = lt + k * ts;
        if (i < N_tag) p.reward[abase + i] = static_cast<float>(L.credits[i]) * p.tag_reward;
      }
      const int tags = L.misc[0];
      const int nlr = nlr_in - tags;
      t_out = t_in + 1;
      done_now = (nlr == 0) || (t_out >= p.T);
      if (lt == 0) {
        p.t[e] = t_out;
        p.n_live_runners[e] = nlr;
        p.tags_step[e] = tags;
        p.done[e] = done_now ? 1 : 0;
      }
      out_act = true;
    }
  }

  if (mode != kModeStep) {
    // ---- reset: restore the start state of envs that are done (or of all) -------------
    const bool reset_act = valid && (mode == kModeResetAll || done_now);
    const bool any_reset = (mode == kModeIterate) ? (__syncthreads_or(reset_act ? 1 : 0) != 0) : true;
    if (any_reset) {
      bk = reset_act ? choose_buckets(p, N) : bk;
      if (reset_act) {
        for (int k = 0; k < p.apt; ++k) {
          const int i = lt + k * ts;
          if (i < N) {
            const int x = min(max(p.pos_x0[abase + i], 0), G - 1), y = min(max(p.pos_y0[abase + i], 0), G - 1);
            p.pos_x[abase + i] = x;
            p.pos_y[abase + i] = y;
            p.live[abase + i] = 1;
            L.pl[i] = pack_pos(x, y, true);
          }
        }
        for (int j = lt; j < p.nb_cap; j += ts) L.counts[j] = 0u;
        t_out = 0;
        if (lt == 0) {
          p.t[e] = 0;
          p.n_live_runners[e] = N - N_tag;
          p.tags_step[e] = 0;
          p.done[e] = 0;
        }
        out_act = true;
      }
      __syncthreads();
      build_buckets<KeyT>(p, L, reset_act, lt, ts, bk);
    }
  }

  // ---- observations --------------------------------------------------------------------
  if (lt == 0) {
    L.misc[1] = t_out;
    L.misc[2] = out_act ? 1 : 0;
  }
  if constexpr (KT > 0) {
    // K nearest, in bucket order (neighbouring lanes search neighbouring cells)
    if (out_act && K > 0) {
      const int n_sorted = int(L.starts[p.nb_cap]);
      for (int k = 0; k < p.apt; ++k) {
        const int q = lt + k * ts;
        if (q < n_sorted) {
          const uint2 ent = L.sorted[q];
          if (!(ent.x & kDeadBit)) {
            KeyT keys[KT];
            nearest_keys<KeyT, KT>(keys, K, pos_x_of(ent.x), pos_y_of(ent.x), uint32_t(q), bk, p.idx_bits,
                                   L.sorted, L.starts);
#pragma unroll
            for (int kk = 0; kk < KT; ++kk)
              if (kk < K)
                L.nbr[ent.y * K + kk] =
                    keys[kk] == KeyLimits<KeyT>::kNone ? uint16_t(kNoNeighbour) : uint16_t(keys[kk] & idx_mask);
          }
        }
      }
    }
    const bool all_out = __syncthreads_and((out_act || !valid) ? 1 : 0) != 0;  // also the barrier before the rows

    // rows, in index order; a wave builds 64 rows, transposes them through LDS and
    // writes them as one contiguous run
    const int wave = tid >> 6, lane = tid & (kWaveSize - 1);
    const int D = p.D;
    float* stage = reinterpret_cast<float*>(smem + p.off_stage) + wave * kWaveSize * D;
    const int rows_total = min(p.teams_per_wg, p.E - e0) * N;
    const int64_t obs_base = int64_t(e0) * N * D;
    const bool vec_ok = (obs_base & 3) == 0;
    for (int c = wave; c * kWaveSize < rows_total; c += kWavesPerWorkgroup) {
      const int R = c * kWaveSize + lane;
      if (R < rows_total) {
        const int tm = int(fastdiv(uint32_t(R), p.div_N));
        const int i = R - tm * N;
        const TeamLds<KeyT> Lr(smem + tm * p.team_stride, p);
        if (all_out || Lr.misc[2]) {
          float* row = all_out ? stage + lane * D : p.obs + obs_base + int64_t(R) * D;
          const uint32_t me = Lr.pl[i];
          const int x = pos_x_of(me), y = pos_y_of(me);
          const bool lv = !(me & kDeadBit);
          row[0] = static_cast<float>(x) * p.inv_G;
          row[1] = static_cast<float>(y) * p.inv_G;
          row[2] = i < N_tag ? 1.0f : 0.0f;
          row[3] = lv ? 1.0f : 0.0f;
          row[4] = static_cast<float>(Lr.misc[1]) * p.inv_T;
          for (int kk = 0; kk < K; ++kk) {
            const uint32_t j = lv ? uint32_t(Lr.nbr[i * K + kk]) : kNoNeighbour;
            float f0 = 0.0f, f1 = 0.0f, f2 = 0.0f, f3 = 0.0f;
            if (j != kNoNeighbour) {
              const uint32_t other = Lr.pl[j];
              f0 = static_cast<float>(pos_x_of(other) - x) * p.inv_G;
              f1 = static_cast<float>(pos_y_of(other) - y) * p.inv_G;
              f2 = int(j) < N_tag ? 1.0f : 0.0f;
              f3 = 1.0f;
            }
            row[5 + 4 * kk + 0] = f0;
            row[5 + 4 * kk + 1] = f1;
            row[5 + 4 * kk + 2] = f2;
            row[5 + 4 * kk + 3] = f3;
          }
        }
      }
      if (all_out) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const int nfl = min(kWaveSize, rows_total - c * kWaveSize) * D;
        float* dst = p.obs + obs_base + int64_t(c) * kWaveSize * D;
        if (vec_ok) {
          const int nvec = nfl >> 2;
          for (int v = lane; v < nvec; v += kWaveSize)
            reinterpret_cast<float4*>(dst)[v] = reinterpret_cast<const float4*>(stage)[v];
          for (int f = (nvec << 2) + lane; f < nfl; f += kWaveSize) dst[f] = stage[f];
        } else {
          for (int f = lane; f < nfl; f += kWaveSize) dst[f] = stage[f];
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      }
    }
  } else {
    // any K: the k-th neighbour is the smallest key above the (k-1)-th; rows written in place
    __syncthreads();
    if (out_act) {
      const int D = p.D;
      const int n_sorted = int(L.starts[p.nb_cap]);
      const float tf = static_cast<float>(t_out) * p.inv_T;
      for (int k = 0; k < p.apt; ++k) {
        const int i = lt + k * ts;
        if (i >= N) continue;
        float* row = p.obs + (abase + i) * D;
        const uint32_t me = L.pl[i];
        const int x = pos_x_of(me), y = pos_y_of(me);
        const bool lv = !(me & kDeadBit);
        row[0] = static_cast<float>(x) * p.inv_G;
        row[1] = static_cast<float>(y) * p.inv_G;
        row[2] = i < N_tag ? 1.0f : 0.0f;
        row[3] = lv ? 1.0f : 0.0f;
        row[4] = tf;
        bool have_prev = false, exhausted = !lv;
        KeyT prev = 0;
        for (int kk = 0; kk < K; ++kk) {
          KeyT bestk = KeyLimits<KeyT>::kNone;
          if (!exhausted) {
            for (int q = 0; q < n_sorted; ++q) {
              const uint2 ent = L.sorted[q];
              if (int(ent.y) == i || (ent.x & kDeadBit)) continue;
              const int dx = pos_x_of(ent.x) - x, dy = pos_y_of(ent.x) - y;
              const uint32_t d2 = uint32_t(__mul24(dx, dx)) + uint32_t(__mul24(dy, dy));
              const KeyT key = (KeyT(d2) << p.idx_bits) | KeyT(ent.y);
              if ((!have_prev || key > prev) && key < bestk) bestk = key;
            }
          }
          float f0 = 0.0f, f1 = 0.0f, f2 = 0.0f, f3 = 0.0f;
          if (bestk != KeyLimits<KeyT>::kNone) {
            const int j = int(bestk & idx_mask);
            const uint32_t other = L.pl[j];
            f0 = static_cast<float>(pos_x_of(other) - x) * p.inv_G;
            f1 = static_cast<float>(pos_y_of(other) - y) * p.inv_G;
            f2 = j < N_tag ? 1.0f : 0.0f;
            f3 = 1.0f;
            prev = bestk;
            have_prev = true;
          } else {
            exhausted = true;
          }
          row[5 + 4 * kk + 0] = f0;
          row[5 + 4 * kk + 1] = f1;
          row[5 + 4 * kk + 2] = f2;
          row[5 + 4 * kk + 3] = f3;
        }
      }
    }
  }
}

template <typename KeyT, int KT>
hipError_t launch_env_variant(const Params& p, int mode, const float* probs, uint64_t g, hipStream_t stream) {
  const int groups = (p.E + p.teams_per_wg - 1) / p.teams_per_wg;
  hipLaunchKernelGGL((env_kernel<KeyT, KT>), dim3(groups), dim3(kWorkgroupSize), size_t(p.lds_bytes), stream, p,
                     mode, probs, uint32_t(g), uint32_t(g >> 32));
  return hipGetLastError();
}

template <typename KeyT, int KT>
hipError_t prepare_env_variant(const Params& p) {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&env_kernel<KeyT, KT>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, p.lds_bytes);
}

// Register list length for K: the smallest compiled size that holds it; 0 = any-K path.
int register_k(const Params& p) {
  if (p.K > kMaxRegisterK) return 0;
  if (p.K <= 1) return 1;
  if (p.K <= 2) return 2;
  if (p.K <= 4) return 4;
  return 8;
}

bool wide_keys(const Params& p) { return p.idx_bits < 0; }

}  // namespace

// The key width is chosen by the host: idx_bits >= 0 with a 32-bit key when
// (max squared distance + 1) << idx_bits fits below 2^32, else 64-bit keys and ~idx_bits.
#define WD_DISPATCH(fn, ...)                                                   \
  do {                                                                         \
    const int kt = register_k(p);                                              \
    Params q = p;                                                              \
    const bool wide = wide_keys(p);                                            \
    if (wide) q.idx_bits = ~p.idx_bits;                                        \
    if (!wide) {                                                               \
      switch (kt) {                                                            \
        case 0: return fn<uint32_t, 0>(q, ##__VA_ARGS__);                      \
        case 1: return fn<uint32_t, 1>(q, ##__VA_ARGS__);                      \
        case 2: return fn<uint32_t, 2>(q, ##__VA_ARGS__);                      \
        case 4: return fn<uint32_t, 4>(q, ##__VA_ARGS__);                      \
        default: return fn<uint32_t, 8>(q, ##__VA_ARGS__);                     \
      }                                                                        \
    } else {                                                                   \
      switch (kt) {                                                            \
        case 0: return fn<unsigned long long, 0>(q, ##__VA_ARGS__);            \
        case 1: return fn<unsigned long long, 1>(q, ##__VA_ARGS__);            \
        case 2: return fn<unsigned long long, 2>(q, ##__VA_ARGS__);            \
        case 4: return fn<unsigned long long, 4>(q, ##__VA_ARGS__);            \
        default: return fn<unsigned long long, 8>(q, ##__VA_ARGS__);           \
      }                                                                        \
    }                                                                          \
  } while (0)

hipError_t launch_env_kernel(const Params& p, int mode, const float* probs, uint64_t g, hipStream_t stream) {
  WD_DISPATCH(launch_env_variant, mode, probs, g, stream);
}

hipError_t prepare_env_kernels(const Params& p) { WD_DISPATCH(prepare_env_variant); }

bool env_kernel_available(const Params& p) { return p.obs_mode == 0; }

hipError_t launch_sample(const Params& p, const float* probs, uint64_t g, hipStream_t stream) {
  const int64_t total = int64_t(p.E) * p.N;
  const int groups = int((total + kWorkgroupSize - 1) / kWorkgroupSize);
  hipLaunchKernelGGL(sample_kernel, dim3(groups), dim3(kWorkgroupSize), 0, stream, p, probs, uint32_t(g),
                     uint32_t(g >> 32));
  return hipGetLastError();
}

hipError_t launch_init_start_positions(const Params& p, hipStream_t stream) {
  const int64_t total = int64_t(p.E) * p.N;
  const int groups = int((total + kWorkgroupSize - 1) / kWorkgroupSize);
  hipLaunchKernelGGL(init_start_positions_kernel, dim3(groups), dim3(kWorkgroupSize), 0, stream, p);
  return hipGetLastError();
}

}  // namespace wd
