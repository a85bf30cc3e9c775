// wd_kernels.hip — device code of libwd for gfx950 (wave64, 160 KB LDS per CU).
//
// Three services of the roll-out loop (arXiv 2108.13976, Sec. 4.4: sampler and reset
// kernels of the service layer, step kernel of the environment; Sec. 4.5 items 3-6),
// for the discrete Tag rules of Sec. 5.1.  The paper maps one thread block to an env
// and one thread to an agent; here a TEAM of 8..1024 threads owns an env (several small
// envs share a 256-thread workgroup), a thread owns groups of four consecutive agents
// (16-byte loads and stores, one random block per group), the env's positions are staged
// in LDS, the pairwise passes (tag check, K-nearest search) run over a bucket-sorted copy
// of the live agents instead of over all pairs, and observation rows leave through an LDS
// transpose so that HBM sees whole lines.
#include <cstring>
#include <type_traits>

#include "wd_dev_common.h"
#include "wd_dev_rows.h"
#include "wd_dev_strips.h"
#include "wd_dev_tables.h"
#include "wd_internal.h"

namespace wd {
namespace {

using namespace dev;

// ----------------------------------------------------------------------------------
// Flat kernels: the separately callable sampler (one thread per group of four agents)
// and the start positions (one thread per agent)
// ----------------------------------------------------------------------------------
__global__ __launch_bounds__(kWorkgroupSize) void sample_kernel(const Params p, const float* __restrict__ probs,
                                                                uint32_t g_lo, uint32_t g_hi) {
  const int64_t total = int64_t(p.E) * p.NG;
  const int64_t gid = int64_t(blockIdx.x) * kWorkgroupSize + threadIdx.x;
  if (gid >= total) return;
  const uint32_t e = fastdiv(uint32_t(gid), p.div_NG);
  const uint32_t grp = uint32_t(gid) - e * uint32_t(p.NG);
  const int i0 = int(grp) * 4;
  const int64_t a0 = int64_t(e) * p.N + i0;
  const Block4 r = random_block(p, e, grp, g_lo, g_hi, kStreamAction);
  int act[4];
  sample_group(probs, a0, min(4, p.N - i0), p.vec4 != 0, r, act);
  store4(p.action, a0, min(4, p.N - i0), p.vec4 != 0, act);
}

__global__ __launch_bounds__(kWorkgroupSize) void init_start_positions_kernel(const Params p) {
  const int64_t total = int64_t(p.E) * p.N;
  const int64_t a = int64_t(blockIdx.x) * kWorkgroupSize + threadIdx.x;
  if (a >= total) return;
  const uint32_t e = fastdiv(uint32_t(a), p.div_N);
  const uint32_t i = uint32_t(a) - e * uint32_t(p.N);
  const Block4 r = random_block(p, e, i, 0u, 0u, kStreamInit);
  p.pos_x0[a] = int32_t(__umulhi(r.w[0], uint32_t(p.G)));
  p.pos_y0[a] = int32_t(__umulhi(r.w[1], uint32_t(p.G)));
}

// ----------------------------------------------------------------------------------
// The env-per-team kernel: step, reset, or a whole iteration (sample + step + reset).
// KX > 0: K == KX known at compile time (1..8): the neighbour list and the row live in registers
// and rows leave through the LDS transpose.  KX == 0: K <= 8 at run time, KX == -2: K <= 16 (the
// list in registers, rows built in LDS).  KX == -1: any K, sixteen neighbours at a time, rows
// written directly (slow path).
// ----------------------------------------------------------------------------------
// Where one iteration's outputs go: the in-place buffers, or a slice of a roll-out's arrays.
struct StepOut {
  int32_t* action;   // written by the sampler of an iterate-mode call (the step reads p.action otherwise)
  float* reward;
  float* obs;
  int32_t* done_log; // optional: done flags before the reset clears them
};

// The parameters are read through a pointer into the kernel-argument segment that is made
// opaque to the optimiser at every phase boundary (WD_NEW_PHASE): a phase then loads the
// fields it uses with scalar loads of its own, instead of holding the ~100 fields of all
// phases in scalar registers and spilling them into vector-register lanes.  The roll-out loop
// does this once per iteration (measured: per phase is no gain there).
typedef const __attribute__((address_space(4))) Params* KernargParams;
#define WD_NEW_PHASE()                                   \
  do {                                                   \
    if constexpr (!LOOPED) asm volatile("" : "+s"(pk)); \
  } while (0)
#define p (*(const Params*)pk)

// What the roll-out loop keeps on chip between the iterations of one launch: the env clock and
// the live-runner count in registers, positions and live flags in the LDS position table.
// Only the last iteration of a launch writes the in-place state arrays (all of them); nobody
// can read the others' state before the launch ends.
struct LoopState {
  int t, nlr;
  bool resident;  // false in the first iteration of a launch: state comes from device memory
  bool last;      // the in-place state arrays are written in this iteration
};

template <int WIDE, int KX, bool CN, bool BIG, bool LOOPED, bool ONE>
__device__ __forceinline__ void env_body(KernargParams pk, const StepOut out, const int mode,
                                         const float* __restrict__ probs, uint32_t g_lo, uint32_t g_hi,
                                         unsigned char* smem, const int tid, LoopState& ls) {
  using SL = SortedList<WIDE>;
  using Key = typename SL::Key;
  // 32-bit keys with K compiled in, small layout: the live agents are sorted by strip and column
  // and the neighbour search reads fixed windows of that list; the other variants sort by
  // square buckets and search bucket rings
  constexpr bool STRIP = WIDE == kKeys31 && !BIG && KX > 0;
  // ONE: the launch has one team per workgroup, so everything that depends on the team (table
  // addresses, the env's scalars, the strip geometry) is uniform and lives in scalar registers
  const int ts = 1 << p.ts_log2;
  const int team = ONE ? 0 : tid >> p.ts_log2;
  const int lt = ONE ? tid : tid & (ts - 1);
  const int e0 = ONE ? int(blockIdx.x) : blockIdx.x * p.teams_per_wg;
  const int e = e0 + team;
  const int N = p.N, N_tag = p.N_tag, G = p.G, NG = p.NG;
  const int K = KX > 0 ? KX : p.K;
  const bool vec = p.vec4 != 0;
  const bool valid = e < p.E;
  const int64_t abase = int64_t(valid ? e : 0) * N;
  const TeamLds<WIDE, BIG> L(smem, team, p, e);
  const Key idx_mask = (Key(1) << p.idx_bits) - 1;

  const bool from_chip = LOOPED && ls.resident;
  const bool write_state = !LOOPED || ls.last;
  int done_in = 0, t_in = 0, nlr_in = 0;
  if (from_chip) {  // an env that was done has been reset by the iteration before
    t_in = ls.t;
    nlr_in = ls.nlr;
  } else if (valid) {
    done_in = p.done[e];
    t_in = p.t[e];
    nlr_in = p.n_live_runners[e];
  }
  int nlr_out = nlr_in;
  const bool stepping = (mode == kModeStep || mode == kModeIterate);
  const bool step_act = stepping && valid && !done_in;
  bool out_act = false;  // this team's env gets new observation rows
  int t_out = t_in;
  bool done_now = done_in != 0;
  Buckets bk = {};
  Strips sg = {};
  if constexpr (STRIP)
    sg = choose_strips(p, nlr_in + N_tag);
  else
    bk = choose_buckets(p, nlr_in + N_tag);
  if (lt == 0) {  // every mode passes a barrier before the neighbour search appends
    L.misc[2] = 0;  // set where the team's env is stepped or reset
    L.misc[3] = 0;
    L.misc[kMiscQueue2] = 0;
  }
  // Two workgroup-wide votes: some env of the workgroup is being reset; some env gets no new
  // rows.  Inside the roll-out loop (LOOPED) they are flags in the first team's scalars, cleared
  // here, set before a barrier that the code needs anyway and read after it; the one-step
  // kernel uses the voting barriers (each form measured faster where it is used).
  int32_t* const wg_flags = reinterpret_cast<int32_t*>(smem + p.off_misc) + 20;
  if (LOOPED && tid == 0) {
    wg_flags[0] = 0;
    wg_flags[1] = 0;
  }

  if (stepping) {
    if (step_act) {
      if constexpr (STRIP) {
        strip_prepare(p, L, sg, lt, ts);
      } else {
        for (int j = lt; j < p.nb_cap; j += ts) L.counts[j] = 0u;
        for (int j = lt; j <= bk.nbx; j += ts) L.edges[j] = uint16_t(min(bucket_first_cell(j, bk), G));
      }
      for (int j = lt; j < N_tag; j += ts) L.credits[j] = 0;
      if (lt == 0) L.misc[0] = 0;
    }
    __syncthreads();
    WD_NEW_PHASE();
    // ---- sample (iterate mode), move, stage positions in LDS, count buckets -------------
    for (int k = 0; k < p.gpt; ++k) {
      const int grp = lt + k * ts;
      if (valid && grp < NG) {
        const int i0 = 4 * grp, n = min(4, N - i0);
        const int64_t a0 = abase + i0;
        int act[4] = {0, 0, 0, 0};
        if (mode == kModeIterate) {
          const Block4 r = random_block(p, uint32_t(e), uint32_t(grp), g_lo, g_hi, kStreamAction);
          sample_group(probs, a0, n, vec, r, act);
          store4(out.action, a0, n, vec, act);
        } else if (step_act) {
          load4(p.action, a0, n, vec, act);
        }
        if (step_act) {
          int x[4], y[4], lv[4];
          if (from_chip) {
            const uint4 q4 = *reinterpret_cast<const uint4*>(L.pl + i0);
            const uint32_t q[4] = {q4.x, q4.y, q4.z, q4.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              x[j] = pos_x_of(q[j]);
              y[j] = pos_y_of(q[j]);
              lv[j] = (q[j] & kDeadBit) ? 0 : 1;
            }
          } else {
            load4(p.pos_x, a0, n, vec, x);
            load4(p.pos_y, a0, n, vec, y);
            load4(p.live, a0, n, vec, lv);
          }
          bool moved = LOOPED;  // the last iteration of a roll-out writes every group
          uint32_t packed[4];
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const bool is_live = j < n && lv[j] != 0;
            // positions are kept on the grid by every writer; the clamp also keeps a
            // caller's stray value from indexing outside the bucket table
            const int dxm = is_live ? (act[j] == 4) - (act[j] == 3) : 0;
            const int dym = is_live ? (act[j] == 1) - (act[j] == 2) : 0;
            const int nx = min(max(x[j] + dxm, 0), G - 1);
            const int ny = min(max(y[j] + dym, 0), G - 1);
            moved |= (nx != x[j]) | (ny != y[j]);
            x[j] = nx;
            y[j] = ny;
            packed[j] = pack_pos(nx, ny, is_live) | (is_live ? 0u : kStaleBit);
            if (is_live) {
              if constexpr (STRIP)
                strip_count(reinterpret_cast<uint32_t*>(L.starts), strip_bin(nx, ny, sg));
              else
                atomicAdd(&L.counts[bucket_of(nx, ny, bk)], 1u);
            }
            L.best[i0 + j] = key_none<Key>();
          }
          if (moved && write_state) {
            store4(p.pos_x, a0, n, vec, x);
            store4(p.pos_y, a0, n, vec, y);
          }
          *reinterpret_cast<uint4*>(L.pl + i0) = make_uint4(packed[0], packed[1], packed[2], packed[3]);
        }
      }
    }
    __syncthreads();
    WD_NEW_PHASE();
    if constexpr (STRIP)
      strip_scan_and_scatter(p, L, step_act, lt, ts, sg);
    else
      scan_and_scatter<WIDE>(p, L, step_act, lt, ts, bk);
    WD_NEW_PHASE();

    // ---- tag check, from the tagger's side: runners in range get the smallest
    //      (distance, tagger) key; min is order-independent, so the result is unique ----
    if constexpr (STRIP) {
      if (step_act && p.tag_r2 >= 0)
        for (int i = lt; i < N_tag; i += ts) strip_tag_scan(p, L, sg, i);
    } else if (step_act && p.tag_r2 >= 0) {
      for (int i = lt; i < N_tag; i += ts) {
        const uint32_t me = L.pl[i];
        const int x = pos_x_of(me), y = pos_y_of(me);
        const int bx0 = bucket_coord(max(x - p.tag_rad, 0), bk), bx1 = bucket_coord(min(x + p.tag_rad, G - 1), bk);
        const int by0 = bucket_coord(max(y - p.tag_rad, 0), bk), by1 = bucket_coord(min(y + p.tag_rad, G - 1), bk);
        for (int row = by0; row <= by1; ++row) {
          const uint32_t q_end = L.starts[row * bk.nbx + bx1 + 1];
          for (uint32_t q = L.starts[row * bk.nbx + bx0]; q < q_end; ++q) {
            const Ent ent = L.sorted.get(q);
            const int j = int(ent.id);
            if (j < N_tag) continue;
            const int dx = SL::x(ent) - x, dy = SL::y(ent) - y;
            const uint32_t d2 = uint32_t(__mul24(dx, dx)) + uint32_t(__mul24(dy, dy));
            if (d2 <= uint32_t(p.tag_r2)) atomicMin(&L.best[j], (Key(d2) << p.idx_bits) | Key(i));
          }
        }
      }
    }
    __syncthreads();
    WD_NEW_PHASE();
    // ---- runners in range leave the game and credit their tagger ---------------------------
    if (step_act) {
      int my_tags = 0;
      for (int k = 0; k < p.gpt; ++k) {
        const int i0 = 4 * (lt + k * ts);
        if (i0 + 3 >= N_tag && i0 < N) {
          bool any = false;
          int lv[4];
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const int i = i0 + j;
            uint32_t me = L.pl[i];
            if (i >= N_tag && i < N) {
              const Key b = L.best[i];
              if (b != key_none<Key>()) {
                me |= kDeadBit;
                L.pl[i] = me;
                if constexpr (STRIP)
                  L.sorted.pos[L.slot[i]] |= kStripDeadY << 16;
                else
                  L.sorted.mark_dead(L.slot[i]);
                atomicAdd(&L.credits[int(b & idx_mask)], 1);
                ++my_tags;
                any = true;
              }
            }
            lv[j] = (me & kDeadBit) ? 0 : 1;
          }
          if ((any || LOOPED) && write_state) store4(p.live, abase + i0, min(4, N - i0), vec, lv);
        }
      }
      if (my_tags) atomicAdd(&L.misc[0], my_tags);
    }
    __syncthreads();
    WD_NEW_PHASE();
    // ---- rewards, env clock and termination -----------------------------------------------
    if (step_act) {
      for (int k = 0; k < p.gpt; ++k) {
        const int i0 = 4 * (lt + k * ts);
        if (i0 < N) {
          float rew[4];
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const int i = i0 + j;
            rew[j] = 0.0f;
            if (i < N_tag)
              rew[j] = static_cast<float>(L.credits[i]) * p.tag_reward;
            else if (i < N && L.best[i] != key_none<Key>())
              rew[j] = p.tag_penalty;
          }
          store4(out.reward, abase + i0, min(4, N - i0), vec, rew);
        }
      }
      const int tags = L.misc[0];
      const int nlr = nlr_in - tags;
      nlr_out = nlr;
      t_out = t_in + 1;
      done_now = (nlr == 0) || (t_out >= p.T);
      if (lt == 0 && write_state) {
        p.t[e] = t_out;
        p.n_live_runners[e] = nlr;
        p.tags_step[e] = tags;
        p.done[e] = done_now ? 1 : 0;
      }
      out_act = true;
      if (lt == 0) {  // for the observation phase, where waves also serve teams other than their lanes' own
        L.misc[1] = t_out;
        L.misc[2] = 1;
        L.misc[kMiscStripMul] = int32_t(sg.mul);
        L.misc[kMiscStripRows] = sg.R;
      }
    }
    __syncthreads();  // tag keys and credits are read; the neighbour lists may overlay them
  }

  if (mode != kModeStep) {
    // ---- reset: restore the start state of envs that are done (or of all) ------------------
    if (out.done_log && valid && lt == 0) out.done_log[e] = done_now ? 1 : 0;  // the flag before the reset clears it
    const bool reset_act = valid && (mode == kModeResetAll || done_now);
    bool any_reset = true;
    if (mode == kModeIterate) {
      if constexpr (LOOPED) {
        if (reset_act && lt == 0) wg_flags[0] = 1;
        __syncthreads();
        any_reset = wg_flags[0] != 0;
      } else {
        any_reset = __syncthreads_or(reset_act ? 1 : 0) != 0;
      }
    }
    if (any_reset) {
      if (reset_act) {
        if constexpr (STRIP) {
          sg = choose_strips(p, N);
          strip_prepare(p, L, sg, lt, ts);
        } else {
          bk = choose_buckets(p, N);
          for (int j = lt; j < p.nb_cap; j += ts) L.counts[j] = 0u;
          for (int j = lt; j <= bk.nbx; j += ts) L.edges[j] = uint16_t(min(bucket_first_cell(j, bk), G));
        }
      }
      __syncthreads();
      if (reset_act) {
        for (int k = 0; k < p.gpt; ++k) {
          const int grp = lt + k * ts;
          if (grp < NG) {
            const int i0 = 4 * grp, n = min(4, N - i0);
            const int64_t a0 = abase + i0;
            int x[4], y[4];
            load4(p.pos_x0, a0, n, vec, x);
            load4(p.pos_y0, a0, n, vec, y);
            uint32_t packed[4];
            int ones[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              x[j] = min(max(x[j], 0), G - 1);
              y[j] = min(max(y[j], 0), G - 1);
              packed[j] = pack_pos(x[j], y[j], j < n);
              ones[j] = 1;
              if (j < n) {
                if constexpr (STRIP)
                  strip_count(reinterpret_cast<uint32_t*>(L.starts), strip_bin(x[j], y[j], sg));
                else
                  atomicAdd(&L.counts[bucket_of(x[j], y[j], bk)], 1u);
              }
            }
            if (write_state) {
              store4(p.pos_x, a0, n, vec, x);
              store4(p.pos_y, a0, n, vec, y);
              store4(p.live, a0, n, vec, ones);
            }
            *reinterpret_cast<uint4*>(L.pl + i0) = make_uint4(packed[0], packed[1], packed[2], packed[3]);
          }
        }
        t_out = 0;
        nlr_out = N - N_tag;
        if (lt == 0 && write_state) {
          p.t[e] = 0;
          p.n_live_runners[e] = N - N_tag;
          p.tags_step[e] = 0;
          p.done[e] = 0;
        }
        out_act = true;
        if (lt == 0) {
          L.misc[1] = 0;
          L.misc[2] = 1;
          L.misc[kMiscStripMul] = int32_t(sg.mul);
          L.misc[kMiscStripRows] = sg.R;
        }
      }
      __syncthreads();
      if constexpr (STRIP)
        strip_scan_and_scatter(p, L, reset_act, lt, ts, sg);
      else
        scan_and_scatter<WIDE>(p, L, reset_act, lt, ts, bk);
    }
  }

  if constexpr (LOOPED) {
    ls.t = t_out;
    ls.nlr = nlr_out;
    ls.resident = true;
  }
  WD_NEW_PHASE();
  // ---- observations ---------------------------------------------------------------------------
  // (misc[1], the env clock, and misc[2], "this env gets new rows", were written where the env was
  // stepped or reset, in front of a barrier)
  if constexpr (BIG) {
    // A large env hands its tables (positions, bucket-sorted list, bucket starts and edges) to
    // big_obs_kernel, which spreads the neighbour search and the rows of this env over many
    // workgroups: the kept and the sorted part of LDS go to device memory as they are.
    if (lt == 0) {
      L.misc[kMiscBucketMul] = int32_t(bk.mul);
      L.misc[kMiscBucketSide] = bk.nbx;
    }
    __syncthreads();
    if (valid) {
      uint4* image = reinterpret_cast<uint4*>(p.g_image + int64_t(e) * p.g_stride_image);
      const uint4* src = reinterpret_cast<const uint4*>(smem);
      for (int j = tid; j < p.y_base / 16; j += p.wg_size) image[j] = src[j];
    }
    return;
  }
  if constexpr (KX != -1) {
    constexpr int KT = register_list_size(KX);
    // K nearest, in bucket order (neighbouring lanes search neighbouring cells).  Two passes:
    // every live agent tries the 3x3 buckets around it; the few that this does not settle
    // (sparse spots, grid borders) queue up and are searched with widening rings afterwards,
    // packed into full waves, so that a wave of the first pass never waits for one such lane.
    // (a key of the strip search is empty, or an entry's that is out of play, from dead_key_min on)
    const auto is_none = [&](Key k) {
      if constexpr (STRIP) return k >= Key(p.dead_key_min);
      return key_is_none<WIDE>(k);
    };
    const auto put_neighbours_of = [&](const TeamLds<WIDE, BIG>& Lt, uint32_t me, const Key(&keys)[KT]) {
      if constexpr (CN) {
        uint32_t id[4];
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) id[kk] = is_none(keys[kk]) ? kCompactNone : uint32_t(keys[kk] & idx_mask);
        Lt.nbr_lo[me] = id[0] | (id[1] << 10) | (id[2] << 20) | (id[3] << 30);
        Lt.nbr_hi[me] = uint8_t(id[3] >> 2);
      } else {
#pragma unroll
        for (int kk = 0; kk < KT; ++kk)
          if (kk < K)
            Lt.nbr[me * K + kk] = is_none(keys[kk]) ? uint16_t(kNoNeighbour) : uint16_t(keys[kk] & idx_mask);
      }
    };
    const auto put_neighbours = [&](uint32_t me, const Key(&keys)[KT]) { put_neighbours_of(L, me, keys); };
    const bool search = out_act && K > 0;
    if (LOOPED && valid && !out_act && lt == 0) wg_flags[1] = 1;  // read after the two barriers below
    // Strip variant: a wave serves the teams that its lanes belong to one after the other, with all
    // 64 lanes (a team of 32 lanes or fewer shares its wave with others), so that everything that
    // depends on the team is uniform over the wave and lives in scalar registers.
    const int wave_teams = ONE ? 1 : (p.ts_log2 >= 6 ? 1 : kWaveSize >> p.ts_log2);
    const int wave_team0 = ONE ? 0 : (p.ts_log2 >= 6 ? team : (tid >> 6) * wave_teams);
    const int wave_lane = ONE ? tid : (p.ts_log2 >= 6 ? lt : (tid & (kWaveSize - 1)));
    const int wave_stride = p.ts_log2 >= 6 ? ts : kWaveSize;
    // calls body(tables, strips, number of agents in the list) for each of the wave's teams whose env gets new rows
    const auto for_each_wave_team = [&](auto body) {
      for (int w = 0; w < wave_teams; ++w) {
        const int tm = ONE ? 0 : __builtin_amdgcn_readfirstlane(wave_team0 + w);
        const TeamLds<WIDE, BIG> Lt(smem, tm, p, e0 + tm);
        if (K > 0 && __builtin_amdgcn_readfirstlane(Lt.misc[2]) != 0) {
          const Strips st = strips_of_env(p, uint32_t(__builtin_amdgcn_readfirstlane(Lt.misc[kMiscStripMul])),
                                          __builtin_amdgcn_readfirstlane(Lt.misc[kMiscStripRows]));
          body(Lt, st, __builtin_amdgcn_readfirstlane(int(Lt.starts[st.R * st.C])));
        }
      }
    };
    // One team per workgroup whose list is scanned whole (or that gets no new rows): nothing is ever
    // queued, so the two later tries and their barriers are left out; the whole workgroup agrees on it.
    bool no_retries = false;
    if constexpr (STRIP && ONE) {
      const TeamLds<WIDE, BIG> L0(smem, 0, p, e0);
      no_retries = __builtin_amdgcn_readfirstlane(L0.misc[2]) == 0;
      if (!no_retries) {
        const int rows = __builtin_amdgcn_readfirstlane(L0.misc[kMiscStripRows]);
        no_retries = __builtin_amdgcn_readfirstlane(int(L0.starts[rows * p.strip_C])) <= kStripScanAll;
      }
    }
    bool queued = false;  // this lane has put an agent into a retry queue
    if constexpr (STRIP) {
      // the fixed windows of the strip-sorted list; what they do not settle is queued
      for_each_wave_team([&](const TeamLds<WIDE, BIG>& Lt, const Strips st, int n_sorted) {
        const bool few = n_sorted <= kStripScanAll;  // (uniform: an env's whole list is cheaper than its windows)
        for (int q = wave_lane; q < n_sorted; q += wave_stride) {
          const uint32_t me = Lt.sorted.pos[q];
          if ((me >> 16) != kStripDeadY) {  // not tagged in this step
            Key keys[KT];
            if (few) {
              strip_scan_all<KX>(keys, me, uint32_t(q), uint32_t(n_sorted), p.key_shift, Lt.sorted.pos, Lt.sorted.id);
              put_neighbours_of(Lt, Lt.sorted.id[q], keys);
            } else if (strip_window_search<KX, strip_half_own(KX), strip_half_adj(KX), 0, false>(
                           keys, me, q, 0, st, p.key_shift, n_sorted, p.pad_l, Lt.sorted.pos, Lt.sorted.id, Lt.starts,
                           Lt.edges)) {
              put_neighbours_of(Lt, Lt.sorted.id[q], keys);
            } else {
              Lt.retry[atomicAdd(&Lt.misc[3], 1)] = uint16_t(q);
              queued = true;
            }
          }
        }
      });
      // second try, wider windows and two more strips, for the few that are queued; what is left
      // after that (hardly ever anything) waits in a short queue of its own for the block search
      // (two lanes per agent: an even lane takes what lies below the agent's slot, its odd neighbour
      // what lies above)
      // (no lane of the workgroup has queued anything: as good as no retries at all)
      // (workgroups of several small envs only: the roll-out loop and the one-env workgroups, which
      // nearly always have something queued, keep the plain barrier; the vote costs them more than it saves)
      if (!no_retries) {
        if constexpr (LOOPED || ONE)
          __syncthreads();
        else
          no_retries = __syncthreads_or(queued ? 1 : 0) == 0;
      }
      if (!no_retries) {
      const auto second_try = [&](const TeamLds<WIDE, BIG>& Lt, const Strips st, int n_sorted, int j, int side) {
        const int q = Lt.retry[j];
        const uint32_t me = Lt.sorted.pos[q];
        Key keys[KT];
        bool ok = strip_window_search<KX, strip_half_own2(KX), strip_half_adj2(KX), strip_half_far2(KX), true>(
            keys, me, q, side, st, p.key_shift, n_sorted, p.pad_l, Lt.sorted.pos, Lt.sorted.id, Lt.starts, Lt.edges);
        if (side) return;  // the even lane goes on for both
        if (!ok) {
          const int at = atomicAdd(&Lt.misc[kMiscQueue2], 1);
          if (at < kStripQueue2) {
            reinterpret_cast<uint16_t*>(Lt.misc + 4)[at] = uint16_t(q);  // (the scan scratch, idle by now)
          } else {  // the queue is full: search here and now
            strip_block_search<KX>(keys, me, uint32_t(q), st, p.key_shift, G, Lt.sorted.pos, Lt.sorted.id, Lt.starts,
                                   Lt.edges);
            ok = true;
          }
        }
        if (ok) put_neighbours_of(Lt, Lt.sorted.id[q], keys);
      };
      if constexpr (ONE) {
        for_each_wave_team([&](const TeamLds<WIDE, BIG>& Lt, const Strips st, int n_sorted) {
          const int n_retry = __builtin_amdgcn_readfirstlane(Lt.misc[3]);
          for (int j = wave_lane >> 1; j < n_retry; j += wave_stride >> 1) second_try(Lt, st, n_sorted, j, wave_lane & 1);
        });
      } else {
        // Several teams per workgroup: a team queues one or two agents as a rule, so the queues of all
        // teams are served as one list by the lane pairs of the whole workgroup (what depends on the
        // team is per lane here), instead of one run through this code per team.
        const int pairs = p.wg_size >> 1;
        for (int first = 0;; first += pairs) {
          const int i = first + (tid >> 1);
          int mine = -1, j = 0, seen = 0;
          for (int tm = 0; tm < p.teams_per_wg; ++tm) {
            const int32_t* m = reinterpret_cast<const int32_t*>(smem + tm * p.keep_stride + p.off_misc);
            const int c = (K > 0 && e0 + tm < p.E && m[2]) ? m[3] : 0;
            if (mine < 0 && i < seen + c) {
              mine = tm;
              j = i - seen;
            }
            seen += c;
          }
          if (first >= seen) break;  // (`seen` ends as the length of the whole list, the same in every lane)
          if (mine >= 0) {
            const TeamLds<WIDE, BIG> Lt(smem, mine, p, e0 + mine);
            const Strips st = strips_of_env(p, uint32_t(Lt.misc[kMiscStripMul]), Lt.misc[kMiscStripRows]);
            second_try(Lt, st, int(Lt.starts[st.R * st.C]), j, tid & 1);
          }
        }
      }
      }  // (!no_retries)
    } else if (search) {
      const int n_sorted = int(L.starts[p.nb_cap]);
      for (int q = lt; q < n_sorted; q += ts) {
        const Ent ent = L.sorted.get(q);
        if (!L.sorted.dead(ent)) {
          Key keys[KT];
          if (nearest_keys<WIDE, KT, true>(keys, K, SL::x(ent), SL::y(ent), uint32_t(q), bk, p.idx_bits, L.sorted,
                                           L.starts, L.edges))
            put_neighbours(ent.id, keys);
          else
            L.retry[atomicAdd(&L.misc[3], 1)] = uint16_t(q);
        }
      }
    }
    if (!no_retries) __syncthreads();
    if constexpr (STRIP) {
      if (!no_retries)
      for_each_wave_team([&](const TeamLds<WIDE, BIG>& Lt, const Strips st, int) {
        const int n_wait = min(__builtin_amdgcn_readfirstlane(Lt.misc[kMiscQueue2]), kStripQueue2);
        const uint16_t* const queue2 = reinterpret_cast<const uint16_t*>(Lt.misc + 4);
        for (int j = wave_lane; j < n_wait; j += wave_stride) {
          const uint32_t q = queue2[j];
          Key keys[KT];
          strip_block_search<KX>(keys, Lt.sorted.pos[q], q, st, p.key_shift, G, Lt.sorted.pos, Lt.sorted.id, Lt.starts,
                                 Lt.edges);
          put_neighbours_of(Lt, Lt.sorted.id[q], keys);
        }
      });
    } else if (search) {
      const int n_retry = L.misc[3];
      for (int j = lt; j < n_retry; j += ts) {
        const uint32_t q = L.retry[j];
        const Ent ent = L.sorted.get(q);
        Key keys[KT];
        nearest_keys<WIDE, KT, false>(keys, K, SL::x(ent), SL::y(ent), q, bk, p.idx_bits, L.sorted, L.starts, L.edges);
        put_neighbours(ent.id, keys);
      }
    }
    bool all_out;  // also the barrier after which the rows may overlay the sort tables
    if constexpr (LOOPED) {
      __syncthreads();
      all_out = wg_flags[1] == 0;
    } else {
      all_out = __syncthreads_and((out_act || !valid) ? 1 : 0) != 0;
    }

    WD_NEW_PHASE();
    // Rows, in index order.  A wave builds 64 rows in registers and sends them, 32 at a
    // time, through an LDS transpose (which overlays the sort tables) so that each store
    // instruction writes a contiguous run.
    const int wave = tid >> 6, lane = tid & (kWaveSize - 1);
    const int D = KX > 0 ? 5 + 4 * KX : p.D;
    const int rows_total = ONE ? N : min(p.teams_per_wg, p.E - e0) * N;
    float* const obs_wg = out.obs + int64_t(e0) * N * D;
    if (all_out) {
      const int srl = p.stage_rows_log2, stage_rows = 1 << srl, flushes = kWaveSize >> srl;
      float* stage = reinterpret_cast<float*>(smem + p.x_base) + wave * stage_rows * D;
      const bool vec_ok = (reinterpret_cast<uintptr_t>(obs_wg) & 15) == 0;  // (a roll-out slice may start on a 4-byte boundary)
      const int waves = p.wg_size >> 6;
      for (int c = wave; c * kWaveSize < rows_total; c += waves) {
        const int R0 = c * kWaveSize;
        const int Rr = R0 + lane;
        const bool have = Rr < rows_total;
        int tm = 0, i = Rr;
        if (!ONE && p.teams_per_wg > 1) {
          tm = int(fastdiv(uint32_t(Rr), p.div_N));
          i = Rr - tm * N;
        }
        const TeamLds<WIDE, BIG> Lr(smem, have ? tm : 0, p, e0 + (have ? tm : 0));
        const float t_frac = static_cast<float>(Lr.misc[1]) * p.inv_T;
        float row[5 + 4 * (KX > 0 ? KX : 1)];
        if constexpr (KX > 0) {
          if (have) write_row<KX, CN>(row, p, Lr, i, KX, t_frac);
        }
        if constexpr (KX > 0) {
          constexpr int DD = 5 + 4 * KX;
          // Two flushes of 32 rows = 8 DD 16-byte pieces each (168 at K = 4): kFull stores that
          // every lane takes part in and one more for the first kRem lanes.  A whole chunk has
          // no bounds to test; the last chunk of the workgroup stores only the pieces that exist
          // (its rows end on a 16-byte boundary when the row count times DD is a multiple of four).
          const auto flush_chunk = [&](auto whole_chunk) {
            constexpr bool kWhole = decltype(whole_chunk)::value;
            constexpr int kPieces = 32 * DD / 4;
            constexpr int kFull = kPieces / kWaveSize, kRem = kPieces % kWaveSize;
            const int limit = kWhole ? 0 : (rows_total - R0) * DD / 4 - lane;  // pieces of this chunk from this lane on
            float4* out4 = reinterpret_cast<float4*>(obs_wg + int64_t(R0) * DD) + lane;
            const float4* st4 = reinterpret_cast<const float4*>(stage) + lane;
            float* dst = stage + (lane & 31) * DD;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
              if ((lane >> 5) == h) {
#pragma unroll
                for (int d = 0; d < DD; ++d) dst[d] = row[d];
              }
              wave_sync_lds();
              if constexpr (kFull == 2) {
                // (K = 3, 4, written out: this form keeps the multi-step kernel's loop to the
                // fewest spilled registers)
                const float4 a = st4[0], b = st4[kWaveSize];
                float4 c = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
                if (lane < kRem) c = st4[2 * kWaveSize];
                if (kWhole || h * kPieces < limit) out4[h * kPieces] = a;
                if (kWhole || h * kPieces + kWaveSize < limit) out4[h * kPieces + kWaveSize] = b;
                if (lane < kRem && (kWhole || h * kPieces + 2 * kWaveSize < limit)) out4[h * kPieces + 2 * kWaveSize] = c;
              } else {
                // (the last load is unconditional, lanes from kRem on re-read the last staged piece
                // and store nothing: a predicated load makes the compiler emit the whole sequence
                // twice, once per half of the lanes)
                float4 v[kFull + 1];
#pragma unroll
                for (int m = 0; m < kFull; ++m) v[m] = st4[m * kWaveSize];
                v[kFull] = reinterpret_cast<const float4*>(stage)[min(kFull * kWaveSize + lane, kPieces - 1)];
#pragma unroll
                for (int m = 0; m < kFull; ++m)
                  if (kWhole || h * kPieces + m * kWaveSize < limit) out4[h * kPieces + m * kWaveSize] = v[m];
                if (kRem > 0 && lane < kRem && (kWhole || h * kPieces + kFull * kWaveSize < limit))
                  out4[h * kPieces + kFull * kWaveSize] = v[kFull];
              }
              wave_sync_lds();
            }
          };
          if (vec_ok && srl == 5) {
            if (R0 + kWaveSize <= rows_total) {
              flush_chunk(std::true_type{});
              continue;
            }
            if (((rows_total * DD) & 3) == 0) {
              flush_chunk(std::false_type{});
              continue;
            }
          }
        }
        for (int h = 0; h < flushes; ++h) {
          if (have && (lane >> srl) == h) {
            float* dst = stage + (lane & (stage_rows - 1)) * D;
            if constexpr (KX > 0) {
#pragma unroll
              for (int d = 0; d < 5 + 4 * KX; ++d) dst[d] = row[d];
            } else {
              write_row<0, false>(dst, p, Lr, i, K, t_frac);
            }
          }
          wave_sync_lds();
          const int nfl = min(max(rows_total - (R0 + h * stage_rows), 0), stage_rows) * D;
          float* out = obs_wg + int64_t(R0 + h * stage_rows) * D;
          if (vec_ok) {
            const int nvec = nfl >> 2;
            if constexpr (KX > 0 && KX <= 4) {  // at most 32 * 21 / 4 = 168 vectors: three predicated stores
#pragma unroll
              for (int it = 0; it < 3; ++it) {
                const int v = lane + it * kWaveSize;
                if (v < nvec) reinterpret_cast<float4*>(out)[v] = reinterpret_cast<const float4*>(stage)[v];
              }
            } else {
              for (int v = lane; v < nvec; v += kWaveSize)
                reinterpret_cast<float4*>(out)[v] = reinterpret_cast<const float4*>(stage)[v];
            }
            for (int f = (nvec << 2) + lane; f < nfl; f += kWaveSize) out[f] = stage[f];
          } else {
            // the rows start on a 4-byte boundary only: 16-byte stores at that alignment
            const int nvec = nfl >> 2;
            for (int v = lane; v < nvec; v += kWaveSize) {
              const float4 q = reinterpret_cast<const float4*>(stage)[v];
              reinterpret_cast<Quad32*>(out)[v] =
                  Quad32{__float_as_uint(q.x), __float_as_uint(q.y), __float_as_uint(q.z), __float_as_uint(q.w)};
            }
            for (int f = (nvec << 2) + lane; f < nfl; f += kWaveSize) out[f] = stage[f];
          }
          wave_sync_lds();
        }
      }
    } else {
      // some envs of this workgroup keep their rows: each lane writes its own row in place
      for (int Rr = tid; Rr < rows_total; Rr += p.wg_size) {
        const int tm = int(fastdiv(uint32_t(Rr), p.div_N));
        const int i = Rr - tm * N;
        const TeamLds<WIDE, BIG> Lr(smem, tm, p, e0 + tm);
        if (Lr.misc[2])
          write_row<(KX > 0 ? KX : 0), CN>(obs_wg + int64_t(Rr) * D, p, Lr, i, K, static_cast<float>(Lr.misc[1]) * p.inv_T);
      }
    }
  } else {
    __syncthreads();
    if (p.obs_mode == 1) {
      // Full observations (the second observation mode of Sec. 5.1): row i holds the own
      // features and one slot per agent j in index order, zeros unless both are in play.  The
      // team walks the N * N slots of its env; consecutive lanes write consecutive 16-byte
      // slots, so the stream to HBM is contiguous except for the five own features per row.
      if (out_act) {
        const int64_t D = p.D;
        float* env_obs = out.obs + abase * D;
        const float tf = static_cast<float>(t_out) * p.inv_T;
        if (vec && ts >= kWaveSize) {
          // N % 4 == 0: the env's block starts on a 16-byte boundary, and so does every fourth
          // float of it.  A wave takes a run of whole rows and writes them as ALIGNED 16-byte pieces; a
          // row starts 0..3 floats past such a boundary, so a piece holds the tail of one slot
          // and the head of the next, at an offset that is the same for the whole row.
          const int wv = lt >> 6, lane = lt & (kWaveSize - 1), n_waves = ts >> 6;
          const uint32_t Du = uint32_t(D);
          float4* const env_q = reinterpret_cast<float4*>(env_obs);
          const int rows_per_wave = (N + n_waves - 1) / n_waves;  // contiguous rows: one sequential stream per wave
          for (int i = wv * rows_per_wave; i < min(N, (wv + 1) * rows_per_wave); ++i) {
            const uint32_t row_f = uint32_t(i) * Du;                       // first float of row i in the block
            const uint32_t g_lo = (row_f + 3u) >> 2, g_hi = (row_f + Du + 3u) >> 2;  // pieces that start in row i
            const uint32_t shift = (4u * g_lo - row_f - 5u) & 3u;          // slot component a piece starts with
            const uint32_t me = L.pl[i];
            const auto emit = [&](uint32_t g) {
              const int c0 = int(4u * g - row_f);  // column of the piece's first float
              float4 v;
              if (c0 >= 5 && c0 + 3 < int(Du)) {
                const int ja = (c0 - 5) >> 2, jb = min(ja + 1, N - 1);
                const FullSlot A = full_slot(me, L.pl[ja], ja < N_tag, p.inv_G);
                const FullSlot B = full_slot(me, L.pl[jb], jb < N_tag, p.inv_G);
                switch (shift) {  // uniform over the wave
                  case 0: v = make_float4(A.a, A.b, A.c, A.d); break;
                  case 1: v = make_float4(A.b, A.c, A.d, B.a); break;
                  case 2: v = make_float4(A.c, A.d, B.a, B.b); break;
                  default: v = make_float4(A.d, B.a, B.b, B.c); break;
                }
              } else {
                // the piece holds own features, or runs into the next row (never past the
                // block: its length is a multiple of four floats)
                float f[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                  int col = c0 + k, r = i;
                  if (col >= int(Du)) {
                    col -= int(Du);
                    r = i + 1;
                  }
                  const uint32_t mr = L.pl[r];
                  if (col < 5) {
                    f[k] = col == 0   ? static_cast<float>(pos_x_of(mr)) * p.inv_G
                           : col == 1 ? static_cast<float>(pos_y_of(mr)) * p.inv_G
                           : col == 2 ? (r < N_tag ? 1.0f : 0.0f)
                           : col == 3 ? ((mr & kDeadBit) ? 0.0f : 1.0f)
                                      : tf;
                  } else {
                    const int j = (col - 5) >> 2, comp = (col - 5) & 3;
                    const FullSlot S = full_slot(mr, L.pl[j], j < N_tag, p.inv_G);
                    f[k] = comp == 0 ? S.a : comp == 1 ? S.b : comp == 2 ? S.c : S.d;
                  }
                }
                v = make_float4(f[0], f[1], f[2], f[3]);
              }
              env_q[g] = v;
            };
            // A row whose agent was out of play before the step began differs from what a kept
            // buffer holds in its time feature only: its first two pieces (one of them holds
            // that feature) and its last (which may run into the next row) are written.  A row
            // has at least five pieces.
            if (p.rows_kept && (me & kStaleBit)) {
              if (lane < 2)
                emit(g_lo + uint32_t(lane));
              else if (lane == 2)
                emit(g_hi - 1u);
            } else {
              for (uint32_t g = g_lo + uint32_t(lane); g < g_hi; g += kWaveSize) emit(g);
            }
          }
        } else {
          const uint32_t slots = uint32_t(N) * uint32_t(N);
          for (uint32_t u = uint32_t(lt); u < slots; u += uint32_t(ts)) {
            const uint32_t i = fastdiv(u, p.div_N);
            const uint32_t j = u - i * uint32_t(N);
            const uint32_t me = L.pl[i];
            float* row = env_obs + int64_t(i) * D;
            if (p.rows_kept && (me & kStaleBit)) {  // only the time feature of such a row changes
              if (j == 0) row[4] = tf;
              continue;
            }
            const FullSlot S = full_slot(me, L.pl[j], int(j) < N_tag, p.inv_G);
            Slot4 v;
            v.a = S.a;
            v.b = S.b;
            v.c = S.c;
            v.d = S.d;
            *reinterpret_cast<Slot4*>(row + 5 + 4 * j) = v;
            if (j == 0) {
              row[0] = static_cast<float>(pos_x_of(me)) * p.inv_G;
              row[1] = static_cast<float>(pos_y_of(me)) * p.inv_G;
              row[2] = int(i) < N_tag ? 1.0f : 0.0f;
              row[3] = (me & kDeadBit) ? 0.0f : 1.0f;
              row[4] = tf;
            }
          }
        }
      }
    } else if (out_act) {
      // any K: sixteen neighbours at a time by the ring search, each further sixteen as the smallest
      // keys above the last one found (keys are unique, so no agent comes twice); rows written in place
      const int D = p.D;
      const float tf = static_cast<float>(t_out) * p.inv_T;
      for (int i = lt; i < N; i += ts) {
        float* row = out.obs + (abase + i) * D;
        const uint32_t me = L.pl[i];
        if (p.rows_kept && (me & kStaleBit)) {  // only the time feature of such a row changes
          row[4] = tf;
          continue;
        }
        const int x = pos_x_of(me), y = pos_y_of(me);
        const bool lv = !(me & kDeadBit);
        row[0] = static_cast<float>(x) * p.inv_G;
        row[1] = static_cast<float>(y) * p.inv_G;
        row[2] = i < N_tag ? 1.0f : 0.0f;
        row[3] = lv ? 1.0f : 0.0f;
        row[4] = tf;
        bool exhausted = !lv;  // no further neighbour exists
        Key floor = 0;
        for (int k0 = 0; k0 < K; k0 += kMaxRegisterK2) {
          const int kc = min(kMaxRegisterK2, K - k0);
          Key keys[kMaxRegisterK2];
          if (!exhausted) {
            const uint32_t self_slot = L.slot[i];
            if (k0 == 0)
              nearest_keys<WIDE, kMaxRegisterK2, false>(keys, kc, x, y, self_slot, bk, p.idx_bits, L.sorted, L.starts,
                                                        L.edges);
            else
              nearest_keys<WIDE, kMaxRegisterK2, false, true>(keys, kc, x, y, self_slot, bk, p.idx_bits, L.sorted,
                                                              L.starts, L.edges, floor);
          }
#pragma unroll
          for (int kk = 0; kk < kMaxRegisterK2; ++kk) {
            if (kk < kc) {
              float f0 = 0.0f, f1 = 0.0f, f2 = 0.0f, f3 = 0.0f;
              if (!exhausted && !key_is_none<WIDE>(keys[kk])) {
                const int j = int(keys[kk] & idx_mask);
                const uint32_t other = L.pl[j];
                f0 = static_cast<float>(pos_x_of(other) - x) * p.inv_G;
                f1 = static_cast<float>(pos_y_of(other) - y) * p.inv_G;
                f2 = j < N_tag ? 1.0f : 0.0f;
                f3 = 1.0f;
                floor = keys[kk];
              } else {
                exhausted = true;
              }
              float* slot_out = row + 5 + 4 * (k0 + kk);
              slot_out[0] = f0;
              slot_out[1] = f1;
              slot_out[2] = f2;
              slot_out[3] = f3;
            }
          }
        }
      }
    }
  }
}

#undef p
#undef WD_NEW_PHASE

template <int WIDE, int KX, bool CN, bool BIG, bool ONE>
__global__ __launch_bounds__(BIG ? kBigEnvWorkgroupSize : kMaxEnvWorkgroupSize)
    __attribute__((amdgpu_waves_per_eu((WIDE || BIG || KX <= 1 || KX > 4) ? 4 : 8, 8))) void env_kernel(const Params p, const int mode,
                                                             const float* __restrict__ probs, uint32_t g_lo,
                                                             uint32_t g_hi) {
  extern __shared__ __align__(16) unsigned char smem[];
  LoopState ls = {0, 0, false, true};
  // p is the first kernel argument: offset 0 of the kernel-argument segment
  env_body<WIDE, KX, CN, BIG, false, ONE>((KernargParams)__builtin_amdgcn_kernarg_segment_ptr(),
                                     StepOut{p.action, p.reward, p.obs, p.done_log}, mode, probs, g_lo, g_hi, smem,
                                     int(threadIdx.x), ls);
}

// ----------------------------------------------------------------------------------
// Observations of large envs.  env_kernel<..., BIG> leaves each env's tables in device memory;
// here workgroup (e, s) reloads them into LDS and serves slice s of env e: the live agents in
// slots [s, s + 1) * chunk of the bucket-sorted list search their K nearest and write their
// rows straight from registers, and the agents of index slice s that are out of the game get
// their rows of zeros.  A row is 20 + 16 K contiguous bytes; the rows of a large-env batch are
// a few megabytes, so scattered rows cost nothing that matters.
// ----------------------------------------------------------------------------------
template <int WIDE, int KX>
__global__ __launch_bounds__(kBigObsWorkgroupSize) void big_obs_kernel(const Params p) {
  extern __shared__ __align__(16) unsigned char smem[];
  using SL = SortedList<WIDE>;
  using Key = typename SL::Key;
  constexpr int KT = register_list_size(KX);
  const int tid = threadIdx.x;
  const int e = blockIdx.x / p.big_slices, s = blockIdx.x - e * p.big_slices;
  {
    const uint4* image = reinterpret_cast<const uint4*>(p.g_image + int64_t(e) * p.g_stride_image);
    uint4* dst = reinterpret_cast<uint4*>(smem);
    for (int j = tid; j < p.y_base / 16; j += kBigObsWorkgroupSize) dst[j] = image[j];
  }
  __syncthreads();
  const TeamLds<WIDE, true> L(smem, 0, p, e);
  if (!L.misc[2]) return;  // this env keeps its rows (a step call on an env that was done)
  Buckets bk;
  bk.mul = uint32_t(L.misc[kMiscBucketMul]);
  bk.nbx = L.misc[kMiscBucketSide];
  bk.bmin = 0;
  const int N = p.N, K = KX > 0 ? KX : p.K;
  const int64_t D = KX > 0 ? 5 + 4 * KX : p.D;
  float* const env_obs = p.obs + int64_t(e) * N * D;
  const float t_frac = static_cast<float>(L.misc[1]) * p.inv_T;
  // live agents, in bucket order
  const int n_sorted = int(L.starts[p.nb_cap]);
  const int q_chunk = (n_sorted + p.big_slices - 1) / p.big_slices;
  const int q_end = min(n_sorted, (s + 1) * q_chunk);
  for (int q = s * q_chunk + tid; q < q_end; q += kBigObsWorkgroupSize) {
    const Ent ent = L.sorted.get(q);
    if (L.sorted.dead(ent)) continue;  // tagged in this step: served below
    Key keys[KT];
    if (K > 0) {
      nearest_keys<WIDE, KT, false>(keys, K, SL::x(ent), SL::y(ent), uint32_t(q), bk, p.idx_bits, L.sorted, L.starts,
                                    L.edges);
    } else {
#pragma unroll
      for (int kk = 0; kk < KT; ++kk) keys[kk] = key_none<Key>();
    }
    store_row<WIDE, KT>(env_obs + int64_t(ent.id) * D, p, L.pl, int(ent.id), K, t_frac, keys, true);
  }
  // agents out of the game, in index order
  const int i_chunk = (N + p.big_slices - 1) / p.big_slices;
  const int i_end = min(N, (s + 1) * i_chunk);
  for (int i = s * i_chunk + tid; i < i_end; i += kBigObsWorkgroupSize) {
    const uint32_t me = L.pl[i];
    if (!(me & kDeadBit)) continue;
    if (p.rows_kept && (me & kStaleBit)) {  // out of play before this step: only the time feature changes
      env_obs[int64_t(i) * D + 4] = t_frac;
      continue;
    }
    Key keys[KT];
#pragma unroll
    for (int kk = 0; kk < KT; ++kk) keys[kk] = key_none<Key>();
    store_row<WIDE, KT>(env_obs + int64_t(i) * D, p, L.pl, i, K, t_frac, keys, false);
  }
}

// ----------------------------------------------------------------------------------
// Large envs of a small batch: the step spread over many workgroups (Sec. 4.5 item 4 holds the step
// at constant time only while an env has a thread per agent; this is the layout past that point).
//
// spread_move_kernel, workgroup (e, s): lane l of the first two waves owns group 128 s + l of env
// e: samples (iterate mode), moves, and checks its live runners against the taggers.  The tag check
// needs every tagger's position after the move, and a tagger's position is written in place by
// nobody in this kernel (a workgroup reading it could otherwise meet the new value): every
// workgroup moves all taggers of its env itself, in its other two waves, into a table in LDS
// (taggers chained by coarse cell), and the second kernel writes their positions.  A runner then
// takes the smallest (distance, tagger) pair in range, which is what the tagger-side scan with a
// minimum per runner gives.  Global atomics collect credits and the number of tags.
// ----------------------------------------------------------------------------------
struct GroupInput {  // what a group's move needs from memory
  float f[20];
  int act[4], x[4], y[4], lv[4];
};
struct MovedGroup {
  int act[4], x[4], y[4], lv[4];
  int n;
  bool moved;
};

// Loads only: a caller issues those of several groups before it waits for any.  The state is read
// whether or not the env is stepped, so that the loads do not wait for its done flag either.
__device__ __forceinline__ void load_group(const Params& p, int mode, const float* __restrict__ probs, int e, int grp,
                                           GroupInput& in) {
  const int i0 = 4 * grp, n = min(4, p.N - i0);
  const bool vec = p.vec4 != 0;
  const int64_t a0 = int64_t(e) * p.N + i0;
  if (mode == kModeIterate) {
    load_group_probs(probs, a0, n, vec, in.f);
  } else {
    load4(p.action, a0, n, vec, in.act);
  }
  load4(p.pos_x, a0, n, vec, in.x);
  load4(p.pos_y, a0, n, vec, in.y);
  load4(p.live, a0, n, vec, in.lv);
}

__device__ __forceinline__ void move_group(const Params& p, int mode, int e, int grp, uint32_t g_lo, uint32_t g_hi,
                                           bool step_act, const GroupInput& in, MovedGroup& m) {
  m.n = min(4, p.N - 4 * grp);
  m.moved = false;
  if (mode == kModeIterate) {
    const Block4 r = random_block(p, uint32_t(e), uint32_t(grp), g_lo, g_hi, kStreamAction);
    draw_group(in.f, r, m.act);
  } else {
#pragma unroll
    for (int j = 0; j < 4; ++j) m.act[j] = in.act[j];
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const bool is_live = step_act && j < m.n && in.lv[j] != 0;
    const int dxm = is_live ? (m.act[j] == 4) - (m.act[j] == 3) : 0;
    const int dym = is_live ? (m.act[j] == 1) - (m.act[j] == 2) : 0;
    const int nx = min(max(in.x[j] + dxm, 0), p.G - 1);
    const int ny = min(max(in.y[j] + dym, 0), p.G - 1);
    m.moved |= (nx != in.x[j]) | (ny != in.y[j]);
    m.x[j] = nx;
    m.y[j] = ny;
    m.lv[j] = is_live ? 1 : 0;
  }
}

__global__ __launch_bounds__(2 * kSpreadMoveThreads) void spread_move_kernel(const Params p, const int mode,
                                                                             const float* __restrict__ probs, uint32_t g_lo,
                                                                             uint32_t g_hi) {
  __shared__ int32_t head[kSpreadTagSide * kSpreadTagSide];  // last tagger put into each coarse cell, -1: none
  __shared__ uint32_t tagger_pos[kSpreadMaxTaggers];         // x | y << 16 after the move
  __shared__ int16_t next_in_cell[kSpreadMaxTaggers];
  // Two halves of kSpreadMoveThreads lanes: the first moves and checks the slice's own groups, the
  // second moves the env's taggers into the table meanwhile (half the chain of either doing both).
  const int tid = threadIdx.x, lt = tid & (kSpreadMoveThreads - 1);
  const bool tagger_half = tid >= kSpreadMoveThreads;
  const int e = blockIdx.x / p.spread_slices, s = blockIdx.x - e * p.spread_slices;
  const int done_in = p.done[e], t_in = p.t[e], nlr_in = p.n_live_runners[e];
  if (s == 0 && tid == 0) {  // the second kernel overwrites these while its other workgroups still need them
    p.g_env[4 * e + 0] = done_in;
    p.g_env[4 * e + 1] = t_in;
    p.g_env[4 * e + 2] = nlr_in;
  }
  if (mode != kModeStep && mode != kModeIterate) return;
  const int N = p.N, N_tag = p.N_tag;
  // this lane's group (own half) or its first group of taggers (other half): the loads go out before anything waits
  const int grp = s * kSpreadMoveThreads + lt;
  const bool have = !tagger_half && grp < p.NG, have_tagger = tagger_half && p.tag_r2 >= 0 && 4 * lt < N_tag;
  GroupInput in;
  if (have) load_group(p, mode, probs, e, grp, in);
  if (have_tagger) load_group(p, mode, probs, e, lt, in);
  const bool step_act = !done_in;
  const bool tagging = step_act && p.tag_r2 >= 0;
  Buckets tb;
  tb.mul = p.tag_mul;
  tb.nbx = p.tag_nbx;
  tb.bmin = 0;
  if (tagging)
    for (int j = tid; j < tb.nbx * tb.nbx; j += 2 * kSpreadMoveThreads) head[j] = -1;
  MovedGroup mine;
  mine.n = 0;
  if (have) move_group(p, mode, e, grp, g_lo, g_hi, step_act, in, mine);
  if (have_tagger) move_group(p, mode, e, lt, g_lo, g_hi, step_act, in, mine);
  __syncthreads();
  if (tagging && tagger_half) {
    for (int tg = lt; 4 * tg < N_tag; tg += kSpreadMoveThreads) {
      if (tg != lt) {  // more taggers than one group per lane
        load_group(p, mode, probs, e, tg, in);
        move_group(p, mode, e, tg, g_lo, g_hi, true, in, mine);
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int i = 4 * tg + j;
        if (i < N_tag) {
          tagger_pos[i] = uint32_t(mine.x[j]) | (uint32_t(mine.y[j]) << 16);
          next_in_cell[i] = int16_t(atomicExch(&head[bucket_of(mine.x[j], mine.y[j], tb)], i));
        }
      }
    }
  }
  __syncthreads();
  if (!have) return;
  const int i0 = 4 * grp;
  const int64_t a0 = int64_t(e) * N + i0;
  const bool vec = p.vec4 != 0;
  if (mode == kModeIterate) store4(p.action, a0, mine.n, vec, mine.act);
  if (!step_act) return;
  uint32_t* const acc = p.g_acc + (int64_t(p.spread_parity) * p.E + e) * p.g_stride_acc;
  int my_tags = 0;
  bool live_after[4];
  // A coarse cell is at least a tag radius wide, so a runner's reach touches at most 3 x 3 of them.
  // The heads of all of them, for the four agents, are read before any chain is followed: 36 reads
  // in flight instead of 36 in a row (a cell beyond the reach repeats the last one in it and is dropped).
  int heads[4][9];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int x = mine.x[j], y = mine.y[j];
    const int bx0 = bucket_coord(max(x - p.tag_rad, 0), tb), bx1 = bucket_coord(min(x + p.tag_rad, p.G - 1), tb);
    const int by0 = bucket_coord(max(y - p.tag_rad, 0), tb), by1 = bucket_coord(min(y + p.tag_rad, p.G - 1), tb);
    live_after[j] = mine.lv[j] != 0;
    const bool check = tagging && live_after[j] && i0 + j >= N_tag;
#pragma unroll
    for (int r = 0; r < 3; ++r)
#pragma unroll
      for (int c = 0; c < 3; ++c) {
        const int h = tagging ? head[min(by0 + r, by1) * tb.nbx + min(bx0 + c, bx1)] : -1;
        heads[j][3 * r + c] = (check && by0 + r <= by1 && bx0 + c <= bx1) ? h : -1;
      }
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int x = mine.x[j], y = mine.y[j];
    uint32_t best_d2 = ~0u;
    int best_i = -1;
#pragma unroll
    for (int k = 0; k < 9; ++k)
      for (int c = heads[j][k]; c >= 0; c = next_in_cell[c]) {
        const uint32_t tp = tagger_pos[c];
        const int dx = int(tp & 0xFFFFu) - x, dy = int(tp >> 16) - y;
        const uint32_t d2 = uint32_t(__mul24(dx, dx)) + uint32_t(__mul24(dy, dy));
        if (d2 <= uint32_t(p.tag_r2) && (d2 < best_d2 || (d2 == best_d2 && c < best_i))) {
          best_d2 = d2;
          best_i = c;
        }
      }
    if (best_i >= 0) {
      live_after[j] = false;
      atomicAdd(&acc[p.acc_credits + best_i], 1u);
      ++my_tags;
    }
  }
  if (my_tags) atomicAdd(&acc[p.acc_tags], uint32_t(my_tags));
  uint32_t packed[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    // (dead bit alone: tagged in this step; with the stale bit: out of play before it)
    packed[j] = pack_pos(mine.x[j], mine.y[j], live_after[j]) | (mine.lv[j] ? 0u : kStaleBit);
    mine.lv[j] = live_after[j] ? 1 : 0;
  }
  *reinterpret_cast<uint4*>(p.g_pl + int64_t(e) * p.NPAD + i0) = make_uint4(packed[0], packed[1], packed[2], packed[3]);
  if (mine.moved && i0 >= N_tag) {
    store4(p.pos_x, a0, mine.n, vec, mine.x);
    store4(p.pos_y, a0, mine.n, vec, mine.y);
  }
  if (my_tags) store4(p.live, a0, mine.n, vec, mine.lv);
}

// spread_obs_kernel, workgroup (e, s): finishes the step of env e for index slice s (rewards, the
// taggers' positions, and in slice 0 the env's clock, counts and done flag, from the complete
// accumulators), resets the env if it is done (iterate and reset modes), then builds the env's
// tables in LDS: after a step from the packed positions, the bucket counts and the ranks that
// spread_move_kernel left (scan of the counts, then every live agent goes to start of its bucket +
// its rank: no counting pass), after a reset by a counting sort of the start positions.  Every
// workgroup of an env builds the same tables; then it serves its slice as big_obs_kernel does.
template <int WIDE, int KX>
__global__ __launch_bounds__(kSpreadObsThreads) void spread_obs_kernel(const Params p, const int mode) {
  extern __shared__ __align__(16) unsigned char smem[];
  using SL = SortedList<WIDE>;
  using Key = typename SL::Key;
  constexpr int KT = register_list_size(KX);
  constexpr int ts = kSpreadObsThreads;
  const int tid = threadIdx.x;
  const int e = blockIdx.x / p.big_slices, s = blockIdx.x - e * p.big_slices;
  const int N = p.N, N_tag = p.N_tag, G = p.G, K = KX > 0 ? KX : p.K;
  const bool vec = p.vec4 != 0;
  const int64_t abase = int64_t(e) * N;
  const TeamLds<WIDE, true> L(smem, 0, p, e);
  const int done_in = p.g_env[4 * e + 0], t_in = p.g_env[4 * e + 1], nlr_in = p.g_env[4 * e + 2];
  const bool stepping = mode == kModeStep || mode == kModeIterate;
  const uint32_t* const acc = p.g_acc + (int64_t(p.spread_parity) * p.E + e) * p.g_stride_acc;
  const uint32_t* const env_pl = p.g_pl + int64_t(e) * p.NPAD;
  const int acc_tags = int(acc[p.acc_tags]);
  // The packed positions of a stepped env go straight into LDS, and the bucket counters are cleared,
  // before anything waits for the env's scalars (a reset does not use the positions).
  {
    const uint4* src = reinterpret_cast<const uint4*>(env_pl);
    uint4* dst = reinterpret_cast<uint4*>(L.pl);
#pragma unroll 2
    for (int j = tid; j < p.NPAD / 4; j += ts) dst[j] = src[j];
    for (int j = tid; j < p.nb_cap; j += ts) L.counts[j] = 0u;
  }
  if (stepping) {  // the other set of accumulators is clear when the next call's first kernel starts
    uint32_t* const other = p.g_acc + (int64_t(p.spread_parity ^ 1) * p.E + e) * p.g_stride_acc;
    for (int64_t j = int64_t(s) * ts + tid; j < p.g_stride_acc; j += int64_t(p.big_slices) * ts) other[j] = 0u;
  }
  const bool stepped = stepping && !done_in;
  int t_out = t_in, tags = 0;
  bool done_now = done_in != 0;
  if (stepped) {
    tags = acc_tags;
    t_out = t_in + 1;
    done_now = (nlr_in - tags == 0) || (t_out >= p.T);
  }
  const bool reset_act = mode != kModeStep && (mode == kModeResetAll || done_now);
  if (mode != kModeStep && p.done_log && s == 0 && tid == 0) p.done_log[e] = done_now ? 1 : 0;
  if (!stepped && !reset_act) return;  // this env keeps its state and its rows
  const int i_chunk = (N + p.big_slices - 1) / p.big_slices;
  const int i_begin = s * i_chunk, i_end = min(N, i_begin + i_chunk);
  if (stepped) {
    // rewards of this slice and the positions of the groups that hold a tagger, from the quads this
    // thread has just put into LDS itself
    const int tag_groups_end = 4 * ((N_tag + 3) / 4);
    for (int k = 0; k < p.gpt; ++k) {
      const int i0 = 4 * (tid + k * ts);
      if (i0 + 3 >= i_begin && i0 < i_end) {
        const uint4 v4 = *reinterpret_cast<const uint4*>(L.pl + i0);
        const uint32_t v[4] = {v4.x, v4.y, v4.z, v4.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int i = i0 + j;
          if (i >= i_begin && i < i_end) {
            float rew = 0.0f;
            if (i < N_tag)
              rew = static_cast<float>(int(acc[p.acc_credits + i])) * p.tag_reward;
            else if ((v[j] & kDeadBit) && !(v[j] & kStaleBit))
              rew = p.tag_penalty;
            p.reward[abase + i] = rew;
            if (i < tag_groups_end) {
              p.pos_x[abase + i] = pos_x_of(v[j]);
              p.pos_y[abase + i] = pos_y_of(v[j]);
            }
          }
        }
      }
    }
    if (s == 0 && tid == 0) {
      p.t[e] = t_out;
      p.n_live_runners[e] = nlr_in - tags;
      p.tags_step[e] = tags;
      p.done[e] = done_now ? 1 : 0;
    }
  }
  // The tables: a counting sort of the live agents by bucket, from the start positions after a reset,
  // else from the packed positions in LDS (a thread counts the groups it put there itself).  Counting
  // in the first kernel instead, with global atomics, was measured: they cost it two microseconds
  // whether or not anything waits for what they return.
  const Buckets bk = choose_buckets(p, reset_act ? N : nlr_in + N_tag);
  for (int j = tid; j <= bk.nbx; j += ts) L.edges[j] = uint16_t(min(bucket_first_cell(j, bk), G));
  __syncthreads();  // the counters are clear
  for (int k = 0; k < p.gpt; ++k) {
    const int grp = tid + k * ts;
    if (grp < p.NG) {
      const int i0 = 4 * grp, n = min(4, N - i0);
      uint32_t packed[4];
      if (reset_act) {
        int x[4], y[4];
        load4(p.pos_x0, abase + i0, n, vec, x);
        load4(p.pos_y0, abase + i0, n, vec, y);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          x[j] = min(max(x[j], 0), G - 1);
          y[j] = min(max(y[j], 0), G - 1);
          packed[j] = pack_pos(x[j], y[j], j < n);
          const int i = i0 + j;
          if (j < n && i >= i_begin && i < i_end) {  // this slice's part of the state
            p.pos_x[abase + i] = x[j];
            p.pos_y[abase + i] = y[j];
            p.live[abase + i] = 1;
          }
        }
        *reinterpret_cast<uint4*>(L.pl + i0) = make_uint4(packed[0], packed[1], packed[2], packed[3]);
      } else {
        const uint4 v4 = *reinterpret_cast<const uint4*>(L.pl + i0);
        packed[0] = v4.x;
        packed[1] = v4.y;
        packed[2] = v4.z;
        packed[3] = v4.w;
      }
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (!(packed[j] & kDeadBit)) atomicAdd(&L.counts[bucket_of(pos_x_of(packed[j]), pos_y_of(packed[j]), bk)], 1u);
    }
  }
  if (reset_act) {
    t_out = 0;
    if (s == 0 && tid == 0) {
      p.t[e] = 0;
      p.n_live_runners[e] = N - N_tag;
      p.tags_step[e] = 0;
      p.done[e] = 0;
    }
  }
  __syncthreads();
  scan_and_scatter<WIDE>(p, L, true, tid, ts, bk);

  const int64_t D = KX > 0 ? 5 + 4 * KX : p.D;
  float* const env_obs = p.obs + abase * D;
  const float t_frac = static_cast<float>(t_out) * p.inv_T;
  // live agents, in bucket order
  const int n_sorted = int(L.starts[p.nb_cap]);
  const int q_chunk = (n_sorted + p.big_slices - 1) / p.big_slices;
  int q_begin = min(n_sorted, s * q_chunk), q_end = min(n_sorted, (s + 1) * q_chunk);
  {
    // The counting sort leaves the order inside a bucket to chance, so the lists of an env's workgroups
    // agree on the buckets only: a slice runs from the first bucket start at or behind its first slot
    // to the first at or behind its end.  Every thread looks at its own few bucket starts (a binary
    // search would be two dozen dependent reads for every thread).
    int32_t* const bound = L.misc + 4;  // (scan scratch, free again)
    const int j0 = tid * p.scan_chunk;
    int prev = j0 ? int(L.starts[j0 - 1]) : -1;
    for (int c = 0; c <= p.scan_chunk; ++c) {
      const int j = j0 + c;
      if (c == p.scan_chunk && tid != ts - 1) break;  // (entry nb_cap, the number of agents, belongs to the last thread)
      const int v = int(L.starts[j]);
      if (v >= q_begin && prev < q_begin) bound[0] = v;
      if (v >= q_end && prev < q_end) bound[1] = v;
      prev = v;
    }
    __syncthreads();
    q_begin = bound[0];
    q_end = bound[1];
  }
  // Two neighbouring lanes per agent: each searches half of the candidates and writes half of the
  // row (collecting a wave's rows in LDS and writing them out whole was measured: slower).
  const int side = tid & 1;
  for (int q = q_begin + (tid >> 1); q < q_end; q += ts / 2) {
    const Ent ent = L.sorted.get(q);
    Key keys[KT];
    if (K > 0) {
      nearest_keys_pair<WIDE, KT>(keys, K, SL::x(ent), SL::y(ent), uint32_t(q), side, bk, p.idx_bits, L.sorted,
                                  L.starts, L.edges);
    } else {
#pragma unroll
      for (int kk = 0; kk < KT; ++kk) keys[kk] = key_none<Key>();
    }
    store_row_half<WIDE, KT>(env_obs + int64_t(ent.id) * D, p, L.pl, int(ent.id), K, t_frac, keys, side);
  }
  // agents out of the game, in index order
  for (int i = i_begin + tid; i < i_end; i += ts) {
    const uint32_t me = L.pl[i];
    if (!(me & kDeadBit)) continue;
    if (p.rows_kept && (me & kStaleBit)) {  // out of play before this step: only the time feature changes
      env_obs[int64_t(i) * D + 4] = t_frac;
      continue;
    }
    Key keys[KT];
#pragma unroll
    for (int kk = 0; kk < KT; ++kk) keys[kk] = key_none<Key>();
    store_row<WIDE, KT>(env_obs + int64_t(i) * D, p, L.pl, i, K, t_frac, keys, false);
  }
}

// Workgroup-wide copy of `count` 4-byte words: 16-byte pieces when both ends are aligned.
template <typename T>
__device__ __forceinline__ void copy_words(T* __restrict__ dst, const T* __restrict__ src, int64_t count) {
  static_assert(sizeof(T) == 4, "4-byte elements");
  const bool aligned = ((reinterpret_cast<uintptr_t>(dst) | reinterpret_cast<uintptr_t>(src)) & 15) == 0;
  const int64_t quads = aligned ? count >> 2 : 0;
  for (int64_t i = threadIdx.x; i < quads; i += blockDim.x)
    reinterpret_cast<uint4*>(dst)[i] = reinterpret_cast<const uint4*>(src)[i];
  for (int64_t i = 4 * quads + threadIdx.x; i < count; i += blockDim.x) dst[i] = src[i];
}

// Several roll-out iterations in one launch.  Envs never interact, so a workgroup can run its
// envs through `steps` iterations on its own: step s samples from ring entry (ring_pos + s) mod
// ring_len, writes action / reward / observations of that iteration to the s-th slice of the
// roll-out buffers (the data a trainer batches, Sec. 4.5 item 7) and the done flags as they
// were before the reset; the last iteration writes the caller's in-place buffers, from which
// the last slice is then copied.
struct RollArgs {  // the one kernel argument of rollout_kernel
  Params p;
  Roll roll;
  const float* ring;
  uint64_t g0;
};

template <int WIDE, int KX, bool CN, bool ONE>
__global__ __launch_bounds__(kMaxEnvWorkgroupSize)
    __attribute__((amdgpu_waves_per_eu((WIDE || KX <= 1 || KX > 4) ? 4 : 8, 8))) void rollout_kernel(const RollArgs args) {
  extern __shared__ __align__(16) unsigned char smem[];
  // The loop reads its parameters from the kernel-argument segment (args is the only argument,
  // at offset 0) through a pointer that is opaque to the optimiser in every iteration: loads of
  // the many fields then stay next to their uses, as in the one-step kernel, instead of being
  // hoisted out of the loop into more scalar registers than there are.
  typedef const __attribute__((address_space(4))) RollArgs* KernargPtr;
  KernargPtr ak = (KernargPtr)__builtin_amdgcn_kernarg_segment_ptr();
  const int steps = args.roll.steps;
  int ring_at = args.roll.ring_pos;
  int tid = threadIdx.x;
  LoopState ls = {0, 0, false, false};
  for (int s = 0; s < steps; ++s) {
    ls.last = s + 1 == steps;
    asm volatile("" : "+s"(ak));
    asm volatile("" : "+v"(tid));  // likewise: what a thread derives from its id is recomputed per step, not kept
    const RollArgs& a = *(const RollArgs*)ak;
    const Params& p = a.p;
    const Roll& roll = a.roll;
    const int64_t EN = int64_t(p.E) * p.N;
    StepOut out = {p.action, p.reward, p.obs, roll.done ? roll.done + int64_t(s) * p.E : nullptr};
    if (s + 1 < steps) {
      if (roll.action) out.action = roll.action + s * EN;
      if (roll.reward) out.reward = roll.reward + s * EN;
      if (roll.obs) out.obs = roll.obs + s * EN * p.D;
    }
    const uint64_t g = a.g0 + uint64_t(s);
    env_body<WIDE, KX, CN, false, true, ONE>((KernargParams)ak, out, kModeIterate, a.ring + int64_t(ring_at) * EN * kNumActions, uint32_t(g),
                                  uint32_t(g >> 32), smem, tid, ls);
    ring_at = ring_at + 1 == roll.ring_len ? 0 : ring_at + 1;
    __syncthreads();  // this step's state and LDS use are complete before the next step starts
  }
  const Params& p = args.p;
  const Roll& roll = args.roll;
  const int64_t EN = int64_t(p.E) * p.N;
  const int e0 = blockIdx.x * p.teams_per_wg;
  const int64_t first = int64_t(e0) * p.N;
  const int64_t count = int64_t(min(p.teams_per_wg, p.E - e0)) * p.N;
  const int64_t last = int64_t(steps - 1) * EN;
  if (roll.action) copy_words(roll.action + last + first, p.action + first, count);
  if (roll.reward) copy_words(roll.reward + last + first, p.reward + first, count);
  if (roll.obs) copy_words(roll.obs + (last + first) * p.D, p.obs + first * p.D, count * p.D);
}

// ----------------------------------------------------------------------------------
// Small envs of a small batch: one wave per env, one lane per agent, everything in registers.
// Such a batch is bound by the latency of one workgroup's chain of phases, not by any pipe (the
// regime in which the paper's own throughput grows linearly with the number of envs, Sec. 5.3), and
// the general kernel's chain (tables in LDS, a dozen workgroup barriers) is long for an env that
// fits a wave.  Here a lane reads any other agent's position with a lane read: the tag check is
// a loop over the taggers (a runner keeps the smallest (distance, tagger) key in range, credits
// are counted by votes), the K nearest a loop over the agents in play with the same sorted
// insertion as elsewhere; rows go to memory straight from registers.  Several iterations per launch
// (wd_rollout) keep the whole state in registers in between.  Same results as env_kernel.
// ----------------------------------------------------------------------------------
struct WaveArgs {
  Params p;
  Roll roll;           // a single call: steps = 1, ring_len = 1, no slices but roll.done = p.done_log
  const float* probs;  // the ring's base, or the one array of a single call
  uint64_t g0;
  int32_t mode;
};

template <int KC>
__global__ __launch_bounds__(kWaveSize) void wave_env_kernel(const WaveArgs args) {
  const Params& p = args.p;
  const Roll& roll = args.roll;
  constexpr int KT = register_list_size(KC);  // KC > 0: K compiled in; 0: K <= 8 at run time; -2: K <= 16
  const int a = threadIdx.x, e = blockIdx.x;
  const int N = p.N, N_tag = p.N_tag, G = p.G;
  const int K = KC > 0 ? KC : p.K;
  const int64_t D = 5 + 4 * K;
  const bool active = a < N;
  const int64_t EN = int64_t(p.E) * N, ai = int64_t(e) * N + (active ? a : 0);
  const int mode = args.mode;
  const bool stepping = mode == kModeStep || mode == kModeIterate;
  int x = 0, y = 0;
  bool lv = false;
  int done = 0, t = 0, nlr = 0, tags_out = -1;  // (tags_out < 0: tags_step keeps its value)
  if (mode != kModeResetAll) {
    if (active) {
      x = min(max(p.pos_x[ai], 0), G - 1);
      y = min(max(p.pos_y[ai], 0), G - 1);
      lv = p.live[ai] != 0;
    }
    done = p.done[e];
    t = p.t[e];
    nlr = p.n_live_runners[e];
  }
  // (the first four probabilities decide a draw, the fifth action is the fall-through; those of the
  // next iteration are requested while this one runs)
  const auto load_probs = [&](int s, float (&f)[4]) {
    const float* pr = args.probs + int64_t((roll.ring_pos + s) % roll.ring_len) * EN * kNumActions + ai * kNumActions;
#pragma unroll
    for (int c = 0; c < 4; ++c) f[c] = active ? pr[c] : 0.0f;
  };
  float f_next[4] = {0.0f, 0.0f, 0.0f, 0.0f};
  if (mode == kModeIterate) load_probs(0, f_next);
  for (int s = 0; s < roll.steps; ++s) {
    const bool last = s + 1 == roll.steps;
    const uint64_t g = args.g0 + uint64_t(s);
    int act = 0;
    if (mode == kModeIterate) {
      const float f[4] = {f_next[0], f_next[1], f_next[2], f_next[3]};
      if (!last) load_probs(s + 1, f_next);
      const Block4 r = random_block(p, uint32_t(e), uint32_t(a >> 2), uint32_t(g), uint32_t(g >> 32), kStreamAction);
      const uint32_t w = (a & 2) ? ((a & 1) ? r.w[3] : r.w[2]) : ((a & 1) ? r.w[1] : r.w[0]);
      act = sample_action(f[0], f[1], f[2], f[3], w);
      if (active) {
        if (last) p.action[ai] = act;
        if (roll.action) roll.action[int64_t(s) * EN + ai] = act;
      }
    } else if (stepping && active) {
      act = p.action[ai];
    }
    bool out_act = false;
    if (stepping && !done) {
      if (active && lv) {
        x = min(max(x + (act == 4) - (act == 3), 0), G - 1);
        y = min(max(y + (act == 1) - (act == 2), 0), G - 1);
      }
      uint32_t best = ~0u;
      if (p.tag_r2 >= 0)
        for (int tg = 0; tg < N_tag; ++tg) {
          const int dx = __builtin_amdgcn_readlane(x, tg) - x, dy = __builtin_amdgcn_readlane(y, tg) - y;
          const uint32_t d2 = uint32_t(__mul24(dx, dx)) + uint32_t(__mul24(dy, dy));
          if (d2 <= uint32_t(p.tag_r2)) best = min(best, (d2 << 6) | uint32_t(tg));
        }
      const bool tagged = active && a >= N_tag && lv && best != ~0u;
      const int tags = __popcll(__ballot(tagged));
      int credit = 0;
      if (tags)
        for (int tg = 0; tg < N_tag; ++tg) {
          const int c = __popcll(__ballot(tagged && int(best & 63u) == tg));
          if (a == tg) credit = c;
        }
      if (tagged) lv = false;
      if (active) {
        const float rew = a < N_tag ? static_cast<float>(credit) * p.tag_reward : (tagged ? p.tag_penalty : 0.0f);
        if (last) p.reward[ai] = rew;
        if (roll.reward) roll.reward[int64_t(s) * EN + ai] = rew;
      }
      nlr -= tags;
      t += 1;
      done = (nlr == 0 || t >= p.T) ? 1 : 0;
      tags_out = tags;
      out_act = true;
    }
    if (mode != kModeStep) {
      if (roll.done && a == 0) roll.done[int64_t(s) * p.E + e] = done;  // the flag before the reset clears it
      if (mode == kModeResetAll || done) {
        if (active) {
          x = min(max(p.pos_x0[ai], 0), G - 1);
          y = min(max(p.pos_y0[ai], 0), G - 1);
        }
        lv = active;
        t = 0;
        nlr = N - N_tag;
        done = 0;
        tags_out = 0;
        out_act = true;
      }
    }
    if (!out_act) continue;  // this env keeps its rows
    // ---- observations: the K nearest agents in play, by (squared distance, index) ----
    const uint64_t in_play = __ballot(active && lv);
    uint32_t keys[KT];
#pragma unroll
    for (int kk = 0; kk < KT; ++kk) keys[kk] = ~0u;
    if (K > 0)
      for (uint64_t left = in_play; left != 0; left &= left - 1) {  // the agents in play, in index order
        const int j = __builtin_ctzll(left);
        const int dx = __builtin_amdgcn_readlane(x, j) - x, dy = __builtin_amdgcn_readlane(y, j) - y;
        const uint32_t key = ((uint32_t(__mul24(dx, dx)) + uint32_t(__mul24(dy, dy))) << 6) | uint32_t(j);
        insert_key<KT>(keys, j == a ? ~0u : key);
      }
    float* const rows[2] = {last ? p.obs + ai * D : nullptr, roll.obs ? roll.obs + (int64_t(s) * EN + ai) * D : nullptr};
    const float t_frac = static_cast<float>(t) * p.inv_T;
    const float own[5] = {static_cast<float>(x) * p.inv_G, static_cast<float>(y) * p.inv_G, a < N_tag ? 1.0f : 0.0f,
                          lv ? 1.0f : 0.0f, t_frac};
    // (a row starts on a 4-byte boundary: its floats leave four at a time, at that alignment)
#pragma unroll
    for (int r = 0; r < 2; ++r)
      if (active && rows[r]) {
        *reinterpret_cast<Slot4*>(rows[r]) = Slot4{own[0], own[1], own[2], own[3]};
        rows[r][4] = own[4];
      }
#pragma unroll
    for (int kk = 0; kk < KT; ++kk) {
      if (kk < K) {
        // no branch: an empty slot looks up the agent itself, whose offsets are zero
        const bool none = !lv || keys[kk] == ~0u;
        const int j = none ? a : int(keys[kk] & 63u);
        const int ox = __shfl(x, j), oy = __shfl(y, j);
        const float slot[4] = {static_cast<float>(ox - x) * p.inv_G, static_cast<float>(oy - y) * p.inv_G,
                               (!none && j < N_tag) ? 1.0f : 0.0f, none ? 0.0f : 1.0f};
#pragma unroll
        for (int r = 0; r < 2; ++r)
          if (active && rows[r]) *reinterpret_cast<Slot4*>(rows[r] + 5 + 4 * kk) = Slot4{slot[0], slot[1], slot[2], slot[3]};
      }
    }
  }
  // the state, once per launch (an env that was neither stepped nor reset gets its own values back)
  if (active) {
    p.pos_x[ai] = x;
    p.pos_y[ai] = y;
    p.live[ai] = lv ? 1 : 0;
  }
  if (a == 0) {
    p.t[e] = t;
    p.n_live_runners[e] = nlr;
    p.done[e] = done;
    if (tags_out >= 0) p.tags_step[e] = tags_out;
  }
}

hipError_t launch_wave_kernel(const Params& p, int mode, const Roll& roll, const float* probs, uint64_t g,
                              hipStream_t stream) {
  WaveArgs args;
  args.p = p;
  args.roll = roll;
  args.probs = probs;
  args.g0 = g;
  args.mode = mode;
  if (p.K == 4)
    hipLaunchKernelGGL(wave_env_kernel<4>, dim3(p.E), dim3(kWaveSize), 0, stream, args);
  else if (p.K <= kMaxRegisterK)
    hipLaunchKernelGGL(wave_env_kernel<0>, dim3(p.E), dim3(kWaveSize), 0, stream, args);
  else
    hipLaunchKernelGGL(wave_env_kernel<-2>, dim3(p.E), dim3(kWaveSize), 0, stream, args);
  return hipGetLastError();
}

// The limit on a kernel's dynamic LDS is a property of the kernel function on a device, not of a
// handle: it is raised whenever a launch needs more than any launch before it on that device.
constexpr int kMaxDevicesTracked = 64;
template <typename Kernel>
hipError_t ensure_dynamic_lds(Kernel kernel, int bytes) {
  static int granted[kMaxDevicesTracked];  // per kernel function (one instance of this template each)
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return hipGetLastError();
  if (dev < 0 || dev >= kMaxDevicesTracked || bytes > granted[dev]) {
    const hipError_t err =
        hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (err != hipSuccess) return err;
    if (dev >= 0 && dev < kMaxDevicesTracked) granted[dev] = bytes;
  }
  return hipSuccess;
}

// (one team per workgroup gets the variant whose team-dependent values are uniform, where one is compiled)
template <int WIDE, int KX, bool BIG>
constexpr bool kHasOneTeamVariant = WIDE == 0 && !BIG && KX > 0;

template <int WIDE, int KX, bool CN, bool BIG, bool ONE = false>
hipError_t launch_env_variant(const Params& p, int mode, const float* probs, uint64_t g, hipStream_t stream,
                              const ObsPipe* pipe) {
  if constexpr (!ONE && kHasOneTeamVariant<WIDE, KX, BIG>) {
    if (p.teams_per_wg == 1) return launch_env_variant<WIDE, KX, CN, BIG, true>(p, mode, probs, g, stream, pipe);
  }
  if constexpr (BIG) {
    if (p.big_spread) {  // both kernels on the caller's stream: the next call's first kernel needs what the second leaves
      hipError_t err = ensure_dynamic_lds(&spread_obs_kernel<WIDE, KX>, p.lds_bytes);
      if (err != hipSuccess) return err;
      hipLaunchKernelGGL(spread_move_kernel, dim3(p.E * p.spread_slices), dim3(2 * kSpreadMoveThreads), 0, stream, p, mode,
                         probs, uint32_t(g), uint32_t(g >> 32));
      err = hipGetLastError();
      if (err != hipSuccess) return err;
      hipLaunchKernelGGL((spread_obs_kernel<WIDE, KX>), dim3(p.E * p.big_slices), dim3(kSpreadObsThreads),
                         size_t(p.lds_bytes), stream, p, mode);
      return hipGetLastError();
    }
  }
  const int groups = (p.E + p.teams_per_wg - 1) / p.teams_per_wg;
  hipError_t lds_err = ensure_dynamic_lds(&env_kernel<WIDE, KX, CN, BIG, ONE>, p.lds_bytes);
  if (lds_err != hipSuccess) return lds_err;
  hipLaunchKernelGGL((env_kernel<WIDE, KX, CN, BIG, ONE>), dim3(groups), dim3(p.wg_size), size_t(p.lds_bytes), stream, p,
                     mode, probs, uint32_t(g), uint32_t(g >> 32));
  hipError_t err = hipGetLastError();
  if constexpr (BIG) {
    if (err != hipSuccess) return err;
    // stream order puts the observation kernel behind the tables it reads; with a pipe it runs on
    // the pipe's stream behind an event, so that the caller's stream can go on with the next step
    err = ensure_dynamic_lds(&big_obs_kernel<WIDE, KX>, p.y_base);
    if (err != hipSuccess) return err;
    hipStream_t obs_stream = stream;
    if (pipe) {
      err = hipEventRecord(pipe->tables_ready, stream);
      if (err == hipSuccess) err = hipStreamWaitEvent(pipe->stream, pipe->tables_ready, 0);
      if (err != hipSuccess) return err;
      obs_stream = pipe->stream;
    }
    hipLaunchKernelGGL((big_obs_kernel<WIDE, KX>), dim3(p.E * p.big_slices), dim3(kBigObsWorkgroupSize),
                       size_t(p.y_base), obs_stream, p);
    err = hipGetLastError();
    if (pipe && err == hipSuccess) err = hipEventRecord(pipe->rows_done, pipe->stream);
  }
  return err;
}

template <int WIDE, int KX, bool CN, bool ONE = false>
hipError_t launch_rollout_variant(const Params& p, const Roll& roll, const float* ring, uint64_t g, hipStream_t stream) {
  if constexpr (!ONE && kHasOneTeamVariant<WIDE, KX, false>) {
    if (p.teams_per_wg == 1) return launch_rollout_variant<WIDE, KX, CN, true>(p, roll, ring, g, stream);
  }
  const hipError_t err = ensure_dynamic_lds(&rollout_kernel<WIDE, KX, CN, ONE>, p.lds_bytes);
  if (err != hipSuccess) return err;
  const int groups = (p.E + p.teams_per_wg - 1) / p.teams_per_wg;
  RollArgs args;
  args.p = p;
  args.roll = roll;
  args.ring = ring;
  args.g0 = g;
  hipLaunchKernelGGL((rollout_kernel<WIDE, KX, CN, ONE>), dim3(groups), dim3(p.wg_size), size_t(p.lds_bytes), stream, args);
  return hipGetLastError();
}

// Which compiled variant serves K: 1..8 (K compiled in; 4 is the benchmark shape, the only one that every key
// width and layout has), 0 (K <= 8 at run time), -2 (K <= 16), -1 (any K).
int variant_of(const Params& p) {
  if (p.obs_mode == 1) return -1;
  if (p.K == 4) return 4;
  if (p.K >= 1 && p.K <= kMaxRegisterK && !p.wide && !p.big) return p.K;  // 32-bit keys in the small layout
  if (p.K <= kMaxRegisterK) return 0;
  if (p.K <= kMaxRegisterK2) return -2;
  return -1;
}

}  // namespace

#define WD_DISPATCH(fn, ...)                                                               \
  do {                                                                                     \
    const int kx = variant_of(p);                                                          \
    if (p.big) {                                                                           \
      if (p.wide == 2) {                                                                   \
        if (kx == 4) return fn<2, 4, false, true>(p, ##__VA_ARGS__);                       \
        if (kx == -2) return fn<2, -2, false, true>(p, ##__VA_ARGS__);                     \
        return fn<2, 0, false, true>(p, ##__VA_ARGS__);                                    \
      }                                                                                    \
      if (!p.wide) {                                                                       \
        if (kx == 4) return fn<false, 4, false, true>(p, ##__VA_ARGS__);                   \
        if (kx == -2) return fn<false, -2, false, true>(p, ##__VA_ARGS__);                 \
        return fn<false, 0, false, true>(p, ##__VA_ARGS__);                                \
      }                                                                                    \
      if (kx == 4) return fn<true, 4, false, true>(p, ##__VA_ARGS__);                      \
      if (kx == -2) return fn<true, -2, false, true>(p, ##__VA_ARGS__);                    \
      return fn<true, 0, false, true>(p, ##__VA_ARGS__);                                   \
    }                                                                                      \
    if (!p.wide) {                                                                         \
      if (kx == 4 && p.compact_nbr) return fn<false, 4, true, false>(p, ##__VA_ARGS__);    \
      if (kx == 4) return fn<false, 4, false, false>(p, ##__VA_ARGS__);                    \
      if (kx == 8) return fn<false, 8, false, false>(p, ##__VA_ARGS__);                    \
      if (kx == 7) return fn<false, 7, false, false>(p, ##__VA_ARGS__);                    \
      if (kx == 6) return fn<false, 6, false, false>(p, ##__VA_ARGS__);                    \
      if (kx == 5) return fn<false, 5, false, false>(p, ##__VA_ARGS__);                    \
      if (kx == 3) return fn<false, 3, false, false>(p, ##__VA_ARGS__);                    \
      if (kx == 2) return fn<false, 2, false, false>(p, ##__VA_ARGS__);                    \
      if (kx == 1) return fn<false, 1, false, false>(p, ##__VA_ARGS__);                    \
      if (kx == 0) return fn<false, 0, false, false>(p, ##__VA_ARGS__);                    \
      if (kx == -2) return fn<false, -2, false, false>(p, ##__VA_ARGS__);                  \
      return fn<false, -1, false, false>(p, ##__VA_ARGS__);                                \
    }                                                                                      \
    if (kx == 4) return fn<true, 4, false, false>(p, ##__VA_ARGS__);                       \
    if (kx == 0) return fn<true, 0, false, false>(p, ##__VA_ARGS__);                       \
    if (kx == -2) return fn<true, -2, false, false>(p, ##__VA_ARGS__);                     \
    return fn<true, -1, false, false>(p, ##__VA_ARGS__);                                   \
  } while (0)

hipError_t launch_env_kernel(const Params& p, int mode, const float* probs, uint64_t g, hipStream_t stream,
                             const ObsPipe* pipe) {
  if (p.wave_envs) {
    Roll one;
    std::memset(&one, 0, sizeof(one));
    one.steps = 1;
    one.ring_len = 1;
    one.done = p.done_log;
    return launch_wave_kernel(p, mode, one, probs, g, stream);
  }
  WD_DISPATCH(launch_env_variant, mode, probs, g, stream, pipe);
}

bool rollout_available(const Params& p) { return p.wave_envs || (!p.big && p.obs_mode == 0 && p.K <= kMaxRegisterK); }

hipError_t launch_rollout(const Params& p, const Roll& roll, const float* ring, uint64_t g, hipStream_t stream) {
  if (p.wave_envs) return launch_wave_kernel(p, kModeIterate, roll, ring, g, stream);
  const int kx = variant_of(p);
  if (!p.wide) {
    if (kx == 4 && p.compact_nbr) return launch_rollout_variant<false, 4, true>(p, roll, ring, g, stream);
    if (kx == 4) return launch_rollout_variant<false, 4, false>(p, roll, ring, g, stream);
    if (kx == 8) return launch_rollout_variant<false, 8, false>(p, roll, ring, g, stream);
    if (kx == 7) return launch_rollout_variant<false, 7, false>(p, roll, ring, g, stream);
    if (kx == 6) return launch_rollout_variant<false, 6, false>(p, roll, ring, g, stream);
    if (kx == 5) return launch_rollout_variant<false, 5, false>(p, roll, ring, g, stream);
    if (kx == 3) return launch_rollout_variant<false, 3, false>(p, roll, ring, g, stream);
    if (kx == 2) return launch_rollout_variant<false, 2, false>(p, roll, ring, g, stream);
    if (kx == 1) return launch_rollout_variant<false, 1, false>(p, roll, ring, g, stream);
    return launch_rollout_variant<false, 0, false>(p, roll, ring, g, stream);
  }
  if (kx == 4) return launch_rollout_variant<true, 4, false>(p, roll, ring, g, stream);
  return launch_rollout_variant<true, 0, false>(p, roll, ring, g, stream);
}

bool env_kernel_available(const Params& p) { return !(p.big && (p.obs_mode == 1 || p.K > kMaxRegisterK2)); }

hipError_t launch_sample(const Params& p, const float* probs, uint64_t g, hipStream_t stream) {
  const int64_t total = int64_t(p.E) * p.NG;
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
