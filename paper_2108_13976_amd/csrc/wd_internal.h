// wd_internal.h — shared between the host API (wd_api.hip) and the device code
// (wd_kernels.hip) of libwd.  Nothing here is part of the public ABI.
#ifndef WD_INTERNAL_H
#define WD_INTERNAL_H

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace wd {

constexpr int kWorkgroupSize = 256;     // flat per-agent kernels: four wave64s
constexpr int kMaxEnvWorkgroupSize = 1024; // env-per-team kernels run 256, 512 or 1024 threads (by agent count);
constexpr int kBigEnvWorkgroupSize = 1024; // 1024 in the step kernel of the large-env layout
constexpr int kBigObsWorkgroupSize = 512;  // observation kernel of the large-env layout
// Large envs of a small batch, step spread over many workgroups: the move kernel gives a lane a
// group of four agents, the table kernel runs 1024 threads per slice of an env
constexpr int kSpreadMoveThreads = 128;
constexpr int kSpreadMoveAgents = 4 * kSpreadMoveThreads;
constexpr int kSpreadObsThreads = 1024;
constexpr int kSpreadMaxTaggers = 2048;  // every workgroup of the move kernel moves all taggers of its env
constexpr int kSpreadTagSide = 64;       // its table of taggers: at most this many coarse cells per grid side
constexpr int kWaveSize = 64;
constexpr int kNumActions = 5;
constexpr int kMaxRegisterK = 8;        // K up to this keeps the candidate list in 8 registers,
constexpr int kMaxRegisterK2 = 16;      // up to this in 16 (a variant of its own)
// List size of a kernel variant KX (KX > 0: exactly K; 0: K <= 8; -2: K <= 16).
constexpr int register_list_size(int kx) { return kx > 0 ? kx : (kx == -2 ? kMaxRegisterK2 : kMaxRegisterK); }
// Window sizes of the strip search for K neighbours: entries on either side of the agent's slot in
// its own strip, and on either side of its column in the strip above and the strip below; for
// the agents that these do not settle, a second try with windows twice as wide and two more
// strips.  Simulated at the headline density (strips 1.5 expected K-th-neighbour distances tall): the first
// try settles 95 % of the agents, the second all but about one in ten thousand.
// (K = 1 takes the windows of K = 2: with its own, too many agents go on to the later tries)
constexpr int strip_window_k(int k) { return k < 2 ? 2 : k; }
constexpr int strip_half_own(int k) { return strip_window_k(k) + 3; }
constexpr int strip_half_adj(int k) { return strip_window_k(k) + 2; }
constexpr int strip_half_own2(int k) { return 2 * strip_window_k(k) + 6; }
constexpr int strip_half_adj2(int k) { return 2 * strip_window_k(k) + 4; }
constexpr int strip_half_far2(int k) { return 2 * strip_window_k(k); }
constexpr int strip_pad(int k) {
  const int a = strip_half_own(k) + 2 * strip_half_adj(k), b = 2 * strip_half_adj2(k), c = strip_half_own2(k);
  return a > b ? (a > c ? a : c) : (b > c ? b : c);
}
constexpr int kStripScanAll = 64;  // lists up to this length are scanned whole instead of through windows
constexpr int kStripQueue2 = 32;  // agents per env that may wait for the third, exact block search
constexpr uint32_t kStreamAction = 0;   // random streams (low byte of the fourth counter word)
constexpr uint32_t kStreamInit = 1;

// Exact unsigned division by a run-time constant (Granlund & Montgomery 1994):
// q = (t + ((a - t) >> sh1)) >> sh2 with t = mulhi(a, mul).
struct FastDiv {
  uint32_t mul, sh1, sh2, div;
};

inline FastDiv make_fastdiv(uint32_t d) {
  FastDiv f;
  f.div = d;
  uint32_t l = 0;
  while ((uint64_t(1) << l) < d) ++l;  // ceil(log2 d)
  f.mul = uint32_t(((uint64_t(1) << 32) * ((uint64_t(1) << l) - d)) / d + 1);
  f.sh1 = l < 1 ? l : 1;
  f.sh2 = l == 0 ? 0 : l - 1;
  return f;
}

// Everything a kernel needs: sizes, rule constants, launch geometry, LDS map, buffers.
struct Params {
  // sizes and rule constants
  int32_t E, N, N_tag, G, T, tag_r2, tag_rad, K, D, obs_mode;
  uint32_t env_offset, seed_lo, seed_hi;
  float tag_reward, tag_penalty, inv_G, inv_T;
  // Geometry of the env-per-team kernels.  Agents are handled in groups of four
  // consecutive indices (one 16-byte load per array, one random block per group).  A
  // workgroup holds teams_per_wg teams of (1 << ts_log2) threads; a team owns one env;
  // thread lt of a team owns groups lt, lt + ts, ... (gpt of them).
  int32_t NG;            // groups per env = ceil(N / 4)
  int32_t NPAD;          // 4 * NG rounded up to 8: per-agent LDS arrays are padded to this
  int32_t wg_size;       // 256; 512 or 1024 for one env of more than 1024 or 3072 agents
  int32_t stage_rows_log2;  // rows a wave transposes through LDS per flush: 32 or 16
  int32_t ts_log2, teams_per_wg, gpt;
  int32_t vec4;          // N % 4 == 0: a group's global slices are 16-byte aligned
  int32_t nb_cap;        // bucket slots per team (power of two, >= team size)
  int32_t scan_chunk;    // nb_cap / team size
  float bucket_scale;    // 65536 / G: bucket multiplier = scale * sqrt(n_live / lambda)
  float lambda_c, lambda_min, lambda_max;  // live agents per bucket aimed at: lambda_c / sqrt(n_live), clamped
  uint32_t bucket_mul_max;  // largest multiplier whose bucket table fits nb_cap
  // (distance, index) keys and bucket entries: 0 = 32-bit keys below 2^31, 1 = 64-bit, 2 = 32-bit
  // keys using all bits (dead mark in the index array)
  int32_t wide, idx_bits, xy_bits;
  int32_t dead_dx;       // 32-bit form: y offset that marks a runner tagged in this step
  FastDiv div_N, div_NG;
  // Strip-sorted list (32-bit keys, K = 1 .. 8 compiled in, small layout): strips of the grid times
  // columns of 2^cshift cells; the table of bin starts takes the place of the bucket tables.
  int32_t strips;        // 1: this configuration runs the strip variant of the env kernels
  int32_t cshift, strip_C;  // column of cell x = x >> cshift; columns per strip
  int32_t strip_rmax;    // most strips the table holds (and the grid has rows for)
  float strip_scale;     // strips aimed at = strip_scale * sqrt(live agents)
  int32_t pad_l, pad_r;  // entries in front of and behind the list that read as "no agent"
  int32_t pos_shift;     // positions in the list are scaled by 2^pos_shift per axis, so that the squared length
  int32_t key_shift;     // of a packed difference is the squared distance << key_shift (= 2 pos_shift >= idx_bits)
  uint32_t dead_key_min; // keys of list entries out of play start here, above every key of a live pair
  // LDS map.  Per team: a kept part (positions, scalars); an X part (bucket-sorted entries
  // and bucket starts) that the row staging area overlays once the neighbour search is done;
  // a Y part (slots, tag keys, credits, bucket counters) that the neighbour lists overlay
  // once the rewards are out.
  int32_t keep_stride, off_pl, off_misc, off_edges;
  int32_t x_base, x_stride, off_sorted, off_sorted_id, off_starts;
  int32_t y_base, y_stride, off_slot, off_best, off_credits, off_counts, off_nbr, off_retry;
  int32_t compact_nbr;   // K = 4 neighbour ids of an agent packed into 40 bits (N < 1024)
  int32_t lds_bytes;
  // Large envs (big != 0): one 1024-thread workgroup per env; slots, tag keys, credits and
  // neighbour lists live in library-owned device memory instead of LDS (per-env strides in
  // elements of each array's type).
  int32_t big;
  int32_t big_lds_tables;  // 1: slots, tag keys and credits of a large env are in LDS after all (they fit)
  uint16_t* g_slot;
  void* g_best;
  int32_t* g_credits;
  unsigned char* g_image;  // per env: the kept and sorted parts of LDS as the env kernel left them
  int64_t g_stride_agents, g_stride_credits, g_stride_image;
  int32_t big_slices;      // workgroups per env in the observation kernel
  // Spread form of the large-env pair (big_spread != 0): spread_move_kernel (sample, move, tag check
  // by slices of 512 agents) leaves packed positions, ranks inside the buckets and, in the
  // accumulators, bucket counts, credits and the number of tags; spread_obs_kernel finishes the step
  // and builds the tables per slice.  Two sets of accumulators take turns: the kernels of one call
  // use set `spread_parity`, and the second kernel clears the other set for the next call.
  int32_t big_spread;
  int32_t spread_slices;   // workgroups per env in spread_move_kernel
  int32_t spread_parity;
  uint32_t tag_mul;        // coarse cell of a tagger: (x * tag_mul) >> 16 per axis, tag_nbx cells per side
  int32_t tag_nbx;
  uint32_t* g_pl;          // [E][NPAD] packed positions after the move and the tag check
  int32_t* g_env;          // [E][4] done, t, n_live_runners as the call found them
  uint32_t* g_acc;         // [2][E][g_stride_acc]: credits per tagger, number of tags
  int64_t g_stride_acc;
  int32_t acc_credits, acc_tags;  // word offsets inside one env's accumulators
  int32_t wave_envs;     // 1: envs of at most 64 agents in a small batch run in wave_env_kernel, a wave per env
  // device buffers (borrowed from the caller)
  int32_t *pos_x, *pos_y, *pos_x0, *pos_y0, *live, *action;
  float* reward;
  float* obs;
  int32_t *t, *done, *n_live_runners, *tags_step;
  int32_t* done_log;     // optional [E]: done flags of an iteration before its reset (roll-outs)
  int32_t rows_kept;     // 1: the obs buffer this launch writes still holds the rows this library wrote for
                         // the state the step starts from (a row whose agent was already out of play then
                         // differs from it in the time feature only)
};

// A multi-step roll-out: iteration s reads ring entry (ring_pos + s) mod ring_len and writes
// slice s of the buffers that are not NULL (action, reward [steps][E][N]; done [steps][E];
// obs [steps][E][N][D]).
struct Roll {
  int32_t steps, ring_len, ring_pos, pad;
  int32_t* action;
  float* reward;
  int32_t* done;
  float* obs;
};

enum EnvKernelMode { kModeStep = 0, kModeResetAll = 1, kModeResetDone = 2, kModeIterate = 3 };

// Launchers (wd_kernels.hip).  Each enqueues on `stream` and returns the HIP status of the launch.
hipError_t launch_sample(const Params& p, const float* probs, uint64_t g, hipStream_t stream);
hipError_t launch_init_start_positions(const Params& p, hipStream_t stream);
// Large-env layout only: where the observation kernel of a call runs when it is not to hold up the
// caller's stream (roll-outs overlap it with the next iteration's step kernel).  The launcher
// records `tables_ready` on the caller's stream behind the step kernel, makes `stream` wait for
// it, launches the observation kernel there and records `rows_done` behind it.
struct ObsPipe {
  hipStream_t stream;
  hipEvent_t tables_ready, rows_done;
};
hipError_t launch_env_kernel(const Params& p, int mode, const float* probs, uint64_t g, hipStream_t stream,
                             const ObsPipe* pipe = nullptr);
hipError_t launch_rollout(const Params& p, const Roll& roll, const float* ring, uint64_t g, hipStream_t stream);
bool rollout_available(const Params& p);
// True if the env-per-team kernels cover this configuration.
bool env_kernel_available(const Params& p);

}  // namespace wd
#endif  // WD_INTERNAL_H
