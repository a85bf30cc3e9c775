/*
 * wd.h — C ABI of libwd: the batched discrete Tag roll-out path on one MI355X.
 *
 * The library runs the three device-side services of a WarpDrive-style roll-out
 * (arXiv 2108.13976, Sec. 4.4: the sampler and reset kernels of the service layer and
 * the step kernel of the environment layer; Sec. 4.5, items 2-6 of the workflow) for
 * the discrete Tag environment of Sec. 5.1, on ONE device-resident struct-of-arrays
 * data store that is updated in place (Sec. 4.2; the figure with the step signature:
 * float observations and rewards, int actions and done flags).
 *
 * Conventions
 *   - Every function returns WD_OK (0) or a negative wd_status; none throws or
 *     aborts.  On failure nothing has been enqueued unless stated otherwise.
 *   - All pointers inside wd_buffers and the `probs` arguments are DEVICE
 *     pointers (hipMalloc'd or PyTorch-allocated), owned by the caller and only
 *     borrowed until wd_destroy.  Each buffer must be 256-byte aligned (probs:
 *     16-byte aligned) and hold at least the element count that wd_query_layout
 *     reports.  All other pointers
 *     (config, layout, handle, out parameters) are HOST pointers.
 *   - Kernels are enqueued on wd_config.stream (a hipStream_t, borrowed; NULL =
 *     the default stream) and are NOT synchronised: the caller synchronises
 *     before reading results on the host.  Calls on one handle must be issued
 *     from one host thread at a time.
 *   - All state lives in the caller's buffers.  The library allocates no device
 *     memory, with one exception: for envs too large for a workgroup's LDS
 *     (thousands of agents) wd_create allocates per-env work tables once on the
 *     current device (about 20 bytes per agent) and wd_destroy frees them (and
 *     wd_rollout, on its first call for such a configuration, a second copy of part
 *     of them: see there).
 *   - The observations are part of that in-place state (one data store, modified
 *     in place: Sec. 4.2).  The row of an agent that was already out of play
 *     before a step differs from the row the previous call left in `obs` in its
 *     time feature only, and in some configurations (full observations, K > 16,
 *     the large-env layout: see wd_create) a step rewrites just that element; with
 *     partial observations and K <= 16 in the small layout (the five benchmark
 *     workloads but tag_10x8192) every row is always written whole.  What the
 *     library knows about `obs` is kept per handle, so a region of the buffers must
 *     be driven through ONE handle at a time, and a caller that overwrites `obs`
 *     or the state arrays between calls (a restored checkpoint, an agent taken out
 *     of play by hand, observations normalised in place, another handle or
 *     wd_iterate_static used on the same buffers) calls wd_invalidate_obs: the next
 *     call then writes every row whole.  Rows recorded through wd_rollout_buffers
 *     are always written whole.
 *   - The global step g reaches the kernels as a launch argument.  A HIP graph
 *     captured around calls of this library therefore replays the random numbers
 *     of the steps it was captured at; to run many iterations with one launch,
 *     use wd_rollout.
 *   - Random numbers are Philox4x32-10 blocks keyed by (seed, global env id,
 *     agent, global step g, stream), so results do not depend on launch shape,
 *     and a run over envs [a, b) with env_offset = a reproduces those envs of the
 *     full run.
 *
 * Array layouts (row-major): per-agent arrays are [E][N]; obs is [E][N][D];
 * per-env arrays are [E].  int32 and float32 throughout.
 */
#ifndef WD_H
#define WD_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum wd_status {
  WD_OK = 0,
  WD_E_NULL = -1,   /* a required pointer is NULL                                   */
  WD_E_CONFIG = -2, /* a config field is out of range or struct_size mismatches     */
  WD_E_ALIGN = -3,  /* a device buffer is not aligned as required                   */
  WD_E_STATE = -4,  /* call order: sample/step/reset(DONE) before the first reset(ALL) */
  WD_E_HIP = -5,    /* a HIP call failed; wd_last_error(handle) has the text        */
  WD_E_UNSUPPORTED = -6, /* valid config that this build has no kernel for          */
  WD_E_SCRATCH = -7 /* wd_iterate_static: the configuration's work tables exceed
                       WD_STATIC_SCRATCH_BYTES                                      */
} wd_status;

enum { WD_RESET_ALL = 0, WD_RESET_DONE = 1 };
enum { WD_OBS_PARTIAL = 0, WD_OBS_FULL = 1 };

/* Configuration of one batch of Tag environments (Sec. 5.1, Tag paragraph). */
typedef struct wd_config {
  uint32_t struct_size;   /* = sizeof(wd_config); ABI check                              */
  int32_t num_envs;       /* E >= 1 environments in the buffers                          */
  int32_t env_offset;     /* >= 0: global id of env 0 (shard of a larger run)            */
  int32_t num_agents;     /* N: 2 <= N <= 32768                                          */
  int32_t num_taggers;    /* N_tag: 1 <= N_tag <= N-1; agents 0..N_tag-1 are taggers     */
  int32_t grid_size;      /* G: square grid, 1 <= G <= 32767                             */
  int32_t num_actions;    /* must be 5: stay, up (y+1), down (y-1), left (x-1), right (x+1) */
  int32_t episode_length; /* T >= 1: an episode ends after T steps at the latest         */
  int32_t tag_r2;         /* a runner is tagged iff some tagger is at squared distance
                             <= tag_r2 after the moves; negative disables tagging        */
  int32_t obs_mode;       /* WD_OBS_PARTIAL (K nearest agents) or WD_OBS_FULL            */
  int32_t obs_k;          /* K: 0 <= K <= N-1 (ignored in full mode)                     */
  float tag_reward;       /* to the credited tagger, per tag (Sec. 5.1 gives +1 as example) */
  float tag_penalty;      /* to the runner on the step it is tagged (example there: -1)   */
  uint64_t seed;
  void* stream;           /* hipStream_t, borrowed                                       */
} wd_config;

/* The device-resident data store (Sec. 4.5 item 1: state arrays plus the
 * observation / action / reward / done placeholders; pos_x0, pos_y0 are the copies
 * of the start state that item 5 puts back at every reset). */
typedef struct wd_buffers {
  int32_t *pos_x, *pos_y;   /* [E][N] cell coordinates in [0, G)                         */
  int32_t *pos_x0, *pos_y0; /* [E][N] start positions, written by wd_reset(ALL)          */
  int32_t* live;            /* [E][N] 1 = in play, 0 = tagged runner                     */
  int32_t* action;          /* [E][N] written by wd_sample, read by wd_step              */
  float* reward;            /* [E][N] overwritten for every agent by each step           */
  float* obs;               /* [E][N][D] kept up to date in place (see Conventions)        */
  int32_t *t, *done, *n_live_runners, *tags_step; /* [E]                                 */
} wd_buffers;

/* Element counts the caller must allocate, and the algorithmic HBM bytes of one
 * roll-out iteration (sample + step + reset of done envs). */
typedef struct wd_layout {
  int32_t obs_dim;            /* D = 5 + 4K (partial) or 5 + 4N (full)                   */
  int64_t per_agent_elems;    /* E*N      : pos_*, live, action, reward                  */
  int64_t obs_elems;          /* E*N*D                                                   */
  int64_t per_env_elems;      /* E        : t, done, n_live_runners, tags_step           */
  int64_t probs_elems;        /* E*N*5    : the probs argument of wd_sample              */
  int64_t bytes_per_iteration;/* E*N*(4*5 + 36 + 4*D) + 24*E                             */
} wd_layout;

typedef struct wd_handle wd_handle;

/* Fills *out for a configuration.  Host only; touches no device.  (No passage of the
 * paper: this build's own; it takes the place of the data manager's placeholder
 * set-up of Sec. 4.4.) */
int wd_query_layout(const wd_config* cfg, wd_layout* out);

/* (No passage of the paper: this build's own; the paper's managers load kernels and
 * push data at this point, Sec. 4.4.)  Validates cfg and bufs (range, alignment),
 * chooses the launch geometry and returns a handle in *out.  Enqueues nothing; the buffers' contents are not read.
 * WD_E_UNSUPPORTED if no kernel of this build covers the configuration (an env whose
 * tables exceed one workgroup's LDS: beyond about 13 900 agents with 32-bit keys, 11 500
 * with 64-bit keys, 8192 for full observations or K > 16).  Envs too large for one
 * workgroup's LDS, and batches of few envs (at most 450, or 0.3 N up to 1024 agents) of
 * 384 agents or more, run in the large-env layout, whose work tables (about 20 bytes per
 * agent) the library allocates here with hipMalloc: WD_E_HIP if that fails. */
int wd_create(const wd_config* cfg, const wd_buffers* bufs, wd_handle** out);

/* Environment reset (Sec. 4.5 item 5, the automatic reset of done envs).
 * WD_RESET_ALL : draws pos_x0/pos_y0 uniformly on the grid from the seed, then puts
 *                every env in its start state; sets the global step g to 0.
 * WD_RESET_DONE: every env with done == 1 is put back in its start state in place
 *                (pos <- pos0, live <- 1, t <- 0, n_live_runners <- N - N_tag,
 *                tags_step <- 0, done <- 0, obs <- observation of that state;
 *                reward and action untouched); other envs are untouched. */
int wd_reset(wd_handle* h, int mode);

/* Action sampling (Sec. 4.5 item 6, one sampler thread per agent).
 * probs: device [E][N][5] float32 policy outputs.  Writes action[e][i] for EVERY
 * agent of EVERY env by inverse CDF (float32 running sum, left to right, strict
 * "u < sum", last action as fall-through) with u from word i mod 4 of the random
 * block of (seed, env_offset + e, i / 4, g, stream 0).  Does not advance g. */
int wd_sample(wd_handle* h, const float* probs);

/* One Tag step (Sec. 5.1; Sec. 4.5 items 3-4) for every env with done == 0, in
 * place: move, tag check, rewards, t / n_live_runners / tags_step / done,
 * observations.  Envs with done == 1 are left untouched.  Consumes
 * buffers.action; then advances the global step g by one. */
int wd_step(wd_handle* h);

/* One whole roll-out iteration in a single launch: wd_sample(probs), wd_step,
 * wd_reset(WD_RESET_DONE), with identical results (Sec. 4.5 items 3-6 fused; the fusion
 * itself is this build's own). */
int wd_iterate(wd_handle* h, const float* probs);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): wd_iterate without a handle and without
 * any allocation, on the host or on the device.  One whole roll-out iteration (sample,
 * step, reset of done envs) at global step g on the state in `bufs`, which must be a state
 * that this library left there (wd_reset / wd_step / wd_iterate / wd_rollout on a handle of
 * the same configuration, or earlier calls of this function).  Same arguments otherwise:
 * cfg (host), bufs (DEVICE pointers, 256-byte aligned), probs (device [E][N][5]); the
 * kernels are enqueued on cfg->stream and not synchronised; results equal wd_iterate's.
 * Every observation row is written whole.  The work tables that a large-env configuration
 * needs (see wd_create) live in a static device array of WD_STATIC_SCRATCH_BYTES that every
 * call on a GPU shares (each GPU the library runs on holds it until the process ends):
 * WD_E_SCRATCH if the configuration needs more; calls that overlap in time on one GPU, on
 * any streams, race on that array and must be serialised by the caller.  Calls no
 * hipMalloc / hipFree. */
#define WD_STATIC_SCRATCH_BYTES (8u << 20)
int wd_iterate_static(const wd_config* cfg, const wd_buffers* bufs, const float* probs, uint64_t g);

/* Per-iteration outputs of a multi-step roll-out (the experience a trainer batches,
 * Sec. 4.5 item 7): DEVICE pointers, caller-owned, 16-byte aligned, each may be NULL.
 * Slice s (0 <= s < k) holds what iteration s produced. */
typedef struct wd_rollout_buffers {
  int32_t* action; /* [k][E][N]    actions sampled in iteration s                          */
  float* reward;   /* [k][E][N]    rewards of the step of iteration s                      */
  int32_t* done;   /* [k][E]       done flags after the step, before the reset clears them  */
  float* obs;      /* [k][E][N][D] observations after iteration s (after the reset of done envs) */
} wd_rollout_buffers;

/* k whole roll-out iterations in ONE launch (launch latency paid once; Sec. 4.5 items
 * 3-6 repeated).  probs_ring: device [ring_len][E][N][5]; iteration s samples from entry
 * (g + s) mod ring_len.  Results equal k calls of wd_iterate with those probabilities:
 * the in-place buffers end in the state after the last iteration, `out` (may be NULL)
 * receives every iteration's outputs, g advances by k.  Configurations that use the
 * large-env layout, full observations or K > 8 have no multi-step kernel: for them the
 * call enqueues one launch per iteration (and device-to-device copies of the last slice),
 * with the same results.  In the large-env layout the observation kernel of an iteration
 * then runs on a second stream that the handle owns (default priority), beside the step
 * kernel of the next iteration, ordered by events; cfg.stream waits for the last of them
 * before the call's work on it ends, so the caller sees one stream as before.  The first
 * such call creates that stream, four events and a second copy of the env tables (device
 * memory, about 11 bytes per agent); wd_destroy releases them.
 * On WD_E_HIP part of the iterations may have been enqueued. */
int wd_rollout(wd_handle* h, const float* probs_ring, int ring_len, int k, const wd_rollout_buffers* out);

/* The global step counter g used as the RNG step index (checkpoint / resume; no passage
 * of the paper: this build's own).  wd_set_step also does what wd_invalidate_obs does: a
 * resumed run may have restored the state arrays without the observations. */
int wd_get_step(wd_handle* h, uint64_t* g);
int wd_set_step(wd_handle* h, uint64_t g);

/* Tells the library that `obs` (or the state arrays) were changed by someone else since
 * the last call on this handle (see Conventions): the next step, iteration or roll-out
 * writes every observation row whole.  Host only.  (No passage of the paper: this build's
 * own, a consequence of keeping the observations in the in-place store of Sec. 4.2.) */
int wd_invalidate_obs(wd_handle* h);

/* Frees the handle and, for large-env configurations, its work tables (the caller
 * must have synchronised the stream first in that case).  The caller's buffers are
 * not touched.  (No passage of the paper: this build's own.) */
int wd_destroy(wd_handle* h);

/* Static text for a status code.  (This build's own, like wd_last_error.) */
const char* wd_strerror(int status);

/* Text of the last HIP failure seen on this handle ("" if none).  The pointer is
 * valid until the next call on the handle. */
const char* wd_last_error(wd_handle* h);

#ifdef __cplusplus
}
#endif
#endif /* WD_H */
