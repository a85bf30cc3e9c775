/*
 * wdc.h — C ABI of libwd for the CONTINUOUS Tag roll-out path on one MI355X.
 *
 * The second Tag variant of arXiv 2108.13976 (Sec. 5.1, the paragraph on the continuous
 * variant: agents move in a continuous 2-D world, pick among discrete accelerate / brake /
 * turn actions, follow classical mechanics, and a higher skill means a higher top speed;
 * Sec. 5.3 quotes its throughput at 2000 envs x 5 agents), run by the same three
 * services as the discrete variant of wd.h: sampler, step, reset of done envs (Sec. 4.4;
 * Sec. 4.5 items 3-6), in place on one device-resident struct-of-arrays store (Sec. 4.2).
 * The paper gives no state layout, action set, integration rule or constant for this
 * variant; what this library computes is stated here, function by function, and is this
 * build's own reading.
 *
 * Conventions are those of wd.h: every function returns WD_OK (0) or a negative
 * wd_status and never throws; pointers inside wdc_buffers and the `probs` arguments are
 * DEVICE pointers owned by the caller, borrowed until wdc_destroy, 256-byte aligned
 * (probs: 8-byte aligned), with at least the element counts that wdc_query_layout
 * reports; all other pointers are HOST pointers; kernels are enqueued on
 * wdc_config.stream without synchronising; calls on one handle come from one host thread
 * at a time.  wdc_create allocates 8 * num_headings bytes of device memory for the
 * heading table and wdc_destroy frees them; nothing else is allocated.
 *
 * State per agent: position x, y in [0, L] (float32), speed v >= 0 (float32), heading
 * index h in [0, H) (direction 360 h / H degrees), live flag.  Agents 0..N_tag-1 are
 * taggers.  Arrays are row-major [E][N], action [E][N][2], obs [E][N][D], per-env [E].
 */
#ifndef WDC_H
#define WDC_H

#include <stdint.h>

#include "wd.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Configuration of a batch of continuous-Tag envs (this build's own reading of Sec. 5.1). */
typedef struct wdc_config {
  uint32_t struct_size;    /* sizeof(wdc_config)                                      */
  int32_t num_envs;        /* E >= 1                                                  */
  int32_t env_offset;      /* global id of local env 0 (random blocks use global ids) */
  int32_t num_agents;      /* 2 <= N <= 1024                                          */
  int32_t num_taggers;     /* 1 <= N_tag <= N - 1                                     */
  int32_t num_headings;    /* H: a multiple of 4, 4 <= H <= 4096                      */
  int32_t episode_length;  /* T >= 1                                                  */
  int32_t obs_k;           /* K nearest agents observed, 0 <= K <= min(8, N - 1)      */
  float world_size;        /* L > 0                                                   */
  float accel;             /* speed change of one acceleration step                   */
  float max_speed_tagger;  /* top speed by kind: the skill level                      */
  float max_speed_runner;
  float tag_r2;            /* tagged iff squared distance <= tag_r2; < 0: no tagging  */
  float tag_reward;        /* per tag, to the credited tagger                         */
  float tag_penalty;       /* to the runner on the step it is tagged                  */
  uint64_t seed;
  void* stream;            /* hipStream_t, borrowed; NULL = default stream            */
} wdc_config;

/* Device buffers, caller-owned (the in-place data store of Sec. 4.2). */
typedef struct wdc_buffers {
  float *x, *y, *v;        /* [E][N]                                                  */
  int32_t* h;              /* [E][N]                                                  */
  float *x0, *y0;          /* [E][N] start state, written by wdc_reset(ALL)           */
  int32_t* h0;             /* [E][N]                                                  */
  int32_t* live;           /* [E][N]                                                  */
  int32_t* action;         /* [E][N][2]: acceleration level, turn level, each 0..4    */
  float* reward;           /* [E][N]                                                  */
  float* obs;              /* [E][N][D], D = 8 + 6 K                                  */
  int32_t *t, *done, *n_live_runners, *tags_step; /* [E]                              */
} wdc_buffers;

typedef struct wdc_layout {
  int32_t obs_dim;             /* D = 8 + 6 K                                         */
  int64_t agent_elems;         /* E * N                                               */
  int64_t action_elems;        /* 2 * E * N                                           */
  int64_t obs_elems;           /* E * N * D                                           */
  int64_t env_elems;           /* E                                                   */
  int64_t probs_elems;         /* 10 * E * N: [E][N][2][5]                            */
  int64_t bytes_per_iteration; /* algorithmic bytes of one sample + step + reset pass */
} wdc_layout;

typedef struct wdc_handle wdc_handle;

/* Sizes for a configuration (this build's own; no passage).  WD_E_CONFIG if a field is out
 * of range. */
int wdc_query_layout(const wdc_config* cfg, wdc_layout* out);

/* Creates a handle on the current device (this build's own; no passage).  Copies cfg and the
 * buffer pointers, builds the heading table (first octant: cos / sin of 360 h / H degrees
 * in double precision rounded to float32; the other entries by the symmetries of the
 * square, so the four axis directions are exact) and uploads it.  WD_E_NULL, WD_E_CONFIG,
 * WD_E_ALIGN, WD_E_HIP. */
int wdc_create(const wdc_config* cfg, const wdc_buffers* bufs, wdc_handle** out);

/* Reset (Sec. 4.5 items 1 and 5: the arrays of the first reset are kept and re-applied).
 * WD_RESET_ALL: start state of every agent from the random block of (seed, global env,
 * agent, g = 0, stream 3): x0 = u(w0) L, y0 = u(w1) L, u(w) = (w >> 8) 2^-24,
 * h0 = mulhi(w2, H); then every env is put in it: x, y, h <- x0, y0, h0; v <- 0; live <- 1;
 * t <- 0; n_live_runners <- N - N_tag; tags_step <- 0; done <- 0; obs <- rows of that state;
 * the step counter g <- 0.  WD_RESET_DONE: the same restore for envs with done == 1 only
 * (start state not redrawn); reward and action are left as they are.
 * WD_E_STATE for DONE before the first ALL. */
int wdc_reset(wdc_handle* h, int mode);

/* Sampler (Sec. 4.5 item 6).  probs is [E][N][2][5] float32: per agent the probabilities
 * of the five acceleration levels, then of the five turn levels.  action[e][i][c] <- inverse
 * CDF draw (float32 running sum left to right, strict u < c, last level as fall-through)
 * with u from word c of the random block of (seed, global env, agent, g, stream 2).
 * Every agent of every env draws. */
int wdc_sample(wdc_handle* h, const float* probs);

/* One step of every env with done == 0 (Sec. 4.5 items 3-4; rules: Sec. 5.1), then g <- g + 1.
 * Level l means the signed step s = l - 2.  A live agent: h <- (h + s_turn) mod H;
 * v <- v + float(s_acc) * accel, then 0 if negative, then its kind's top speed if above it;
 * x <- x + v * cx[h], y <- y + v * cy[h] (product rounded, then the sum); x, y clamped to
 * [0, L] and v <- 0 if either was clamped.  Then a live runner is tagged iff the smallest
 * d2 = dx * dx + dy * dy to a tagger is <= tag_r2; it leaves play; the tagger with the
 * smallest (d2, index) gets one credit.  reward = credits * tag_reward (taggers),
 * tag_penalty (runner tagged now), else 0; t <- t + 1; n_live_runners, tags_step;
 * done <- (n_live_runners == 0 || t >= T).  obs row of agent i:
 * [x/L, y/L, v, cx[h], cy[h], is_tagger, live, t/T] then K slots
 * [(xj - x)/L, (yj - y)/L, vj cx[hj], vj cy[hj], is_tagger_j, 1] of the nearest other live
 * agents by (d2, j), zeros when fewer and for an agent out of play.  An agent out of play
 * keeps its state.  All arithmetic is float32, each operation rounded on its own. */
int wdc_step(wdc_handle* h);

/* wdc_sample, wdc_step and wdc_reset(DONE) in one launch, same results (this build's own
 * fusion of Sec. 4.5 items 3-6). */
int wdc_iterate(wdc_handle* h, const float* probs);

/* Roll-out arrays of wdc_rollout: DEVICE pointers, 8-byte aligned, each optional (NULL = not
 * recorded): action [k][E][N][2], reward [k][E][N], done [k][E], obs [k][E][N][D]. */
typedef struct wdc_rollout_buffers {
  int32_t* action;
  float* reward;
  int32_t* done;
  float* obs;
} wdc_rollout_buffers;

/* k iterations (each = wdc_iterate) in ONE launch: the roll-out of Sec. 4.5 whose data a trainer
 * gathers into a batch (item 7), here without returning to the host between iterations.
 * probs_ring holds ring_len steps of probabilities [ring_len][E][N][2][5]; iteration s draws with
 * step g + s from entry (g + s) mod ring_len.  Slice s of each array of `out` that is not NULL
 * receives that iteration's actions, rewards, done flags (as they were before the reset of done
 * envs) and rows; `out` may be NULL.  The in-place arrays end as after k calls of wdc_iterate
 * (action, reward and obs hold the last iteration's values); g <- g + k.  Same results as k calls
 * of wdc_iterate.  WD_E_CONFIG for ring_len < 1 or k < 1. */
int wdc_rollout(wdc_handle* h, const float* probs_ring, int ring_len, int k, const wdc_rollout_buffers* out);

/* The global step g that the next draw will use (this build's own; no passage). */
int wdc_get_step(const wdc_handle* h, uint64_t* g);
int wdc_set_step(wdc_handle* h, uint64_t g);

/* Frees the handle and the heading table; NULL is allowed (this build's own). */
int wdc_destroy(wdc_handle* h);

/* Text of the last WD_E_HIP failure on this handle ("" if none). */
const char* wdc_last_error(const wdc_handle* h);

#ifdef __cplusplus
}
#endif
#endif /* WDC_H */
