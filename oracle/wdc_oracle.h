/*
 * wdc_oracle.h — CPU oracle for the batched CONTINUOUS Tag roll-out path.
 *
 * TEST INFRASTRUCTURE ONLY.  The plain, slow, single-threaded definition of what
 * the GPU library's wdc_* entry points compute.  It shares no code, header, table
 * or constant generator with the HIP path, and nothing in the product path may
 * include, link or call it.  It uses the discrete oracle's pinned building blocks
 * (wdo_random_block, wdo_uniform_from_word, wdo_sample_from_u of wd_oracle.h).
 *
 * What it follows (WarpDrive paper, arXiv 2108.13976, Sec. 5.1, the paragraph on
 * the continuous variant of Tag, and Sec. 4.5 items 5 and 6 for reset and
 * sampling): agents move in a continuous 2-D world; each picks among discrete
 * accelerate / brake / turn actions; motion follows classical mechanics; a higher
 * skill means a higher top speed; tagging, rewards and the end of an episode are
 * those of the discrete variant.  The paper gives no state layout, no action
 * set, no integration rule and no constant: every such choice is a reading of this
 * build, C1..C14, listed in wdc_oracle.cpp next to the code that implements it.
 * "Parity unpinned against the paper" for all of them; they are pinned to hand
 * traces with exactly representable numbers, closed forms, the symmetries of the
 * heading table, an independent Python statement and invariants.
 *
 * Precision (C13): the state is float32 and every update is the stated sequence of
 * IEEE float32 operations (compiled without contraction), because comparisons on
 * these values decide clamps, tags and the order of neighbours.
 *
 * All arrays are HOST memory owned by the caller; nothing is retained between
 * calls.  Every function returns 0 on success and a negative value on a bad
 * argument.
 */
#ifndef WDC_ORACLE_H
#define WDC_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct wdco_config {
  int32_t num_envs;        /* E                                                       */
  int32_t env_offset;      /* global id of local env 0 (RNG is keyed by global id)   */
  int32_t num_agents;      /* N                                                       */
  int32_t num_taggers;     /* N_tag; agents 0..N_tag-1 are taggers                    */
  int32_t num_headings;    /* H, a multiple of 4                                      */
  int32_t episode_length;  /* T                                                       */
  int32_t obs_k;           /* K nearest agents observed                               */
  float world_size;        /* L: the world is [0, L] x [0, L]                         */
  float accel;             /* speed change per acceleration step                      */
  float max_speed_tagger;  /* top speed of taggers                                    */
  float max_speed_runner;  /* top speed of runners                                    */
  float tag_r2;            /* tagged iff squared distance <= tag_r2; < 0 disables     */
  float tag_reward;        /* per successful tag, to the credited tagger              */
  float tag_penalty;       /* to the runner on the step it is tagged                  */
  uint64_t seed;
} wdco_config;

typedef struct wdco_state {
  float *x, *y, *v;         /* [E][N] position and speed                              */
  int32_t *h;               /* [E][N] heading index in [0, H)                         */
  float *x0, *y0;           /* [E][N] start positions re-applied at reset             */
  int32_t *h0;              /* [E][N] start headings                                  */
  int32_t *live;            /* [E][N] 1 = in play                                     */
  int32_t *action;          /* [E][N][2] acceleration level, turn level (0..4)        */
  float *reward;            /* [E][N]                                                 */
  float *obs;               /* [E][N][D], D = 8 + 6 K                                 */
  int32_t *t, *done, *n_live_runners, *tags_step; /* [E]                              */
} wdco_state;

enum { WDCO_RESET_ALL = 0, WDCO_RESET_DONE = 1 };

/* D = 8 + 6 K. */
int32_t wdco_obs_dim(const wdco_config* cfg);

/* The heading table of C5: cx[h], cy[h] for h in [0, H).  H must be a positive multiple of 4. */
int wdco_heading_table(int32_t num_headings, float* cx, float* cy);

/* mode ALL: draw the start state from the seed, then put every env in it.
 * mode DONE: put only envs with done == 1 back in their start state. */
int wdco_reset(const wdco_config* cfg, const wdco_state* st, int mode);

/* action[e][i][c] <- categorical draw from probs[e][i][c][0..4] with word c of the random
 * block of (seed, env_offset + e, i, g, stream 2); every agent of every env. */
int wdco_sample(const wdco_config* cfg, const wdco_state* st, const float* probs, uint64_t g);

/* One step for every env with done == 0 (envs with done == 1 are untouched). */
int wdco_step(const wdco_config* cfg, const wdco_state* st);

/* Recompute obs[e] from the current state of local env e. */
int wdco_observe(const wdco_config* cfg, const wdco_state* st, int32_t e);

#ifdef __cplusplus
}
#endif
#endif /* WDC_ORACLE_H */
