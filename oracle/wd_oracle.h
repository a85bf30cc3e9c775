/*
 * wd_oracle.h — CPU oracle for the batched discrete Tag roll-out path.
 *
 * TEST INFRASTRUCTURE ONLY.  This is the plain, slow, single-threaded definition
 * of what the GPU library computes.  It shares no code, header, table or constant
 * generator with the HIP path, and nothing in the product path may include, link
 * or call it.  Only the tests, the smoke check and the benchmark's CPU-baseline
 * leg use it.
 *
 * What it follows (WarpDrive paper, arXiv 2108.13976):
 *   - Sec. 4.5 "The WarpDrive RL Workflow", items 5 and 6: done environments are
 *     re-given the initial data arrays saved at the first reset; actions are
 *     sampled per agent from the policy's probabilities.
 *   - Sec. 5.1 "Benchmark Environments", Tag paragraph: N_tag >= 1 taggers chase
 *     N_run >= 1 runners on a 2-D grid; five moves (up, down, left, right, stay);
 *     a runner is tagged once a tagger is close enough, is penalised and leaves
 *     the game; the tagger is rewarded per tag; the episode ends at the maximum
 *     step count or when every runner is tagged; with partial observations an
 *     agent sees its K closest agents.
 *   - Fig. "A sample CUDA step function signature": float observations and
 *     rewards, int actions and done flags, updated in place.
 * The paper prints no constants, no action encoding, no observation layout and no
 * worked example; every such choice is a reading of this build and is listed, with
 * its identifier R1..R17, in wd_oracle.cpp next to the code that implements it.
 *
 * Pins (tests marked "not gpu"): published Philox4x32-10 known-answer vectors and
 * an independent library implementation; hand traces on 2-4 agent grids; a
 * pure-Python brute-force re-implementation on tiny inputs; invariants and closed
 * forms.  The rule CHOICES themselves cannot be pinned to the paper (it gives
 * none): "parity unpinned against the paper" for R1..R17, pinned to the hand
 * traces and invariants instead.
 *
 * All arrays are HOST memory owned by the caller; nothing is retained between
 * calls.  Every function returns 0 on success and a negative value on a bad
 * argument.
 */
#ifndef WD_ORACLE_H
#define WD_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct wdo_config {
  int32_t num_envs;        /* E: environments held in the arrays below               */
  int32_t env_offset;      /* global id of local env 0 (RNG is keyed by global id)   */
  int32_t num_agents;      /* N                                                       */
  int32_t num_taggers;     /* N_tag; agents 0..N_tag-1 are taggers                    */
  int32_t grid_size;       /* G: square grid, coordinates in [0, G)                   */
  int32_t episode_length;  /* T                                                       */
  int32_t tag_r2;          /* tagged iff squared distance <= tag_r2; <0 disables      */
  int32_t obs_mode;        /* 0 = partial (K nearest), 1 = full                       */
  int32_t obs_k;           /* K (partial mode)                                        */
  float tag_reward;        /* per successful tag, to the credited tagger              */
  float tag_penalty;       /* to the runner on the step it is tagged                  */
  uint64_t seed;
} wdo_config;

typedef struct wdo_state {
  int32_t *pos_x, *pos_y;   /* [E][N]                                                 */
  int32_t *pos_x0, *pos_y0; /* [E][N] start positions re-applied at reset             */
  int32_t *live;            /* [E][N] 1 = in play                                     */
  int32_t *action;          /* [E][N]                                                 */
  float *reward;            /* [E][N]                                                 */
  float *obs;               /* [E][N][D]                                              */
  int32_t *t, *done, *n_live_runners, *tags_step; /* [E]                              */
} wdo_state;

enum { WDO_RESET_ALL = 0, WDO_RESET_DONE = 1 };

/* Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11): one block. */
void wdo_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);

/* The four-word random block of (seed, global env, index, step g, stream); index is
 * agent / 4 for sampling (agent i uses word i mod 4) and the agent for start positions. */
void wdo_random_block(uint64_t seed, uint32_t env, uint32_t index, uint64_t g,
                      uint32_t stream, uint32_t out[4]);

/* Uniform in [0,1) from the top 24 bits of a word. */
float wdo_uniform_from_word(uint32_t w);

/* Inverse-CDF categorical draw from A probabilities and a uniform u. */
int32_t wdo_sample_from_u(const float* p, int32_t num_actions, float u);

/* Observation row length D for a configuration (5 + 4K, or 5 + 4N in full mode). */
int32_t wdo_obs_dim(const wdo_config* cfg);

/* mode ALL: draw start positions from the seed, then put every env in its start
 * state.  mode DONE: put only envs with done == 1 back in their start state. */
int wdo_reset(const wdo_config* cfg, const wdo_state* st, int mode);

/* action[e][i] <- categorical draw from probs[e][i][0..4] with word i mod 4 of the random
 * block of (seed, env_offset + e, i / 4, g, stream 0); every agent of every env. */
int wdo_sample(const wdo_config* cfg, const wdo_state* st, const float* probs, uint64_t g);

/* One Tag step for every env with done == 0 (envs with done == 1 are untouched). */
int wdo_step(const wdo_config* cfg, const wdo_state* st);

/* Recompute obs[e] from the current state of local env e (used by reset and step;
 * exported so that tests can check it alone). */
int wdo_observe(const wdo_config* cfg, const wdo_state* st, int32_t e);

#ifdef __cplusplus
}
#endif
#endif /* WD_ORACLE_H */
