/* Host side of the parallel framework (paper, Section 3 "Parallel Framework" and Algorithm 1: n_e
 * environment instances are stepped by n_w workers in parallel, their states are batched for the one
 * model) with a SYNTHETIC environment in place of the Atari emulator, which this build does not have.
 *
 * The environment is a deterministic function of (seed, environment index, episode, step, action):
 *   - an observation is 4 stacked 84x84 uint8 frames, newest last (the paper's preprocessing);
 *   - a frame is black except for `sprites` 8x8 blocks whose position and brightness come from a
 *     counter-based hash of (seed, env, episode, step, sprite) and of the action taken (Atari-like
 *     sparsity: most pixels constant, a few objects moving);
 *   - reward in {-1, 0, +1} with probabilities 5 / 90 / 5 % from the same hash (clipped rewards);
 *   - the episode ends with probability p_done per step; the environment restarts at once and the
 *     returned state is the first observation of the new episode (three black frames + frame 0).
 * Results do not depend on the number of workers.  All buffers are host memory owned by the caller
 * (pinned memory if they are to be copied to the GPU asynchronously); nothing here touches the GPU.
 * Functions return 0 on success, -1 for a NULL argument, -2 for a bad argument. */
#ifndef PAAC_ACTORS_H
#define PAAC_ACTORS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct paac_actors paac_actors;

/* n_e environments on n_w worker threads (1 <= n_w <= n_e; environment i belongs to worker
 * i * n_w / n_e), `sprites` blocks per frame (also the knob for the cost of one emulated step). */
int paac_actors_create(int32_t n_e, int32_t n_w, uint64_t seed, float p_done, int32_t sprites, paac_actors** out);
void paac_actors_destroy(paac_actors* a);

/* Start a new episode in every environment.  states_host: [n_e, 4, 84, 84] uint8, out. */
int paac_actors_reset(paac_actors* a, uint8_t* states_host);

/* One step of every environment, in parallel over the workers; returns when all are done.
 * actions_host [n_e] in; states_host [n_e,4,84,84] in/out (the previous observation is replaced by
 * the next one, or by the first observation of a new episode); rewards_host [n_e] float and
 * dones_host [n_e] 0/1 out (1: the episode ended with this transition). */
int paac_actors_step(paac_actors* a, const int32_t* actions_host, uint8_t* states_host, float* rewards_host,
                     uint8_t* dones_host);

/* Wall time of the last paac_actors_step in seconds (start of the call to the last worker done). */
double paac_actors_last_step_seconds(const paac_actors* a);

#ifdef __cplusplus
}
#endif
#endif
