/* paac.h -- C ABI of the PAAC hot path on MI355X (gfx950).
 *
 * One synchronous iteration of parallel advantage actor-critic (paper: Section 3 "Parallel
 * Framework", Section 4 "Parallel Advantage Actor Critic", Algorithm 1) is
 *     t_max x paac_select_actions(states[t])   -- the master samples an action for every environment
 *     1     x paac_train_step(rollout)         -- bootstrap, n-step returns, gradients, update
 * Everything between the arguments and the results runs in HIP kernels of this library.
 *
 * Conventions
 *  - Pointers named *_dev are device pointers on the device of the stream given to paac_create;
 *    pointers named *_host are host pointers.  The caller owns every buffer it passes, including
 *    the workspace; the library owns only the context returned by paac_create.
 *  - Rollout tensors are time-major: element (t, e) of a [t_max, n_e] tensor sits at t*n_e + e,
 *    matching the per-timestep vectors of Algorithm 1.
 *  - Every function returning int returns PAAC_OK (0) or a negative PAAC_E_* code; the message of
 *    the last error of a context is available from paac_last_error.  Nothing throws.
 *  - paac_select_actions and paac_train_step only enqueue work on the stream; they do not
 *    synchronise it and read back nothing.  Calls on one context must not overlap in time on
 *    different streams.
 */
#ifndef PAAC_H
#define PAAC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PAAC_OK            0
#define PAAC_E_NULL       -1   /* a required pointer is NULL                                   */
#define PAAC_E_BADCONFIG  -2   /* a field of paac_config / paac_hparams is out of range        */
#define PAAC_E_WORKSPACE  -3   /* workspace missing, misaligned (256 B) or too small           */
#define PAAC_E_HIP        -4   /* a HIP runtime call failed (text in paac_last_error)          */
#define PAAC_E_STATE      -5   /* call made before paac_init_params / paac_set_state, or a read-back
                                  of train-step results before the first paac_train_step          */

#define PAAC_ARCH_NIPS    0    /* conv 16@8x8/4, conv 32@4x4/2, fc 256   (Experiments: arch_nips)   */
#define PAAC_ARCH_NATURE  1    /* conv 32@8x8/4, 64@4x4/2, 64@3x3/1, fc 512 (Experiments: arch_nature) */
#define PAAC_PREC_FP32    0
#define PAAC_PREC_BF16    1    /* bf16 MFMA operands, fp32 accumulation, fp32 master weights/state */
#define PAAC_MAX_ACTIONS  32

typedef struct paac_ctx paac_ctx;  /* opaque */

/* Static shape of the problem.  Convolutions use no padding and are followed by ReLU, as is the
 * hidden fully connected layer; the policy head has n_actions logits, the value head one output. */
typedef struct {
    int32_t arch;        /* PAAC_ARCH_*                                                   */
    int32_t n_e;         /* number of environments, >= 1                                  */
    int32_t t_max;       /* rollout length, >= 1                                          */
    int32_t n_actions;   /* 2 .. PAAC_MAX_ACTIONS                                         */
    int32_t in_c, in_h, in_w;  /* must be 4, 84, 84 (stacked, preprocessed frames)        */
    int32_t precision;   /* PAAC_PREC_*                                                   */
} paac_config;

/* Run-time hyper-parameters (Experiments: gamma .99, beta .01, RMSProp lr .0224 / decay .99 /
 * epsilon .1, clipping threshold).  value_coef scales the squared value error. */
typedef struct {
    float gamma, beta, value_coef, lr, rms_alpha, rms_eps, clip_norm;
} paac_hparams;

/* Scalars of one train step, written to device memory by the last kernel of the step.
 * total_loss = policy_loss - beta*entropy + value_coef*value_loss; grad_norm is the global L2
 * norm before clipping; clip_scale = min(1, clip_norm/grad_norm); nonfinite != 0 when the loss or
 * the norm is not finite (the update is then applied as computed, NaNs included). */
typedef struct {
    float policy_loss, entropy, value_loss, total_loss, grad_norm, clip_scale;
    int32_t nonfinite;
} paac_train_stats;

/* Bytes of device workspace paac_create needs for this configuration. */
int paac_workspace_bytes(const paac_config* cfg, size_t* bytes_out);

/* Create a context.  workspace_dev: device memory, 256-byte aligned, at least
 * paac_workspace_bytes() long, owned by the caller and kept alive until paac_destroy; its content
 * is undefined until paac_init_params or paac_set_state.  hip_stream: a hipStream_t (NULL = the
 * default stream) on which every later call of this context enqueues its work. */
int paac_create(const paac_config* cfg, void* workspace_dev, size_t workspace_bytes,
                void* hip_stream, paac_ctx** ctx_out);
void paac_destroy(paac_ctx* ctx);

/* Algorithm 1, "initialize network weights": Glorot-uniform weights from the seed
 * (W ~ U(-l, l), l = sqrt(6/(fan_in+fan_out)); element i of the canonical parameter vector uses
 * Philox uniform i of stream `seed`), zero biases, zero RMSProp state.  Synchronises the stream. */
int paac_init_params(paac_ctx* ctx, uint64_t seed);

/* Algorithm 1, action selection for one timestep: forward over the n_e states, softmax, and an
 * inverse-CDF draw (smallest k with u < p_0 + ... + p_k, summed in ascending k in fp32; A-1 if none).
 *   states_dev   uint8 [n_e, 4, 84, 84], scaled by 1/255 inside the first convolution
 *   uniforms_dev float [n_e] in [0, 1)
 *   actions_dev  int32 [n_e]            out
 *   values_dev   float [n_e]            out, V(s) of every state; may be NULL
 *   probs_dev    float [n_e, n_actions] out, pi(.|s); may be NULL */
int paac_select_actions(paac_ctx* ctx, const uint8_t* states_dev, const float* uniforms_dev,
                        int32_t* actions_dev, float* values_dev, float* probs_dev);

/* paac_select_actions for callers that must not allocate device memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): same arguments, same kernels, same results,
 * but the buffers a select call writes besides its outputs (the convolution outputs of the n_e states
 * and the fully connected layer's partial sums) live in a static device array of
 * PAAC_NOALLOC_SCRATCH_BYTES inside the library instead of the caller's workspace, the kernels are
 * launched one by one on the context's stream (no graph is built), and the call makes no hipMalloc,
 * hipFree or other allocating call.  Parameters are still read from the context's workspace.
 * A configuration whose select call needs more scratch than that is rejected with
 * PAAC_E_WORKSPACE and a message naming both sizes (the Nature network fits for every n_e up to 159 in
 * fp32 and up to 243 with bf16 operands, the smaller network beyond that).
 * Each GPU holds one such array until the process ends, and every context on that GPU shares it: the
 * array keeps the last call's contents (nothing in it has to start at zero: every byte a call reads
 * it has written before), and two such calls that overlap in time on one GPU (different streams or
 * contexts) race.  The call neither reads nor advances the rollout activation cache. */
#define PAAC_NOALLOC_SCRATCH_BYTES (16u << 20)
int paac_select_actions_noalloc(paac_ctx* ctx, const uint8_t* states_dev, const float* uniforms_dev,
                                int32_t* actions_dev, float* values_dev, float* probs_dev);

/* Algorithm 1, from the bootstrap to the parameter update, over one rollout (Section 4: the two
 * batch gradients; clipping and RMSProp per the Experiments section):
 *   R_{T+1} = V(s_{T+1});  R_t = r_t + gamma (1 - d_t) R_{t+1};  adv = R_t - V(s_t) (a constant);
 *   L = -mean(adv log pi(a_t|s_t)) - beta mean(H(pi(s_t))) + value_coef mean((R_t - V(s_t))^2);
 *   g = dL/dtheta; g *= min(1, clip_norm/||g||_2); g2 = a g2 + (1-a) g^2; theta -= lr g / sqrt(g2+eps).
 *   states_dev  uint8 [t_max+1, n_e, 4, 84, 84]; slab t_max holds s_{t_max+1} (bootstrap only)
 *   actions_dev int32 [t_max, n_e]   actions taken (values outside [0, n_actions) are clamped)
 *   rewards_dev float [t_max, n_e]   reward received for actions[t][e]
 *   dones_dev   uint8 [t_max, n_e]   1 iff the episode of env e ended on transition t
 *   hp_host     hyper-parameters (host memory, copied before the call returns)
 *   stats_dev   paac_train_stats on the device, out; may be NULL */
int paac_train_step(paac_ctx* ctx, const uint8_t* states_dev, const int32_t* actions_dev,
                    const float* rewards_dev, const uint8_t* dones_dev,
                    const paac_hparams* hp_host, paac_train_stats* stats_dev);

/* Number of parameters P (canonical vector length). */
size_t paac_param_count(const paac_ctx* ctx);

/* Copy the parameters, the RMSProp second-moment state and (optionally) the gradient of the last
 * train step (before clipping) to host arrays of P floats each, in canonical order:
 * for every conv layer W[c_out][c_in][k][k], b[c_out]; fc W[fc][c*H*W + y*W + x], fc b;
 * pi W[A][fc], pi b[A]; v W[fc], v b[1].  Any pointer may be NULL.  Synchronises the stream. */
int paac_get_state(paac_ctx* ctx, float* params_host, float* rms_host, float* grads_host);

/* Load parameters and RMSProp state (canonical order, P floats each; rms_host NULL = zeros).
 * Synchronises the stream. */
int paac_set_state(paac_ctx* ctx, const float* params_host, const float* rms_host);

/* Intermediate results of the last paac_train_step, for parity checks: logits [(t_max+1) n_e, A],
 * values [(t_max+1) n_e], returns [t_max, n_e].  Host arrays; any may be NULL.  Synchronises. */
int paac_get_train_outputs(paac_ctx* ctx, float* logits_host, float* values_host, float* returns_host);

/* Stored activations of the forward pass of the last paac_train_step, for parity checks (they decide
 * ReLU'(pre) = 1[pre > 0] in the backward pass of Section 4's gradients): rows [row0, row0 + rows) of
 * the (t_max+1) n_e forward rows.  layer 0 .. n_conv-1: output of that convolution after ReLU, per
 * row [c_out][h][w] (the bf16 configuration's stored values widened to float); layer n_conv: the
 * hidden fully connected layer after ReLU, per row [fc].  out_host: host array of rows x (values
 * per row) floats.  Synchronises the stream. */
int paac_get_train_activations(paac_ctx* ctx, int layer, int row0, int rows, float* out_host);

/* Philox4x32-10 uniforms in [0,1) on the 2^-24 grid, written to device memory: element i takes
 * word i%4 of the block with 64-bit counter offset + i/4 and 64-bit key `seed`. */
int paac_fill_uniforms(paac_ctx* ctx, uint64_t seed, uint64_t offset, float* out_dev, size_t n);

/* use_graphs = 1 (default): each distinct argument tuple of select/train is captured once as a
 * HIP graph and replayed afterwards; 0: kernels are launched one by one. */
int paac_set_graphs(paac_ctx* ctx, int use_graphs);

/* Rollout activation cache (opt-in, default off).  Algorithm 1 computes the network outputs of s_t
 * during action selection and theta does not change until the update at the end of the iteration, so
 * the forward pass of paac_train_step over states[0 .. t_max-1] repeats work already done.  With the
 * cache on, the i-th paac_select_actions call since the last paac_train_step (i = 0 .. t_max-1)
 * keeps its activations, logits and values as rows [i n_e, (i+1) n_e) of the training buffers, and
 * the next paac_train_step computes the forward pass for states[t_max] only.  The caller promises
 * that states[i] of that train step are the states given to the i-th select call (they are still
 * read: the first layer's weight gradient needs them).  If the number of select calls since the last
 * train step, paac_set_state or paac_init_params is not exactly t_max, the train step falls back to
 * the full forward pass.  Results agree with the uncached path to rounding (other tile shapes and
 * split counts are used at the smaller batch), not bit for bit. */
int paac_set_activation_cache(paac_ctx* ctx, int enabled);

/* Which algorithm the three calls run on the shared framework (Section 3: the framework serves
 * value-based methods as well as policy-gradient ones).  Default PAAC_ALG_ACTOR_CRITIC.
 * PAAC_ALG_NSTEP_Q is the value-based method of Section 2.2 on the same network: the A head outputs
 * are Q(s, .), the value node is unused (zero gradient, its parameters stay as they are).
 *   paac_select_actions: epsilon-greedy on argmax_a Q(s, a) (smallest index among equal maxima) from
 *     the one uniform per state: u < epsilon picks action floor((u / epsilon) A) (fp32), else the
 *     greedy one.  probs_dev, if given, receives that distribution; values_dev the unused node.
 *   paac_train_step: R_{T+1} = max_a' Q(s_{T+1}, a'); R_t = r_t + gamma (1 - d_t) R_{t+1} (the Bellman
 *     target, a constant for differentiation; the printed one-step target when t_max = 1);
 *     L = value_coef mean((R_t - Q(s_t, a_t))^2); clip and RMSProp as before.  stats: value_loss is the
 *     mean squared TD error, total_loss = value_coef * value_loss, policy_loss = entropy = 0;
 *     paac_get_train_outputs returns Q in logits_host.
 * epsilon in [0, 1] (ignored for actor-critic).  Takes effect from the next call. */
#define PAAC_ALG_ACTOR_CRITIC 0
#define PAAC_ALG_NSTEP_Q 1
int paac_set_algorithm(paac_ctx* ctx, int algorithm, float epsilon);

/* Per-kernel timing for roofline reports.  While enabled, select/train launch kernel by kernel
 * with a HIP event pair around each on the context's stream.  paac_kernel_times synchronises and
 * returns up to `cap` entries: name_out[i] points to a static string, ms_out[i] is the summed
 * duration and calls_out[i] the number of launches since profiling was enabled. */
int paac_set_profiling(paac_ctx* ctx, int enabled);
int paac_kernel_times(paac_ctx* ctx, int cap, const char** name_out, float* ms_out,
                      int32_t* calls_out, int32_t* n_out);

/* Algorithmic FLOPs (2 x multiply-accumulates of the conv/fc/head contractions) of one
 * select call and one train call at this configuration. */
int paac_flops(const paac_ctx* ctx, double* select_flops, double* train_flops);

const char* paac_last_error(const paac_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* PAAC_H */
