/*
 * ppo_learner.h - C ABI of the MI355X PPO learner library (libppo_learner.so).
 *
 * One context = the dedicated learner GPU of the paper's disaggregated
 * set-up (Sec. III-B, Fig. 2b, Algorithm 2): it owns the experience buffer
 * of depth images + proprioception, the actor-critic parameters, their Adam
 * state and all workspaces, and runs TrainPPO (Algorithm 2, last step) and
 * the stereo-RGB distillation update (Sec. I, Sec. III-C) on them.
 *
 * Conventions
 *  - Every function returns 0 or a negative PPO_E* code; ppo_last_error()
 *    gives the text of the last failure on that context.  No exceptions and
 *    no aborts cross this boundary.  Arguments are validated before any HIP
 *    call is made.
 *  - Pointers named d_* are DEVICE pointers owned by the caller; they must
 *    stay valid until the work enqueued by the call has run on the context's
 *    stream.  Pointers named h_* / host_* are HOST pointers.  The library
 *    never frees or keeps caller memory.
 *  - The library owns everything it allocates (in ppo_create) and releases it
 *    in ppo_destroy.  ppo_buffer_write / ppo_gae / ppo_update /
 *    distill_update allocate nothing.
 *  - Work is enqueued on the HIP stream given to ppo_create (NULL = the
 *    default stream).  Calls that fill host memory synchronise that stream;
 *    all others return as soon as the work is enqueued.
 *  - A flat sample index is s = t*num_envs + n.
 *  - Canonical parameter order (fp32): for each conv layer W[Co][Ci][3][3],
 *    b[Co]; for each hidden layer W[out][in], b[out] (the first hidden
 *    layer's input is [flatten(view0) in (c,h,w) order, flatten(view1), ...,
 *    proprio]); action head W[A][h], b[A]; and, with a value head, w_v[h],
 *    b_v, logstd[A].
 */
#ifndef PPO_LEARNER_H
#define PPO_LEARNER_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PPO_OK 0
#define PPO_EINVAL (-1) /* null pointer, NaN / out-of-range hyper-parameter            */
#define PPO_ESHAPE (-2) /* geometry the kernels do not support, or sizes do not divide */
#define PPO_ESTATE (-3) /* calls out of order (e.g. ppo_gae before all steps written)  */
#define PPO_EHIP (-4)   /* a HIP runtime call failed                                   */
#define PPO_ENOMEM (-5) /* device or host allocation failed                            */

#define PPO_MAX_LAYERS 8

typedef struct ppo_ctx ppo_ctx; /* opaque, library-owned */

/* Network and buffer geometry.  The network is the feed-forward actor-critic
 * of the benchmark configurations: a stack of 3x3 stride-2 pad-1 convolutions
 * with ReLU on each view (shared weights), flatten, concatenate proprioception,
 * ReLU hidden layers, a linear Gaussian-mean head and (optionally) a scalar
 * value head with a state-independent log-std vector (cf. the CNN -> concat
 * proprio -> MLP sketch of Sec. III-C, Fig. 3). */
typedef struct {
  int32_t num_envs, horizon;         /* N, T */
  int32_t n_views, in_c, in_h, in_w; /* 1 x 1xHxW depth, or 2 x 3xHxW stereo RGB */
  int32_t obs_dtype;                 /* element type the CALLER passes to ppo_buffer_write: 0 fp32, 1 bf16 */
  int32_t proprio_dim, act_dim;      /* P (multiple of 8), A (<= 31) */
  int32_t n_conv, conv_ch[PPO_MAX_LAYERS]; /* channel counts, each a multiple of 8 */
  int32_t conv_k, conv_stride, conv_pad;   /* must be 3, 2, 1 */
  int32_t n_fc, fc_dim[PPO_MAX_LAYERS];    /* hidden widths, each a multiple of 8, n_fc >= 1 */
  int32_t has_value_head;            /* 1 actor-critic (PPO), 0 distillation student */
  int32_t max_chunk;                 /* samples per forward/backward pass inside a minibatch; 0 = default */
  /* The deployed student's extra MLP head (Sec. IV-C: "an extra MLP head that predicts the position of the
   * object"): with aux_hidden > 0 (a multiple of 8; students only) the last aux_dim (1 .. act_dim-1) output
   * columns are  W_a2 relu(W_a1 h + b_a1) + b_a2  on the last hidden layer h, and the linear head has
   * act_dim - aux_dim rows.  The targets stay in the last aux_dim columns of the action slot; ppo_hparams.aux_dim
   * must equal this aux_dim and aux_coef weighs their error.  Canonical order: W_a1[aux_hidden][h], b_a1,
   * W_a2[aux_dim][aux_hidden], b_a2 after everything else.  0: no such head. */
  int32_t aux_hidden, aux_dim;
  /* The paper's own teacher (Sec. III-C, Fig. 3): layer normalisation after every convolution (over the C*H*W
   * values of a sample, eps 1e-5, gain and shift per channel, before the ReLU; canonical: g[Co], s[Co] after each
   * conv bias), embed_dim > 0: a linear layer flatten -> embed_dim per view (no activation; canonical W[E][flat],
   * b[E] after the convolutions) whose output is concatenated with the proprioception, and lstm_layers LSTM
   * layers of lstm_units units (gate order i, f, g, o; canonical per layer W_ih[4H][in], W_hh[4H][H], b[4H])
   * between that concatenation and the hidden layers.  With lstm_layers > 0 ppo_update trains on minibatches
   * of whole environments (back-propagation through the T steps of the horizon, the state reset where a done
   * flag is set, initial state from ppo_buffer_write_state) and num_envs must be divisible by
   * hp.minibatches.  All zero: the feed-forward network of the benchmark configurations. */
  int32_t layer_norm, embed_dim, lstm_layers, lstm_units;
} ppo_net_desc;

typedef struct {
  float gamma, lambda;          /* used by ppo_gae only through its own arguments; kept for logging */
  float clip_eps;               /* > 0 */
  float vclip_eps;              /* <= 0: value clipping off */
  float vf_coef, ent_coef;
  float lr, beta1, beta2, adam_eps;
  float max_grad_norm;          /* > 0: global gradient-norm clipping, g *= min(1, c / (||g|| + 1e-6)), before every Adam step; <= 0: off */
  float desired_kl;             /* > 0 (ppo_update only): KL-adaptive learning rate.  Before each Adam step the rate
                                   follows the minibatch's approx_kl = mean((rho-1) - log rho), the sampled estimate of
                                   KL(behaviour policy || current policy): approx_kl > 2 desired_kl divides it by 1.5
                                   (not below lr_min), approx_kl < desired_kl / 2 multiplies it by 1.5 (not above
                                   lr_max).  The rate starts from `lr` and lives on the device (no host round trip);
                                   ppo_mb_stats.lr reports what each step used.  <= 0: off, every step uses `lr`.
                                   The paper gives no schedule (Sec. III-C); this is the common one of on-policy code. */
  float lr_min, lr_max;         /* bounds of the adaptive rate; 0 < lr_min <= lr_max when desired_kl > 0 */
  float aux_coef;               /* distill_update with aux_dim > 0: weight of the auxiliary columns' error (>= 0) */
  int32_t epochs, minibatches;  /* num_envs*horizon must be divisible by minibatches */
  int32_t norm_adv;             /* 1: advantages normalised once per update over the whole rollout,
                                   (A - mean) / (population std + 1e-8); 0: raw advantages */
  int32_t lr_carry;             /* with desired_kl > 0: 1 = start from the rate the previous adaptive update of this
                                   context ended with (if there was one; else from `lr`), 0 = start from `lr` */
  int32_t aux_dim;              /* distill_update: the last aux_dim (< act_dim) head columns are an auxiliary output,
                                   0 = none; see distill_update */
  uint64_t seed;                /* permutation stream seed */
} ppo_hparams;

/* One record per optimiser step, in order epoch-major. */
typedef struct {
  float pi_loss, v_loss, entropy, approx_kl, clip_frac, grad_norm, total_loss;
  int32_t nonfinite; /* 1 if the total loss was not finite */
  float lr;          /* learning rate this step's Adam update used */
} ppo_mb_stats;

/* Create a learner for `desc` on the current HIP device; all device memory is
 * allocated here.  `hip_stream` is a hipStream_t (may be NULL).  Parameters
 * start at zero: load them with ppo_set_params. */
int ppo_create(ppo_ctx** out, const ppo_net_desc* desc, void* hip_stream);
int ppo_destroy(ppo_ctx* ctx);
const char* ppo_last_error(const ppo_ctx* ctx); /* ctx may be NULL: error of the last failed ppo_create */

int64_t ppo_param_count(const ppo_ctx* ctx);
/* Device bytes held by the experience buffer's image part (Sec. III-B sizing example). */
int64_t ppo_buffer_image_bytes(const ppo_ctx* ctx);

/* Parameters / gradients / optimiser state in canonical order, HOST fp32 arrays of
 * n = ppo_param_count() elements.  All synchronise.  ppo_get_grads returns the gradient
 * of the last minibatch processed.  Setting parameters or optimiser state is the
 * checkpoint/resume path: after get -> (new ctx) set, the next update is bit-identical (with
 * desired_kl > 0 and lr_carry = 1 the adaptive rate below belongs to the state as well). */
int ppo_set_params(ppo_ctx* ctx, const float* h_params, int64_t n);
int ppo_get_params(ppo_ctx* ctx, float* h_params, int64_t n);
int ppo_get_grads(ppo_ctx* ctx, float* h_grads, int64_t n);
int ppo_set_opt_state(ppo_ctx* ctx, const float* h_m, const float* h_v, int64_t n, int64_t step, int64_t update_idx);
int ppo_get_opt_state(ppo_ctx* ctx, float* h_m, float* h_v, int64_t n, int64_t* step, int64_t* update_idx);

/* The KL-adaptive learning rate a context carries between updates (hp.desired_kl > 0, hp.lr_carry = 1): part of
 * a checkpoint beside the optimiser state.  get: *h_live = 1 and *h_lr = the rate the last adaptive update ended
 * with, or *h_live = 0 (no adaptive update has run; *h_lr = 0).  set with live = 1 installs `lr` (> 0) as that
 * rate, live = 0 forgets it (the next adaptive update starts from hp.lr).  Both synchronise. */
int ppo_get_adaptive_lr(ppo_ctx* ctx, float* h_lr, int32_t* h_live);
int ppo_set_adaptive_lr(ppo_ctx* ctx, float lr, int32_t live);

/* Append the step-t record of all N environments to the trajectory buffer
 * (Algorithm 2: D <- D u {(obs, actions, rew, done)}), plus the behaviour
 * policy's log-prob and value that PPO needs.  Device inputs:
 *   d_obs     [N][n_views][in_c][in_h][in_w], fp32 or bf16 per desc.obs_dtype
 *   d_proprio [N][P] fp32     d_action [N][A] fp32 (for distillation: the teacher's action)
 *   d_logp, d_value, d_reward [N] fp32, d_done [N] uint8   (may all be NULL for a distillation student)
 * Images are narrowed to bf16 (round to nearest even) and stored channel-last.
 * t must be in [0, T); writing t = 0 starts a new rollout. */
int ppo_buffer_write(ppo_ctx* ctx, int32_t t, const void* d_obs, const float* d_proprio, const float* d_action,
                     const float* d_logp, const float* d_value, const float* d_reward, const uint8_t* d_done);

/* ppo_buffer_write for the environments [env_offset, env_offset + count) of step t only; every array
 * holds `count` rows.  This is the landing call for observations that arrive from several producers
 * (the simulator GPUs of Fig. 2b each own a range of environments and send their slice once per
 * step): the ranges may come in any order; step t counts as written once the ranges received for it
 * cover [0, N); within a rollout a write into a complete step starts that step afresh.  A range that
 * arrives while ALL T steps are complete is the first slice of the next rollout: every step then counts
 * as unwritten until its own ranges have covered [0, N) again (to replace a whole step of a complete
 * rollout in place use ppo_buffer_write).  count = 0 is a no-op; a range outside [0, N) is PPO_EINVAL. */
int ppo_buffer_write_range(ppo_ctx* ctx, int32_t t, int32_t env_offset, int32_t count, const void* d_obs, const float* d_proprio,
                           const float* d_action, const float* d_logp, const float* d_value, const float* d_reward,
                           const uint8_t* d_done);

/* Policy step of the collection loop (Algorithm 2: the policy maps the stacked observations of all
 * environments to actions; the record is appended once the simulators have stepped).  Stores the
 * step-t observations like ppo_buffer_write, runs the network forward on them with the current
 * parameters and samples the diagonal-Gaussian policy,
 *   a = mu + exp(logstd) * xi,   logp = sum_j [-((a_j-mu_j)/sigma_j)^2/2 - logstd_j - ln(2 pi)/2],
 * with the standard-normal draws xi supplied by the caller (d_noise [N][A] fp32, device).  Action,
 * log-prob and value go into the step-t slab and, where the pointers are not NULL, to the DEVICE
 * arrays d_action [N][A], d_logp [N], d_value [N] (fp32).  The step counts as written only after
 * ppo_buffer_write_outcome(t).  Actor-critic contexts only (else PPO_ESTATE); t = 0 starts a new rollout. */
int ppo_act(ppo_ctx* ctx, int32_t t, const void* d_obs, const float* d_proprio, const float* d_noise, float* d_action,
            float* d_logp, float* d_value);
/* Reward and termination flag of step t (device, [N] fp32 / uint8), known only after the
 * simulators have stepped (Algorithm 2: obs, rew, done <- step(actions)); completes a record
 * begun by ppo_act, or replaces these two fields of a record written by ppo_buffer_write.
 * PPO_ESTATE when step t holds no record. */
int ppo_buffer_write_outcome(ppo_ctx* ctx, int32_t t, const float* d_reward, const uint8_t* d_done);

/* Recurrent nets (lstm_layers > 0): the LSTM state of every environment at the START of the rollout in the
 * buffer (the state the acting policy had when it took step 0), DEVICE fp32 arrays [lstm_layers][N][lstm_units];
 * NULL = zeros.  Kept until the next call; a new context starts from zeros.  PPO_ESTATE for a feed-forward net. */
int ppo_buffer_write_state(ppo_ctx* ctx, const float* d_h0, const float* d_c0);

/* Read back the step-t images as stored (bf16) into a DEVICE array in the caller's layout
 * [N][n_views][in_c][in_h][in_w] (bf16).  Test hook for the write path. */
int ppo_buffer_read_obs(ppo_ctx* ctx, int32_t t, void* d_obs_bf16);

/* Generalised advantage estimation over the buffer, per environment, reverse in time:
 *   delta_t = r_t + gamma (1-d_t) V_{t+1} - V_t,  A_t = delta_t + gamma lambda (1-d_t) A_{t+1},  R_t = A_t + V_t
 * with V_T = d_last_value[n] (device, [N] fp32).  Needs all T steps written (else PPO_ESTATE). */
int ppo_gae(ppo_ctx* ctx, const float* d_last_value, float gamma, float lambda);
/* Copy advantages and returns ([T][N] fp32) to DEVICE arrays (either may be NULL). */
int ppo_get_adv_ret(ppo_ctx* ctx, float* d_adv, float* d_ret);

/* The permutation the next update will use for `epoch` (device kernel, result copied to
 * HOST int32[N*T]); minibatch m is entries [m*B, (m+1)*B).  A recurrent net shuffles whole environments:
 * the first N entries are then a permutation of 0..N-1 and the rest of h_perm is left untouched. */
int ppo_permutation(ppo_ctx* ctx, uint64_t seed, uint64_t update_idx, uint64_t epoch, int32_t* h_perm);

/* ppo_permutation for callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): needs no context and calls no hipMalloc / hipFree or any allocating
 * routine.  The same kernels write the permutation of 0..S-1 for (seed, update_idx, epoch) into the DEVICE array
 * d_perm [S] (int32, caller-owned), enqueued on hip_stream (a hipStream_t, may be NULL); nothing synchronises.
 * Their scratch (histogram, bucket starts, bucket-ordered indices) lives in a static device array of the
 * library, 4.4 MiB per GPU the library is used on, resolved once per device on the first call there (or by
 * ppo_create).  S <= PPO_STATIC_PERM_MAX (else PPO_ESHAPE); S = 0 is a no-op.  All calls on one GPU share that
 * array: two calls whose work overlaps in time on one GPU (different streams, or different threads) race;
 * calls on one stream are ordered and safe.  Errors are reported through ppo_last_error(NULL). */
#define PPO_STATIC_PERM_MAX (1 << 20)
int ppo_permutation_static(int64_t S, uint64_t seed, uint64_t update_idx, uint64_t epoch, int32_t* d_perm, void* hip_stream);

/* TrainPPO (Algorithm 2): epochs x minibatches of forward, clipped-surrogate + value +
 * entropy loss, backward and one Adam step each.  Needs ppo_gae (else PPO_ESTATE).
 * host_stats: HOST array [epochs*minibatches] or NULL (NULL = fully asynchronous). */
int ppo_update(ppo_ctx* ctx, const ppo_hparams* hp, ppo_mb_stats* host_stats);

/* Distillation update of a student (has_value_head = 0): MSE between the student's
 * action and the teacher action stored in the buffer's action slot; no GAE needed.
 * With hp->aux_dim = X > 0 the last X head columns are an auxiliary regression output (the deployed
 * student's object-position output, Sec. IV-C) whose target sits in the same columns of the action
 * slot; the paper gives no weighting, the loss taken is
 *   L = mean_b[ 1/(A-X) sum_{j<A-X} e_bj^2 ] + aux_coef * mean_b[ 1/X sum_{j>=A-X} e_bj^2 ],
 * and the two means are reported as pi_loss and v_loss.  X = 0: the mean over batch and all A columns. */
int distill_update(ppo_ctx* ctx, const ppo_hparams* hp, ppo_mb_stats* host_stats);

/* Forward only, on `count` buffer samples given by DEVICE int32 indices d_idx (NULL = samples
 * 0..count-1): action means to d_mu [count][A] fp32 and values to d_v [count] fp32 (may be NULL). */
int ppo_forward(ppo_ctx* ctx, const int32_t* d_idx, int64_t count, float* d_mu, float* d_v);

#ifdef __cplusplus
}
#endif
#endif
