/*
 * libpql — the learner hot path of Parallel Q-Learning (PQL, Li et al., ICML 2023) for one
 * AMD MI355X (gfx950).  C ABI: plain pointers and sizes only.
 *
 * What the calls compute follows the paper's own statement of the method:
 *   - Section 3.1 (Scheme overview, "Data Transfer"): the Actor produces N tuples
 *     (s_t, a_t, s_{t+1}, r_t, d_{t+1}) per step; the V-learner keeps its replay buffer in GPU
 *     memory and samples i.i.d. batches from it;
 *   - Section 3 (Method): built on DDPG with double Q-learning, n-step returns, a target
 *     network Q';
 *   - Section 3.2: the V-learner's lagged local policy pi^v plays the role of the target policy
 *     and is refreshed by hard copies;
 *   - Section 3.3: mixed exploration noise;
 *   - Algorithm 1 (Actor), Algorithm 2 (P-learner), Algorithm 3 (V-learner);
 *   - Table B.1: Adam, target update rate tau, n = 3, gamma = 0.99, batch 8192.
 *
 * CONVENTIONS
 *   Return value   Every function returning int32_t returns PQL_OK (0) or a negative PQL_ERR_*
 *                  code.  Nothing aborts or throws across this boundary.  Argument errors are
 *                  found on the host before any kernel is launched and leave all state
 *                  (context counters and device buffers) unchanged.  PQL_ERR_HIP means the HIP
 *                  runtime refused a launch part-way through a call: the device buffers the
 *                  call writes are then undefined and its counter is not advanced, with one
 *                  exception: pql_replay_push counts the row as soon as its copy is enqueued,
 *                  so a failure of the statistics update that follows leaves ring and cursor
 *                  consistent (the statistics block must then be reset).
 *   Memory         The library allocates NO device memory.  Every pointer marked [device] is
 *                  caller-owned device memory (fp32 unless stated) that must stay valid until
 *                  the stream has drained; the library never frees it.  Pointers marked [host]
 *                  are ordinary host memory.  The context (pql_ctx) is host memory owned by the
 *                  library between pql_create and pql_destroy.
 *   Streams        `stream` is a hipStream_t passed as void* (NULL = the default stream).  Device
 *                  calls enqueue work and return; none of them synchronises.  Scalar results
 *                  (losses) are written to caller-provided device floats.
 *   Threads        A context is plain host state without locks: calls on one context must not overlap
 *                  in time.  Different contexts may be driven from different threads; what the
 *                  library keeps per process (the address of each device's static scratch, the
 *                  dynamic-LDS grants of its kernels per device) is locked.  The per-launch timing
 *                  of pql_profile_begin / pql_profile_end is process-wide and meant for one thread.
 *   Workspace      pql_actor_act, pql_critic_update and pql_actor_update take a caller-owned
 *                  [device] scratch buffer of at least pql_workspace_bytes(cfg) bytes, 256-byte
 *                  aligned.  Its contents are undefined between calls.  Two calls that use the
 *                  same workspace must be ordered on one stream.
 *   Networks       A network is one flat fp32 vector: for each layer in order the weights
 *                  W[in][out] row-major (y = x W + b), then the bias b[out].  Hidden layers use
 *                  ELU (alpha = 1).  Actor: in = obs_dim, hidden..., out = act_dim, then tanh.
 *                  Critic: in = obs_dim + act_dim (s and a concatenated), hidden..., out = 1,
 *                  linear (num_atoms outputs, read as logits over the atoms, when the critics
 *                  are distributional).  "Twin critics" = the vector of Q_1 immediately followed by that of
 *                  Q_2.  Gradients and Adam moments use the same layout.  The caller initialises
 *                  parameters.
 *   Replay layout  The ring has T = capacity / num_envs rows; a row is one Actor step of all N
 *                  environments; slot = row * N + env.  Fields are separate arrays:
 *                  obs[T*N][obs_dim], act[T*N][act_dim], rew[T*N], next_obs[T*N][obs_dim],
 *                  done[T*N] (0.0 / 1.0), all row-major fp32.
 *   Random draws   Philox-4x32-10 (Salmon et al., SC'11) with key = the two halves of
 *                  cfg.seed and counter = (element, stream id, call number low, call number
 *                  high); stream id 1 = index sampling, 2 = exploration noise, 3 = the
 *                  P-learner's state sampling.  The call number is the context's counter for
 *                  that kind of draw, so a run is reproducible from (seed, state).
 */
#ifndef PQL_H
#define PQL_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PQL_OK                     0
#define PQL_ERR_INVALID_ARG       -1   /* a size, dimension or scalar is out of range          */
#define PQL_ERR_NULL              -2   /* a required pointer is NULL                            */
#define PQL_ERR_NOT_ENOUGH_DATA   -3   /* fewer than nstep rows have been pushed                */
#define PQL_ERR_BATCH_TOO_LARGE   -4   /* batch exceeds cfg.max_batch (workspace sizing)        */
#define PQL_ERR_HIP               -5   /* a HIP runtime call failed; see pql_last_error         */
#define PQL_ERR_ALIGNMENT         -6   /* a device pointer is not aligned as required           */
#define PQL_ERR_SCRATCH_TOO_SMALL -7   /* the configuration needs more scratch than a fixed-size */
                                       /* buffer of the library holds                            */

#define PQL_MAX_HIDDEN 8

typedef struct pql_ctx pql_ctx;

typedef struct {
    int32_t  obs_dim;                 /* o >= 1                                                  */
    int32_t  act_dim;                 /* a >= 1                                                  */
    int32_t  num_envs;                /* N >= 1 parallel environments                            */
    int64_t  capacity;                /* replay size in transitions; T = capacity / N >= nstep   */
    int32_t  nstep;                   /* n >= 1 (Table B.1: 3)                                   */
    float    gamma;                   /* discount in (0, 1]                                      */
    int32_t  n_hidden;                /* 1..PQL_MAX_HIDDEN hidden layers, same for actor/critic  */
    int32_t  hidden[PQL_MAX_HIDDEN];  /* widths, each >= 1                                       */
    int32_t  max_batch;               /* largest batch_size / num_envs any call will use;        */
                                      /* (max_batch / 4 + 24) * (widest layer or input + 64) * 4 */
                                      /* must stay below 2^31 (32-bit row offsets of the weight-  */
                                      /* gradient kernel)                                         */
    uint64_t seed;                    /* key of the counter-based generator                      */
    int32_t  num_atoms;               /* 0 or 1: scalar critics.  2..64: distributional critics  */
                                      /* (PQL-D; the paper's appendix uses 51) with that many     */
                                      /* atoms                                                    */
    float    v_min, v_max;            /* support of the atoms, v_max > v_min (paper: -10, 10)     */
    int32_t  stochastic_policy;       /* 0: deterministic policy with exploration noise (PQL).    */
                                      /* 1: tanh-squashed Gaussian policy with a learnable        */
                                      /* temperature (PQL + SAC); scalar critics, act_dim <= 31   */
} pql_config;

/* [device] replay storage, sizes as under "Replay layout". */
typedef struct { float *obs, *act, *rew, *next_obs, *done; } pql_replay_storage;

/* [device] one sampled batch of B rows: idx[B] (int64 start slots), obs[B][o], act[B][a],
 * ret[B] (discounted n-step reward sum), next_obs[B][o] (state after the n-th step),
 * boot[B] (gamma^n times the product of (1 - d) over the window). */
typedef struct { int64_t *idx; float *obs, *act, *ret, *next_obs, *boot; } pql_batch;

/* Optimiser step: Adam hyper-parameters (Table B.1 names the optimiser and the learning rate)
 * and the gradient clipping bound (Table B.1 "Gradient Clipping 0.5"; the kind is not stated there:
 * here the whole gradient of one step is scaled by max_grad_norm / ||g||_2 when its Euclidean norm
 * exceeds max_grad_norm, both critics of the V-learner step counting as one gradient).
 * max_grad_norm = 0 switches clipping off. */
typedef struct { float lr, beta1, beta2, eps, max_grad_norm; } pql_adam;

/* ---- context and host-side queries (no device work) ------------------------------------ */

/* Validates cfg ([host]) and creates a context holding the ring cursor and call counters.
 * Errors: PQL_ERR_NULL, PQL_ERR_INVALID_ARG. */
int32_t pql_create(const pql_config* cfg, pql_ctx** out);
int32_t pql_destroy(pql_ctx* ctx);

int64_t pql_replay_rows(const pql_config* cfg);        /* T, or negative error                  */
int64_t pql_actor_param_count(const pql_config* cfg);  /* floats in the actor vector            */
int64_t pql_critic_param_count(const pql_config* cfg); /* floats in ONE critic vector           */
int64_t pql_workspace_bytes(const pql_config* cfg);    /* bytes of scratch for max_batch rows   */

/* Text of the last error recorded in ctx; owned by the context, valid until the next call. */
const char* pql_last_error(const pql_ctx* ctx);

/* Host state: [0] head row, [1] valid rows, [2] pushes so far, [3] sample calls so far,
 * [4] act calls so far, [5] critic Adam steps, [6] actor Adam steps, [7] state-sample calls.
 * Setting it resumes a run bit-exactly on the same device buffers. */
int32_t pql_get_state(const pql_ctx* ctx, int64_t out[8]);
int32_t pql_set_state(pql_ctx* ctx, const int64_t in[8]);

/* ---- replay (Section 3.1; Algorithm 1 append; Algorithm 3 receive + sample) ------------- */

/* Writes one Actor step — N transitions (obs[N][o], act[N][a], rew[N], next_obs[N][o], done[N],
 * all [device]) — into ring row `head`, then head = (head + 1) mod T and
 * count = min(count + 1, T).  The oldest row is overwritten when the ring is full.  The copy is
 * bit-exact.  Source arrays must not alias the storage. */
int32_t pql_replay_push(pql_ctx* ctx, pql_replay_storage storage, const float* obs, const float* act,
                        const float* rew, const float* next_obs, const float* done, void* stream);

/* Draws `batch` i.i.d. uniform start slots (with replacement) among the (count - n + 1) * N
 * windows of n consecutive rows that lie inside the valid part of the ring, and assembles the
 * n-step batch for them (Section 3: n-step returns; Algorithm 3 "sample a batch"):
 *     ret  = sum_{k<n} gamma^k r_k prod_{j<k} (1 - d_j),   boot = gamma^n prod_{j<n} (1 - d_j),
 * obs/act from the first row of the window, next_obs from its last row.
 * Sample k uses the 64-bit draw u = (word1 << 32) | word0 and position floor(u * V / 2^64).
 * Advances the sample counter.  Errors: PQL_ERR_NOT_ENOUGH_DATA if count < n,
 * PQL_ERR_BATCH_TOO_LARGE, PQL_ERR_NULL. */
int32_t pql_sample_nstep(pql_ctx* ctx, pql_replay_storage storage, int32_t batch, pql_batch out, void* stream);

/* The P-learner's batch (Algorithm 2 "sample a batch of {s_t}"; Section 3.1: the Actor sends it the
 * states only): `batch` i.i.d. uniform slots, with replacement, among all count * N stored
 * transitions (position floor(u * count * N / 2^64), drawn like pql_sample_nstep's but on generator
 * stream 3 with a counter of its own), written to idx_out[batch] ([device] int64) together with their
 * states obs_out[batch][o] ([device]; standardised while a statistics block is attached).  Only
 * storage.obs is read.  Errors: PQL_ERR_NOT_ENOUGH_DATA if nothing has been pushed,
 * PQL_ERR_BATCH_TOO_LARGE, PQL_ERR_NULL. */
int32_t pql_sample_states(pql_ctx* ctx, pql_replay_storage storage, int32_t batch, int64_t* idx_out,
                          float* obs_out, void* stream);

/* Same assembly for caller-given start slots idx[batch] ([device], each slot must start a
 * window inside the valid rows; the caller guarantees it).  out.idx is not written.  Does not
 * touch the sample counter. */
int32_t pql_gather_nstep(pql_ctx* ctx, pql_replay_storage storage, const int64_t* idx, int32_t batch,
                         pql_batch out, void* stream);

/* ---- Actor step (Section 3.3; Algorithm 1 "a_t <- pi(s_t) with mixed exploration noise") -- */

/* act_out[n][j] = clip(pi(obs[n]) [j] + sigma_n * eps, -1, 1) for the `num` environments in
 * obs[num][o] ([device]); sigma_n = sigma_min + n/(num-1) * (sigma_max - sigma_min)
 * (sigma_min when num == 1); eps ~ N(0,1) by Box-Muller from words 0 and 1 of the draw for
 * element n * act_dim + j, each turned into a 24-bit uniform ((w >> 8) + 0.5) / 2^24.
 * num <= cfg.max_batch.  Advances the act counter. */
int32_t pql_actor_act(pql_ctx* ctx, const float* actor_params, const float* obs, int32_t num,
                      float sigma_min, float sigma_max, float* act_out, void* workspace, void* stream);

/* ---- V-learner step (Algorithm 3 "update Q_1, Q_2 by minimizing the mean-squared Bellman
 *      error (with Double Q-learning)"; Section 3.2 for the lagged target policy) ----------- */

/* Distributional critics (cfg.num_atoms = l >= 2; Section 3 "PQL-D", appendix paragraph "Distributional
 * critic update": categorical distribution over l fixed atoms z_k = v_min + k (v_max - v_min)/(l - 1),
 * categorical projection, cross-entropy [Bellemare et al. 2017]): p_i = softmax of critic i's l outputs.
 * The target critic with the smaller mean sum_k p'_ik z_k at (next_obs, pi^v(next_obs)) supplies the
 * next-state distribution p' (ties: the first); its atoms move to T z_j = clip(ret + boot z_j, v_min,
 * v_max) and are projected back: m_k = sum_j [1 - |T z_j - z_k| / dz]_0^1 p'_j;  L_i = -mean_b sum_k m_k
 * log p_ik(obs, act).  pql_actor_update then uses Q_i = sum_k p_ik z_k in place of the scalar critic.
 * Everything else below is unchanged.
 *
 * Scalar critics:
 * y = ret + boot * min_i Q'_i(next_obs, pi^v(next_obs));  L_i = mean_b (Q_i(obs, act) - y)^2;
 * gradient of L_1 + L_2 w.r.t. critic_params (y is a constant) is written to grads_out, then
 * one Adam step (bias-corrected, eps outside the root) updates critic_params, adam_m, adam_v
 * in place.  loss_out[3] ([device]) receives L_1, L_2 evaluated before the step and, when
 * opt.max_grad_norm > 0, the gradient norm before clipping (0 otherwise); with clipping on,
 * grads_out holds the clipped gradient, the one the step used.
 * critic_params / critic_target_params / adam_m / adam_v / grads_out: twin-critic vectors
 * (2 * pql_critic_param_count floats); actor_target_params: the lagged policy pi^v.
 * Advances the critic Adam step counter. */
int32_t pql_critic_update(pql_ctx* ctx, float* critic_params, const float* critic_target_params,
                          const float* actor_target_params, float* adam_m, float* adam_v, float* grads_out,
                          pql_batch batch, int32_t batch_size, pql_adam opt, float* loss_out,
                          void* workspace, void* stream);

/* ---- V-learner step for callers that cannot allocate device memory ----------------------- */

/* pql_critic_update without the workspace argument, for callers that may not call hipMalloc (or any
 * allocating routine) and have no scratch buffer to hand over: code under HIP graph capture, tight
 * serving / training loops, harnesses that forbid allocation.  The scratch that pql_critic_update
 * takes from its caller comes from a device array of pql_static_scratch_bytes() bytes (64 MiB) that is
 * part of the library's code object instead: every GPU the library runs on holds one copy from the
 * first call on it until the process ends.  The call allocates and frees nothing and makes no
 * synchronising call; apart from one address lookup on the first call on a device it only enqueues the
 * same kernels as pql_critic_update on `stream`, with the same arguments, results, state changes and
 * errors (the device that owns `stream` must be the current one).
 * Limit: configurations with pql_workspace_bytes(cfg) > pql_static_scratch_bytes() are rejected with
 * PQL_ERR_SCRATCH_TOO_SMALL before anything is launched (the need grows with cfg.max_batch and the layer
 * widths: obs_dim 60, act_dim 8, two hidden layers of 256 fit up to max_batch 3416).
 * All calls on one GPU, from any context, share that GPU's array: its contents are undefined between
 * calls (nothing in it has to start at zero), and two such calls that overlap on one GPU (different
 * streams or threads) race and give undefined results; order them on one stream.
 * Under graph capture the scalars of the captured call are part of the graph, as with every call of this
 * library: the step number of Adam's bias correction (and, with a stochastic policy, the call number
 * that selects the draws) are those of the capture, and the context's counters advance once, at capture
 * time; a replay repeats exactly that step. */
int64_t pql_static_scratch_bytes(void);
int32_t pql_critic_update_static(pql_ctx* ctx, float* critic_params, const float* critic_target_params,
                                 const float* actor_target_params, float* adam_m, float* adam_v, float* grads_out,
                                 pql_batch batch, int32_t batch_size, pql_adam opt, float* loss_out, void* stream);

/* ---- P-learner step (Algorithm 2 "update pi by maximizing min_i Q_i(s, pi(s))") ---------- */

/* J = -mean_b min(Q_1, Q_2)(obs_b, pi(obs_b)); the gradient w.r.t. actor_params flows through
 * the action input of whichever critic is smaller per row (ties: Q_1); critics are read-only.
 * Writes grads_out (actor layout), performs one Adam step on actor_params/adam_m/adam_v,
 * stores J (before the step) in loss_out[0] and the gradient norm before clipping in loss_out[1]
 * (0 when opt.max_grad_norm == 0); loss_out is float[2] [device].  With clipping on, grads_out holds
 * the clipped gradient.  Advances the actor Adam counter. */
int32_t pql_actor_update(pql_ctx* ctx, float* actor_params, const float* critic_params, float* adam_m,
                         float* adam_v, float* grads_out, const float* obs, int32_t batch_size, pql_adam opt,
                         float* loss_out, void* workspace, void* stream);

/* ---- optimiser (Table B.1 "Optimizer: Adam", learning rate 5e-4) ------------------------ */

/* One Adam step (Kingma & Ba, Algorithm 1: bias-corrected moments, eps added outside the
 * square root) on a flat vector with a caller-given gradient; the same kernel performs the fused
 * step inside pql_critic_update / pql_actor_update.  params/grads/adam_m/adam_v: [device],
 * `count` floats each (count < 2^31); `t` >= 1 is the step number used for the bias correction.
 * opt.max_grad_norm must be 0 (this call has no scratch for the norm).  Context counters are not
 * touched. */
int32_t pql_adam_step(pql_ctx* ctx, float* params, const float* grads, float* adam_m, float* adam_v,
                      int64_t count, pql_adam opt, int64_t t, void* stream);

/* ---- PQL + SAC (Section 3: the scheme extends to SAC; appendix paragraph "PQL for SAC"; Table B.1
 *      "Learnable Entropy Coefficient").  The paper gives no formulas; these are the definitions of
 *      Haarnoja et al. 2018 with automatic temperature. ------------------------------------------ */

/* With cfg.stochastic_policy = 1 the policy network has 2a outputs (mu, raw): log sigma = clip(raw, -5, 2),
 * a = tanh(u), u = mu + sigma eps, eps ~ N(0, 1) per (row, action dimension) (element row * a + dim;
 * generator stream 2 in pql_actor_act, 4 in pql_critic_update, 5 in pql_actor_update, call number = that
 * call's counter), log pi(a|s) = sum_d [-eps^2/2 - log sigma - log(2 pi)/2 - log(1 - a^2)].
 *   pql_actor_act     a sample of the policy; sigma_min / sigma_max are ignored.
 *   pql_critic_update y = ret + boot * (min_i Q'_i(next_obs, a') - alpha log pi^v(a'|next_obs)), a' ~ pi^v.
 *   pql_actor_update  J = mean_b [alpha log pi(a_b|obs_b) - min_i Q_i(obs_b, a_b)] with the reparameterised
 *                     sample; the clip passes no gradient outside (-5, 2); then one Adam step (same
 *                     constants, step number of this call) on log alpha for
 *                     J(alpha) = -alpha mean_b (log pi(a_b|obs_b) + target_entropy).
 *                     loss_out is float[4]: [0] = -mean_b min_i Q_i, [1] = gradient norm (as above),
 *                     [2] = alpha mean_b log pi, [3] = mean_b log pi; J = [0] + [2].
 * alpha = exp(temperature[0]); `temperature` is a caller-owned, caller-initialised [device] float[4]
 * {log alpha, Adam m, Adam v, unused}, 16-byte aligned, that must be attached before the first update
 * (PQL_ERR_NULL otherwise).  Errors: PQL_ERR_INVALID_ARG for a context with a deterministic policy. */
int32_t pql_sac_attach(pql_ctx* ctx, float* temperature, float target_entropy);

/* The V-learner's copy of the temperature (Section 3.1: each part works on local copies): while set,
 * pql_critic_update reads log alpha from log_alpha[0] ([device]) instead of temperature[0].  NULL (and every
 * pql_sac_attach) goes back to the attached block.  Host-side only. */
int32_t pql_sac_attach_lagged(pql_ctx* ctx, const float* log_alpha);

/* ---- observation standardisation (Table B.1 "Normalized Observations: True"; the mechanism is
 *      not described there) ---------------------------------------------------------------- */

/* Running per-dimension statistics of every observation s_t pushed so far: count, mean and
 * sum of squared deviations in double precision (merged batch by batch with the pairwise update
 * of Chan, Golub and LeVeque), population variance = m2 / count.  Before the first push the mean
 * is 0 and the variance 1.  The statistics live in a caller-owned [device] block of
 * pql_obs_norm_bytes(cfg) bytes, 256-byte aligned, laid out as
 *     double count, reserved, mean[o], m2[o];  float mean32[o], rstd32[o];  scratch,
 * rstd32 = 1 / sqrt(var + eps).  While a block is attached:
 *   - pql_replay_push merges its obs[N][o] argument into the statistics (after the copy; the ring
 *     keeps raw observations);
 *   - pql_sample_nstep / pql_gather_nstep write out.obs and out.next_obs standardised,
 *     (x - mean32) * rstd32, with the statistics current on the stream at that point;
 *   - pql_actor_act standardises its obs argument the same way before the policy.
 * pql_obs_norm_attach(ctx, NULL, 0) detaches.  Attach does no device work; pql_obs_norm_reset
 * enqueues the initialisation of the attached block (count 0) and must precede its first use.
 * Errors: PQL_ERR_ALIGNMENT, PQL_ERR_INVALID_ARG (eps < 0), PQL_ERR_NULL (reset with no block). */
int64_t pql_obs_norm_bytes(const pql_config* cfg);
int32_t pql_obs_norm_attach(pql_ctx* ctx, void* stats, float eps);
int32_t pql_obs_norm_reset(pql_ctx* ctx, void* stream);

/* ---- target tracking (Table B.1 target update rate; Section 3.2 hard policy sync) -------- */

/* dst[i] = tau * src[i] + (1 - tau) * dst[i] for i < count ([device], may not partially
 * overlap).  tau = 1 copies src bit-exactly, tau = 0 leaves dst bit-exactly unchanged.
 * 0 <= tau <= 1. */
int32_t pql_soft_update(pql_ctx* ctx, const float* src, float* dst, int64_t count, float tau, void* stream);

/* ---- work that follows an optimiser step, folded into it ----------------------------------- */

/* Algorithm 3 moves the target critics Q' towards Q after every critic update (Table B.1 target update
 * rate), and Section 3.2 has the lagged policy pi^v follow pi by hard copies.  Done with pql_soft_update,
 * each is one more pass over a few MB right after the optimiser's; while a vector is attached here, the
 * optimiser kernel of the update itself performs it on the parameters it has just computed:
 *   PQL_TRACK_CRITIC_TARGETS  at the end of every pql_critic_update: dst (2 * pql_critic_param_count floats)
 *                             = tau * critic_params + (1 - tau) * dst.  dst may be the call's own
 *                             critic_target_params (the target path has read them by then).
 *   PQL_TRACK_LAGGED_POLICY   at the end of every pql_actor_update: dst (pql_actor_param_count floats)
 *                             = tau * actor_params + (1 - tau) * dst (tau = 1: the hard copy).
 * The result equals, bit for bit, that of pql_soft_update(params, dst, count, tau) enqueued right after the
 * update; the caller then omits that call.  tau = 0 and dst = NULL switch it off.  With gradient clipping on
 * it rides on the kernel that applies the clipped step (same result).  Host-side only.
 * Errors: PQL_ERR_INVALID_ARG (unknown vector, tau outside [0, 1]). */
#define PQL_TRACK_CRITIC_TARGETS 0
#define PQL_TRACK_LAGGED_POLICY  1
int32_t pql_track_attach(pql_ctx* ctx, int32_t which, float* dst, float tau);

/* The backward products delta * W^T read transposed copies of the online critics' and the policy's weight
 * matrices.  Without a cache every update transposes them into its workspace first (one small launch per
 * call).  With a caller-owned [device] block of pql_weight_cache_bytes(cfg) bytes, 256-byte aligned,
 * attached, the copies live there between calls: pql_weight_cache_refresh(ctx, critic_params, actor_params)
 * fills it from the given vectors (either may be NULL) and remembers their addresses; a later
 * pql_critic_update / pql_actor_update whose critic_params / actor_params argument is that same address
 * reads the block instead of transposing, and the optimiser kernel writes the transposes of the parameters
 * it has just updated back into it.  Calls with other parameter vectors (a snapshot, another network) are
 * unaffected: they transpose into their workspace as before.
 * The caller must call pql_weight_cache_refresh again after changing a remembered vector by any other
 * means (a copy into it, pql_adam_step, pql_soft_update with it as dst, loading a checkpoint) and before
 * the first update; attaching (also NULL, which detaches) forgets both vectors.  Results are the same with
 * and without the cache, bit for bit.
 * Errors: PQL_ERR_ALIGNMENT, PQL_ERR_NULL (refresh with no block attached). */
int64_t pql_weight_cache_bytes(const pql_config* cfg);
int32_t pql_weight_cache_attach(pql_ctx* ctx, void* cache);
int32_t pql_weight_cache_refresh(pql_ctx* ctx, const float* critic_params, const float* actor_params, void* stream);

/* ---- inspection aid ----------------------------------------------------------------------- */

/* Where the per-row results of the last update lie inside that call's workspace (Algorithm 3: the
 * target y; Algorithms 2 and 3: Q_1, Q_2).  *offset_bytes receives the byte offset, from the start of
 * the workspace, of a float[batch_size] array:
 *   PQL_VIEW_TD_TARGET  y_b = ret_b + boot_b * min_i Q'_i(next_obs_b, pi^v(next_obs_b)) of the last
 *                       pql_critic_update (with the entropy term when the policy is stochastic);
 *                       scalar critics only;
 *   PQL_VIEW_Q1, _Q2    Q_i(obs_b, act_b) as evaluated by the last pql_critic_update before its step
 *                       (scalar critics only), or Q_i(obs_b, pi(obs_b)) of the last pql_actor_update
 *                       (the distribution's mean for distributional critics).
 * Valid once the stream has drained and until the next call that uses the workspace.  Host-side only.
 * Errors: PQL_ERR_NULL, PQL_ERR_INVALID_ARG (bad cfg or `what`). */
#define PQL_VIEW_TD_TARGET 0
#define PQL_VIEW_Q1        1
#define PQL_VIEW_Q2        2
int32_t pql_workspace_view(const pql_config* cfg, int32_t what, int64_t* offset_bytes);

/* ---- measurement aid -------------------------------------------------------------------- */

/* Per-kernel timing with HIP events on the stream each kernel is launched on.  Between
 * pql_profile_begin and pql_profile_end every kernel launch made by this library (any context,
 * one thread) carries a start and a stop event attached to the dispatch itself, up to
 * max_launches launches; later launches run untimed.  pql_profile_end waits for the recorded events and returns one entry per kernel that
 * ran ([host] array `out` of max_out entries; *n_out = number of kernels seen): launches, summed
 * duration in ms, and the summed ALGORITHMIC work of those launches: flops = 2 * M * N * K of the
 * real (unpadded) matrices for the GEMM kernels; bytes = minimum traffic the step implies for
 * the copy / gather / optimiser kernels.  Event recording perturbs timing: do not use it inside
 * a throughput measurement. */
typedef struct {
    char    name[64];
    int64_t launches;
    double  total_ms;
    double  flops;
    double  bytes;
} pql_kernel_stat;

/* Achievable matrix-core rate: `blocks` workgroups of 4 wavefronts each issue 4 * iters independent
 * v_mfma_f32_32x32x2_f32 on register operands (no memory traffic) and store one float per thread to
 * out[blocks * 256] ([device]).  Work = blocks * 4 * 4 * iters * 4096 FLOP; time it with events or
 * through pql_profile_begin / pql_profile_end (kernel "mfma_probe_kernel").  This is the ceiling the
 * matrix pipelines sustain at the clock the chip holds under that load, for comparison with the
 * nominal peak. */
int32_t pql_probe_mfma(pql_ctx* ctx, float* out, int32_t blocks, int32_t iters, void* stream);

int32_t pql_profile_begin(pql_ctx* ctx, int32_t max_launches);
int32_t pql_profile_end(pql_ctx* ctx, pql_kernel_stat* out, int32_t max_out, int32_t* n_out);

#ifdef __cplusplus
}
#endif
#endif /* PQL_H */
