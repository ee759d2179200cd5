/*
 * tsdp.h - C ABI of the MI355X speculative draft-then-verify denoising round of TS-DP.
 *
 * One call of tsdp_round() performs, for a batch of B independent environments, one round of the
 * paper's Section 3.2: the drafter rolls out up to K DDPM reverse steps (Draft Generation Procedure,
 * Eq. (3)), the base denoiser scores all drafted input states in one ragged batch (Verification of
 * Speculative Drafts), and every drafted transition passes the Gaussian likelihood-ratio test of
 * Section 3.1 (Eq. (2), first-rejection index Eq. (3) of the preliminaries) with the first rejected
 * draft corrected by reflection-maximal coupling (Section 3.1, reflection equations).  tsdp_draft,
 * tsdp_verify and tsdp_accept expose the three stages on caller-owned buffers.
 *
 * Conventions
 *  - Every function returns 0 on success or a negative TSDP_E_* code; nothing throws or aborts.
 *    tsdp_last_error() returns a message for the last failing call on that context.
 *  - Pointers named d_* are DEVICE pointers owned by the caller; h_* are HOST pointers.  The library
 *    neither frees nor keeps caller pointers beyond the work it enqueues (exception: tsdp_set_cond
 *    caches derived tensors in context-owned memory, not the pointer).
 *  - `stream` is a hipStream_t passed as void* (NULL = the null stream).  All work is enqueued on it and
 *    no call synchronises, except tsdp_create / tsdp_load_weights / tsdp_destroy / tsdp_status.  (Whole rounds --
 *    tsdp_round, tsdp_round_threshold, the chain drivers -- may run one kernel on a second stream that the context
 *    owns, of the same priority, forked from `stream` and joined back into it by events inside the call: work
 *    enqueued on `stream` after the call still runs after all of the call's work, and the fork / join is recorded
 *    like any other work when `stream` is being captured into a HIP graph.)
 *  - Latents, noise predictions, noises and means are fp32 in every configuration; only the network
 *    internals follow tsdp_config.dtype.  All tensors are dense row-major.
 *  - Timesteps run t = T-1 .. 0; a latent "at t" is x_t; t = -1 marks a finished environment.
 *  - Ragged row table: environment b owns rows row_ptr[b] .. row_ptr[b+1]-1; row row_ptr[b]+k-1 holds the
 *    input state y_{k-1} of drafted transition k at timestep t0[b]-k+1.  K_eff = min(K, t0).  An
 *    environment at t0 = 0 owns one row (the deterministic last base step); a finished one owns none.
 *  - H*A must be a multiple of 4 and at most 512.  The context owns weights, tables and workspace; calls on one
 *    context must not overlap in time (they share the workspace).
 */
#ifndef TSDP_H
#define TSDP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TSDP_OK        0
#define TSDP_E_INVAL  -1   /* null pointer, bad enum, value out of range */
#define TSDP_E_SHAPE  -2   /* shape not supported or exceeding B_max / K_max / blob size mismatch */
#define TSDP_E_NOMEM  -3   /* device or host allocation failed */
#define TSDP_E_HIP    -4   /* a HIP runtime call failed */
#define TSDP_E_STATE  -5   /* weights not loaded / conditioning not set */

typedef struct tsdp_ctx tsdp_ctx;

typedef struct {
  int32_t dtype;          /* 0 = fp32 network, 1 = bf16 weights + bf16 matrix-multiply inputs, fp32 accumulate */
  int32_t H, A;           /* horizon (tokens per latent), action dimension */
  int32_t cond_mode;      /* 0 = conditioning vector through FiLM, 1 = observation tokens through cross-attention */
  int32_t cond_dim;       /* vector length (mode 0) or feature size of one token (mode 1) */
  int32_t cond_tokens;    /* number of observation tokens (mode 1), 0 otherwise */
  int32_t base_layers, base_d, base_heads, base_mlp_ratio;
  int32_t draft_layers, draft_d, draft_heads, draft_mlp_ratio;
  int32_t T;              /* DDPM steps */
  int32_t schedule;       /* 0 = linear beta0..beta1, 1 = squared cosine (offset 0.008, beta cap 0.999) */
  float   beta0, beta1;
  int32_t clip_x0;        /* 1 = clamp the predicted clean sample to [-clip_val, clip_val] */
  float   clip_val;
  int32_t B_max, K_max;   /* largest batch and largest per-environment draft count */
  uint64_t seed;          /* Philox4x32-10 key */
  int32_t sampler;        /* 0 = DDPM posterior step, 1 = DDIM(eta) step (Section 3.2, Draft Model Training, names both schedulers) */
  float   eta;            /* DDIM only, in (0,1]: sigma_t = eta sqrt((1-abar_{t-1})/(1-abar_t)) sqrt(1-abar_t/abar_{t-1});
                             eta = 0 has no Gaussian transition to test against and is rejected */
  int32_t bonus_row;      /* 1 = every running environment gets one more verify row, the state reached by its last
                             draft (the K+1-member candidate set of Section 3.1): if all drafts pass, the base model's
                             prediction there gives an exact extra base step, so a round advances up to K_eff + 1 steps.
                             Row buffers then hold B*(K_max+1) rows and K = 0 (a plain base step) is allowed */
  int32_t norm;           /* normalisation of both networks: 0 = LayerNorm, 1 = RMSNorm (x / sqrt(mean x^2 + 1e-5)),
                             both without affine parameters */
} tsdp_config;

/* Builds the DDPM tables (fp64 on the host, stored fp32) and an empty context.  Synchronous. */
int tsdp_create(const tsdp_config* cfg, tsdp_ctx** out_ctx);

/* Frees everything the context owns.  Synchronises the device.  NULL is allowed. */
void tsdp_destroy(tsdp_ctx* ctx);

/* Environment: TSDP_DISABLE_FUSED (any value), read by tsdp_load_weights, keeps a network on the general fp32
 * operator kernels even where a fused kernel exists for its shape (a diagnostic; tsdp_path_name reports the path). */

/* Loads one denoiser (which: 0 = base, 1 = drafter) from a HOST blob of fp32 values: the tensors
 * tok_w[d,A] tok_b[d] pos[H,d] t_w1[d,d] t_b1[d] t_w2[d,d] t_b2[d] (mode 0: c_w[d,C] c_b[d]) then per
 * layer mod_w[4d,d] mod_b[4d] qkv_w[3d,d] qkv_b[3d] o_w[d,d] o_b[d] (mode 1: cq_w[d,d] cq_b[d]
 * ck_w[d,Cdim] ck_b[d] cv_w[d,Cdim] cv_b[d] co_w[d,d] co_b[d]) up_w[m,d] up_b[m] dn_w[d,m] dn_b[d]
 * and finally head_w[A,d] head_b[A]; Linear weights are [out,in] row-major, m = mlp_ratio*d.
 * nbytes must equal the blob size exactly.  In bf16 mode all values are rounded to bfloat16 (nearest
 * even).  The blob is copied and re-laid-out; the caller may free it on return.  Synchronous. */
int tsdp_load_weights(tsdp_ctx* ctx, int which, const float* h_blob, size_t nbytes);

/* Conditioning of the B environments of the following calls: d_cond is [B,cond_dim] (mode 0) or
 * [B,cond_tokens,cond_dim] (mode 1), fp32.  Caches what depends on it only (conditioning embedding, or
 * the cross-attention keys / values of every layer) for both networks.  Needs both weight sets. */
int tsdp_set_cond(tsdp_ctx* ctx, const float* d_cond, int B, void* stream);

/* Drafter rollout (Section 3.2, Draft Generation Procedure).
 * in : d_x[B,H,A], d_t0[B], d_K[B] (clamped to 1..K_max, to 0..K_max with bonus_row; status bit 0 reports it),
 *      d_sigma_scale[B] (the scheduler's multiplier of sigma_t, must be > 0: it divides the mean difference in the
 *      acceptance ratio; status bit 2 reports a value that is not),
 *      d_env_id[B] global environment index used as Philox counter word (NULL = 0..B-1)
 * out: d_row_ptr[B+1], d_row_t[R_cap], d_row_env[R_cap], d_states[R_cap,H,A], d_eps_p[R_cap,H,A],
 *      d_xi[R_cap,H,A] (NULL = do not store the noise: tsdp_accept can regenerate it from the Philox counters),
 *      d_y_last[B,H,A] (the latent after the last drafted step; x itself if no step
 *      was drafted).  R_cap = B*(K_max + bonus_row) rows must be allocated; rows beyond row_ptr[B] are not
 *      written.  Rows of environment b: K_eff = min(K, t0) drafted rows at timesteps t0, t0-1, ...; an environment
 *      at t0 = 0 has the lone row (x, t = 0) of its deterministic base step; with bonus_row every running
 *      environment ends with the row (y_{K_eff}, t0 - K_eff), whose d_xi is the noise of a base step from it
 *      (zero at timestep 0) and whose d_eps_p is zero. */
int tsdp_draft(tsdp_ctx* ctx, int B, const float* d_x, const int32_t* d_t0, const int32_t* d_K,
               const float* d_sigma_scale, const int32_t* d_env_id,
               int32_t* d_row_ptr, int32_t* d_row_t, int32_t* d_row_env,
               float* d_states, float* d_eps_p, float* d_xi, float* d_y_last, void* stream);

/* Batched verification (Section 3.2, Verification of Speculative Drafts): base-network noise
 * prediction for every row of a ragged batch.  R_cap bounds the launch (<= B_max*(K_max + bonus_row)); the live row
 * count is read on the device from d_row_ptr[B].  Row r uses timestep d_row_t[r] and the conditioning
 * of environment d_row_env[r] (index into the batch given to tsdp_set_cond); both are range-checked on the device
 * (clamped, reported by tsdp_status).  Rows at and beyond row_ptr[B] are neither read nor written.
 * out: d_eps_q[R_cap,H,A]. */
int tsdp_verify(tsdp_ctx* ctx, int B, int R_cap, const int32_t* d_row_ptr, const int32_t* d_row_t,
                const int32_t* d_row_env, const float* d_states, float* d_eps_q, void* stream);

/* Acceptance (Section 3.1 Eqs. (2),(3) and reflection coupling; Section 3.2 log acceptance ratio):
 * per row d = (mu_p - mu_q)/(s sigma_t), log alpha = -|d|^2/2 - <d,xi>; accepted iff
 * log U_{env,t} <= log alpha; first rejection j*; the output latent is y_{K_eff} if all drafts pass,
 * else the reflection of draft j*; t_next = t0 - (steps advanced).  Arithmetic is fp64 on fp32 data.
 * d_xi = NULL: the noise of every row is regenerated in the kernel from (seed, d_env_id, timestep), the same Philox
 * blocks tsdp_draft drew (one third fewer bytes read; tsdp_accept_threshold has no environment ids and needs d_xi).
 * A base row (the lone row at t0 = 0; the last row of every environment with bonus_row) is not tested: when no
 * draft before it was rejected the output is mu_q(state, eps_q) + s sigma_t xi of that row, one more step.
 * out: d_x_out[B,H,A], d_t_next[B], d_n_accept[B]; optional (NULL to skip): d_n_adv[B],
 *      d_flags[R] (1 = accepted draft), d_logratio[R], d_logu[R] (all 0 on base rows). */
int tsdp_accept(tsdp_ctx* ctx, int B, const int32_t* d_row_ptr, const int32_t* d_row_t,
                const int32_t* d_env_id, const float* d_sigma_scale, const float* d_states,
                const float* d_eps_p, const float* d_eps_q, const float* d_xi, const float* d_y_last,
                float* d_x_out, int32_t* d_t_next, int32_t* d_n_accept, int32_t* d_n_adv,
                uint8_t* d_flags, float* d_logratio, float* d_logu, void* stream);

/* One whole round on context-owned ragged buffers: d_x[B,H,A] and d_t[B] are updated in place;
 * d_n_accept[B] = accepted drafts, d_n_advanced[B] = denoising steps advanced (both may be NULL). */
int tsdp_round(tsdp_ctx* ctx, int B, float* d_x, int32_t* d_t, const int32_t* d_K,
               const float* d_sigma_scale, const int32_t* d_env_id,
               int32_t* d_n_accept, int32_t* d_n_advanced, void* stream);

/* Deterministic threshold rule of Section 3.2 (a draft passes when p_i >= lambda, p_i = min{1, exp(log alpha_i)},
 * lambda in (0,1] chosen by the scheduler): the same arithmetic as tsdp_accept / tsdp_round with the comparison
 * log alpha >= log lambda[b] in place of the uniform draw.  d_lambda[B] holds one threshold per environment.  The
 * rule is not lossless with respect to the base model; the corrected sample is still the reflection of the first
 * rejected draft.  No random number is consumed by the test (the noise xi of the drafts is unchanged). */
int tsdp_accept_threshold(tsdp_ctx* ctx, int B, const int32_t* d_row_ptr, const int32_t* d_row_t,
                          const float* d_sigma_scale, const float* d_lambda, const float* d_states,
                          const float* d_eps_p, const float* d_eps_q, const float* d_xi, const float* d_y_last,
                          float* d_x_out, int32_t* d_t_next, int32_t* d_n_accept, int32_t* d_n_adv,
                          uint8_t* d_flags, float* d_logratio, void* stream);
int tsdp_round_threshold(tsdp_ctx* ctx, int B, float* d_x, int32_t* d_t, const int32_t* d_K,
                         const float* d_sigma_scale, const int32_t* d_env_id, const float* d_lambda,
                         int32_t* d_n_accept, int32_t* d_n_advanced, void* stream);

/* Whole denoising chain: rounds repeat until every environment has finished (t = -1), the inference loop of
 * Section 1 and Section 3.2.  Rounds are
 * enqueued back to back; every `check_every` rounds the number of running environments is read back (this call
 * synchronises the stream at those points) and the loop stops when it is zero or after `max_rounds`.  d_x and d_t
 * are updated in place; d_lambda selects the threshold rule (NULL = the lossless stochastic test).  Optional
 * per-environment totals over the chain (NULL to skip, zeroed by the call): accepted drafts, drafted transitions,
 * rounds in which the environment ran.  *h_rounds receives the number of rounds enqueued. */
int tsdp_chain(tsdp_ctx* ctx, int B, float* d_x, int32_t* d_t, const int32_t* d_K, const float* d_sigma_scale,
               const int32_t* d_env_id, const float* d_lambda, int max_rounds, int check_every,
               int32_t* d_tot_accept, int32_t* d_tot_drafts, int32_t* d_tot_rounds, int32_t* h_rounds, void* stream);

/* The same loop with the scheduler's three-stage action (Section 3.3, action space: one sigma scale, acceptance
 * threshold and draft count per denoising stage): d_K3, d_sigma_scale3 and d_lambda3 (NULL = stochastic test) are
 * [B,3] tables; before every round each environment takes column 0 while t >= t_hi, column 1 while t_lo <= t < t_hi,
 * column 2 below t_lo (the paper does not give the stage boundaries: they are arguments, t_hi >= t_lo >= 0). */
int tsdp_chain_staged(tsdp_ctx* ctx, int B, float* d_x, int32_t* d_t, const int32_t* d_K3, const float* d_sigma_scale3,
                      const float* d_lambda3, int t_hi, int t_lo, const int32_t* d_env_id, int max_rounds,
                      int check_every, int32_t* d_tot_accept, int32_t* d_tot_drafts, int32_t* d_tot_rounds,
                      int32_t* h_rounds, void* stream);

/* The same chain with no host round trip (Section 1 and Section 3.2, the inference loop; Section 3.3 for the stage
 * tables): exactly n_rounds rounds are enqueued on `stream` and the call returns; nothing is read back and nothing
 * synchronises.  Every kernel of a round reads the round's live row count on the device and returns at once when no
 * environment is running any more, so rounds past the end of the chain cost a few empty launches and leave latents,
 * timesteps and totals untouched.  A round advances every running environment by at least one step, so
 * n_rounds = (largest t) + 1 <= T always completes the chain.  Finished environments own no rows: the ragged verify
 * batch of a round holds the running environments only, and tiles beyond its live row count exit.
 * staged = 0: d_K[B], d_sigma_scale[B], d_lambda[B] (NULL = stochastic test) as in tsdp_chain; staged = 1: [B,3] stage
 * tables with the bounds t_hi >= t_lo >= 0 as in tsdp_chain_staged.  Totals as in tsdp_chain (device, NULL to skip);
 * d_rounds_run (device int32, NULL to skip) receives the number of rounds in which some environment ran.
 * The call records kernel launches only (no memset, no copy) and allocates nothing once the context's buffers exist
 * (after tsdp_prepare, or after any earlier round / chain call): it can be captured in a HIP graph and replayed.
 * Results are bit-identical to tsdp_chain / tsdp_chain_staged. */
int tsdp_chain_enqueue(tsdp_ctx* ctx, int B, float* d_x, int32_t* d_t, const int32_t* d_K, const float* d_sigma_scale,
                       const float* d_lambda, int staged, int t_hi, int t_lo, const int32_t* d_env_id, int n_rounds,
                       int32_t* d_tot_accept, int32_t* d_tot_drafts, int32_t* d_tot_rounds, int32_t* d_rounds_run,
                       void* stream);

/* Allocates every buffer later calls on this context may need (network workspace, round and chain buffers) and sets
 * the launch attributes of its kernels, so that the calls that follow allocate nothing: to be called once, after both
 * tsdp_load_weights, before a round or chain is captured in a HIP graph.  Synchronous; enqueues no work. */
int tsdp_prepare(tsdp_ctx* ctx);

/* Forward value of the drafter's distillation objective (Section 3.2, Draft Model Training) over R rows:
 * L_pred = mean_r |eps_p[r] - eps_q[r]|^2, L_norm = mean over rows with t > 0 of |(mu_p - mu_q)/sigma_t|^2 (DDPM
 * means from the same state, unscaled sigma_t), L = lambda1 L_pred + lambda2 L_norm.  fp64 reduction in a fixed
 * order (deterministic).  d_states is read only when x0 clipping is on.  out: d_loss[3] = {L_pred, L_norm, L}. */
int tsdp_distill_loss(tsdp_ctx* ctx, int R, const int32_t* d_row_t, const float* d_states, const float* d_eps_p,
                      const float* d_eps_q, float lambda1, float lambda2, double* d_loss, void* stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops, harnesses that
 * forbid it): tsdp_distill_loss with its partial sums in a file-scope device array of the library instead of
 * context memory.  It calls no hipMalloc / hipFree or allocating library routine, on any call.  Same arguments,
 * same kernels and bit-identical results; R is limited to 65536 rows (the array holds 2 * 65536 / 16 + 2 doubles,
 * 64 KiB, on every GPU the library is used on, until the process ends); a larger R returns TSDP_E_SHAPE.  The
 * context's device must be current.  All calls on one GPU share the array, which keeps the last call's partial
 * sums (every entry a call reads it has written first, so nothing needs clearing): calls that overlap in time on
 * one GPU, from any context or stream, race. */
int tsdp_distill_loss_noalloc(tsdp_ctx* ctx, int R, const int32_t* d_row_t, const float* d_states,
                              const float* d_eps_p, const float* d_eps_q, float lambda1, float lambda2,
                              double* d_loss, void* stream);

/* Synchronises `stream` and returns the device status word accumulated since the last call:
 * bit 0 = some K was outside 0..K_max (clamped), bit 1 = some t0 was >= T (treated as T-1) or a row timestep given to
 * tsdp_verify was outside 0..T-1 (clamped), bit 2 = some running environment had sigma_scale <= 0 or NaN (not
 * corrected: the outputs of that environment are undefined, no memory is touched out of bounds), bit 3 = a row
 * environment index given to tsdp_verify was outside the batch of tsdp_set_cond (clamped). */
int tsdp_status(tsdp_ctx* ctx, void* stream, int32_t* h_status);

/* Measurement aid.  tsdp_kernel_timing(ctx, 1) makes the following calls record a pair of HIP events on the
 * caller's stream around the dominant kernel of each stage (0 = drafter rollout kernel, 1 = verify forward
 * kernel, 2 = acceptance kernel, 3 = the FiLM-vector product that tsdp_verify runs before the forward kernel of a
 * bf16 network with vector conditioning); tsdp_kernel_ms waits for the last such pair of a stage and returns its
 * elapsed time in milliseconds.  enable = 0 switches it off; enable = 2 * mask (mask: bit 0 drafter, bit 1 verify,
 * bit 2 acceptance, bit 3 FiLM product) brackets the chosen stages only -- timing events on the launch stream around
 * the drafter take away part of the overlap a whole round has between the rollout and the FiLM vectors of the base
 * network.  Stages that run as a sequence of operator kernels are not timed. */
int tsdp_kernel_timing(tsdp_ctx* ctx, int enable);
int tsdp_kernel_ms(tsdp_ctx* ctx, int stage, float* h_ms);

/* Name of the kernel path used for a network ("f32-ops", "bf16-mfma-fused", ...). which: 0 base, 1 drafter. */
const char* tsdp_path_name(const tsdp_ctx* ctx, int which);

const char* tsdp_last_error(const tsdp_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* TSDP_H */
