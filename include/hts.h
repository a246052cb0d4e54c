/*
 * hts.h -- C ABI of the GPU-resident hot path of HTS-RL's synchronous actor-learner loop
 * (High-Throughput Synchronous Deep RL, Liu/Yeh/Schwing, NeurIPS 2020) for AMD MI355X (gfx950).
 *
 * Three calls follow the paper's decomposition of one training iteration (Sec. 4.1 "Overview"):
 *   hts_act           what an actor does: one batched forward pass over the observations it grabbed and a
 *                     seeded action sample per observation (Sec. 4.1 "Asynchronous actors and executors");
 *   hts_returns_gae   the returns / advantages over one filled data storage (Sec. 3, n-step truncated return);
 *   hts_learner_step  what a learner does with a storage: forward and backward pass on a minibatch and one
 *                     optimiser step (Sec. 3 eq. (4); Sec. 4.1 "Concurrent rollout and learning").
 *
 * Conventions for every function
 *   - All array arguments are DEVICE pointers owned by the caller (the library never frees or keeps them),
 *     unless the comment says "host".  Structs (hts_net_desc, hts_buffer, hts_hparams, hts_opt_state) are host
 *     structs passed by pointer; the device pointers they hold obey the same rule.
 *   - Work is enqueued on the HIP stream given to hts_create and is NOT synchronised: outputs are valid once the
 *     caller has synchronised that stream.
 *   - Return value: 0 on success, a negative HTS_E* code on failure.  On HTS_EINVAL / HTS_ESHAPE nothing has been
 *     launched.  No C++ types or exceptions cross this boundary.
 *   - Same inputs give bit-identical outputs on every run: no atomics, every reduction has a fixed shape.
 *   - The context owns a device workspace sized at creation (activations, split-K partials, permuted conv
 *     weights); no call after hts_create allocates.  Calls on one context must not overlap in time.
 *
 * Network (appendix "Implementation Details"): conv 32@8x8 stride 4 -> conv 64@4x4 stride 2 -> conv 64@3x3
 * stride 1 -> FC 512 -> {policy head with A logits, value head}; ReLU after each of the four hidden layers; no
 * padding; observations are uint8 NCHW and are scaled by 1/255 inside the first layer.
 *
 * Parameter packing (one flat fp32 vector; gradients and optimiser moments use the same packing):
 *   conv1.w[32,C,8,8] conv1.b[32] conv2.w[64,32,4,4] conv2.b[64] conv3.w[64,64,3,3] conv3.b[64]
 *   fc.w[512,F] fc.b[512] pi.w[A,512] pi.b[A] v.w[512] v.b[1],  F = 64*H3*W3 flattened as (channel, y, x).
 */
#ifndef HTS_H
#define HTS_H
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define HTS_OK      0
#define HTS_EINVAL  (-1)   /* null pointer, non-positive size, misaligned pointer, bad enum            */
#define HTS_ESHAPE  (-2)   /* unsupported C/H/W/A/precision, or a batch larger than the context's max  */
#define HTS_EHIP    (-3)   /* a HIP runtime call failed; hts_last_hip_error() returns its code         */
#define HTS_ENOMEM  (-4)   /* host or device allocation failed in hts_create                           */

#define HTS_PRECISION_FP32 0   /* fp32 operands, fp32 accumulate                                        */
#define HTS_PRECISION_BF16 1   /* bf16 matrix operands, fp32 accumulate, fp32 heads/loss/optimiser      */

#define HTS_ALGO_A2C 0
#define HTS_ALGO_PPO 1
#define HTS_ALGO_A2C_TIS 2   /* actor-critic with truncated importance weights (see hts_hparams) */

#define HTS_MAX_ACTIONS 64

typedef struct hts_ctx hts_ctx;

/* Observation shape [C,H,W] (W must be a multiple of 4; all three conv outputs must be non-empty),
 * number of actions A (1..HTS_MAX_ACTIONS) and arithmetic precision. */
typedef struct { int32_t C, H, W, A; int32_t precision; } hts_net_desc;

/* Number of fp32 parameters for a shape; negative error code if the shape is unsupported.  Host only. */
int64_t hts_param_count(const hts_net_desc *desc);

/* Create a context.  max_act_batch bounds N of hts_act, max_learn_batch bounds B of the learner calls (either may
 * be 0 if that call is unused).  hip_stream is a hipStream_t (NULL = the default stream).  Allocates the device
 * workspace.  *out receives the context, to be released with hts_destroy. */
int32_t hts_create(const hts_net_desc *desc, int32_t max_act_batch, int32_t max_learn_batch, void *hip_stream,
                   hts_ctx **out);
int32_t hts_destroy(hts_ctx *ctx);

/* Actor step (Sec. 4.1 "Asynchronous actors and executors").
 *   obs      u8 [N,C,H,W]    the N observations grabbed in this poll
 *   params   f32 [P] or NULL the behaviour parameters.  Non-NULL: the context first loads them (see hts_sync_params).
 *                            NULL: the parameters loaded by the most recent hts_sync_params / hts_act(params) /
 *                            hts_loss_and_grads on this context are used again -- the paper's actors keep one
 *                            parameter version for a whole storage (Sec. 4.1 "Concurrent rollout and learning"), so
 *                            only the first step of a rollout needs to pass them.  HTS_EINVAL if nothing is loaded,
 *                            or if hts_learner_step / hts_adam_apply ran on this context since the last load (with
 *                            hts_track_params on, an update keeps the loaded copy in step instead, and the call uses
 *                            the updated parameters).
 *   seed, step, env_offset   observation i belongs to environment env_offset+i; its action is drawn with the
 *                            uniform u = top 24 bits of word 0 of Philox4x32-10(key = seed lo/hi,
 *                            counter = (env, step, 0, 0)) * 2^-24, so the action does not depend on which call
 *                            or which batch handles the observation.
 *   actions  i32 [N]   logp f32 [N] (log pi(a|s))   values f32 [N]   logits_or_null f32 [N,A]
 * Sampling rule (binary32, sequential): m = max logits; e_j = hts-exp(l_j - m); c_j = c_{j-1} + e_j;
 * action = first j with c_j > u * c_{A-1}, else A-1. */
int32_t hts_act(hts_ctx *ctx, const uint8_t *obs, const float *params, uint64_t seed, uint32_t step, int32_t N,
                int32_t env_offset, int32_t *actions, float *logp, float *values, float *logits_or_null);

/* Load a parameter vector f32 [P] into the context: the kernels read the network from a copy in the workspace
 * (matrix operands converted to the context's precision and re-ordered for their gathers), refreshed by this call.
 * The copy is what hts_act(params = NULL) uses.  The learner calls always load the vector they are given. */
int32_t hts_sync_params(hts_ctx *ctx, const float *params);

/* on = 1: the caller promises that every parameter vector it hands to this context is modified only by this context's
 * learner calls (hts_learner_step, hts_learner_step_delayed, hts_adam_apply on the whole vector) -- or that it calls
 * hts_sync_params after writing the vector itself.  The optimiser kernel then rewrites the context's copy of the network
 * (see hts_sync_params) from the values it has just computed, and a following hts_act / learner call that is handed the
 * same vector skips the load: one pass over all parameters less per update and per rollout.  Results are bit-identical
 * with and without.  on = 0 (the default): every call that is handed a vector loads it.  Either way the call forgets
 * what is loaded.  In the paper's terms: the learner owns the parameters, the actors only read them (Sec. 4.1). */
int32_t hts_track_params(hts_ctx *ctx, int32_t on);

/* The sampling stage of hts_act alone, on caller-supplied logits f32 [N,A] (test hook for bit-exact parity). */
int32_t hts_sample_from_logits(hts_ctx *ctx, const float *logits, uint64_t seed, uint32_t step, int32_t N,
                               int32_t env_offset, int32_t *actions, float *logp);

/* Returns / advantages over one storage (Sec. 3 "Actor-Critic Algorithms"; lambda = 1 gives the n-step return).
 *   rewards f32 [T,N]   values f32 [T+1,N] (row T = value of the state after the last step)
 *   dones u8 [T,N] (1 = the action at step t ended the episode)
 *   delta_t = r_t + gamma (1-d_t) V_{t+1} - V_t;  A_t = delta_t + gamma lambda (1-d_t) A_{t+1}, A_T = 0;
 *   advantages f32 [T,N] = A;   returns f32 [T,N] = A + V.   ctx may be NULL only if stream 0 is intended. */
int32_t hts_returns_gae(hts_ctx *ctx, const float *rewards, const float *values, const uint8_t *dones, float gamma,
                        float lambda, int32_t T, int32_t N, float *advantages, float *returns);

/* In-place (A - mean) / (std + 1e-5) over n entries, std with the n-1 divisor; fixed-shape reduction. */
int32_t hts_normalize_advantages(hts_ctx *ctx, float *adv, int64_t n);

/* One storage as the learner reads it: `count` rows (= T*N, time-major), of which the minibatch is the B rows
 * index[0..B) (NULL = rows 0..B-1).  old_values is read only when hts_hparams.value_clip > 0 and may be NULL otherwise. */
typedef struct {
    const uint8_t *obs;        /* u8 [count,C,H,W] */
    const int32_t *actions;    /* i32 [count]      */
    const float   *old_logp;   /* f32 [count]  log-prob under the behaviour policy (PPO, A2C_TIS; may be NULL for A2C) */
    const float   *old_values; /* f32 [count]  value estimates stored at collection time (value_clip > 0 only)         */
    const float   *advantages; /* f32 [count]  treated as constants                                           */
    const float   *returns;    /* f32 [count]                                                                 */
    int32_t        count;
    const int32_t *index;      /* i32 [B] or NULL */
    int32_t        B;
} hts_buffer;

/* Loss (Sec. 3 eq. (4) as a loss to minimise, plus the squared value loss, no 1/2 factor):
 *   L = L_pi + vf_coef * mean((R - v)^2) - ent_coef * mean(H(pi(.|s)))
 *   A2C: L_pi = -mean(logp * adv);  PPO: L_pi = -mean(min(rho adv, clip(rho, 1-eps, 1+eps) adv)),
 *   rho = exp(logp - old_logp).   max_grad_norm > 0: gradients are scaled by min(1, c / (||g||_2 + 1e-6)).
 *   A2C_TIS (the appendix's ablation "Delayed Gradient" compares the one-step-delayed update with truncated importance
 *     sampling and with no correction; the paper gives no formula, the usual truncated weight is taken):
 *     L_pi = -mean(w logp adv), w = min(rho, rho_bar) held constant in the derivative.  "No correction" is HTS_ALGO_A2C
 *     called with the current parameters on a storage collected with the previous ones.
 *   value_clip > 0 (needs hts_buffer.old_values; the clipped value loss of the PPO code the paper's experiments build
 *     on): a row's value term is max((v - R)^2, (vc - R)^2), vc = old_v + clip(v - old_v, -value_clip, +value_clip).
 *   Statistics: clip_frac = share of rows with rho outside [1-eps, 1+eps] (PPO) or above rho_bar (A2C_TIS);
 *     approx_kl = mean(old_logp - logp).
 *   optimizer = HTS_OPT_ADAM:
 *     m <- b1 m + (1-b1) g; v <- b2 v + (1-b2) g^2; theta <- theta - lr (m/(1-b1^t)) / (sqrt(v/(1-b2^t)) + eps).
 *   optimizer = HTS_OPT_RMSPROP (the optimiser of the paper's experiments, appendix "Implementation Details":
 *     momentum 0, epsilon 1e-5; the decay constant is not given there, 0.99 is the usual choice):
 *     v <- alpha v + (1-alpha) g^2; theta <- theta - lr g / (sqrt(v) + eps), eps = adam_eps, alpha = rms_alpha;
 *     hts_opt_state.m is overwritten with the clipped gradient. */
#define HTS_OPT_ADAM    0
#define HTS_OPT_RMSPROP 1
typedef struct {
    int32_t algo;
    float clip_eps, vf_coef, ent_coef, max_grad_norm;
    float lr, beta1, beta2, adam_eps;
    int32_t optimizer;
    float rms_alpha;
    float rho_bar;       /* A2C_TIS: truncation level of the importance weight (> 0; 1 is the usual choice) */
    float value_clip;    /* <= 0: plain squared value loss */
} hts_hparams;

/* Optimiser state: m, v device f32 [P]; step is a host counter of completed updates (the call uses t = step+1 and
 * increments it). */
typedef struct { float *m; float *v; int64_t step; } hts_opt_state;

/* Device struct written by the learner calls when requested. */
typedef struct {
    float policy_loss, value_loss, entropy, grad_norm, clip_frac, approx_kl;
    int32_t nonfinite;      /* 1 if the loss terms or the gradient norm are not finite */
} hts_stats;

/* One optimisation step on one minibatch: forward, loss, backward, optional clip, Adam on params (in/out). */
int32_t hts_learner_step(hts_ctx *ctx, const hts_buffer *buf, float *params, hts_opt_state *opt,
                         const hts_hparams *hp, hts_stats *stats_or_null);

/* The paper's update rule (Sec. 4.1 "Delayed gradient"): theta_{j+1} = theta_j + eta * grad J(theta_{j-1}; D^{theta_{j-1}}).
 * The storage `buf` was collected with params_behaviour = theta_{j-1}; forward, loss and backward run at theta_{j-1};
 * the clipped gradient goes through the optimiser into params_target = theta_j (in/out), which the forward pass never
 * reads.  With one update per storage this lets the learner work on storage j-1 while the actors fill storage j with
 * theta_j.  params_behaviour and params_target must be different vectors (HTS_EINVAL otherwise); both f32 [P]. */
int32_t hts_learner_step_delayed(hts_ctx *ctx, const hts_buffer *buf, const float *params_behaviour,
                                 float *params_target, hts_opt_state *opt, const hts_hparams *hp,
                                 hts_stats *stats_or_null);

/* The same forward/loss/backward without the update: grads f32 [P] receives dL/dparams (unclipped). */
int32_t hts_loss_and_grads(hts_ctx *ctx, const hts_buffer *buf, const float *params, const hts_hparams *hp,
                           float *grads, hts_stats *stats_or_null);

/* Clip (if hp->max_grad_norm > 0) and Adam alone, on caller-supplied gradients f32 [P]. */
int32_t hts_adam_apply(hts_ctx *ctx, float *params, const float *grads, hts_opt_state *opt, const hts_hparams *hp,
                       int64_t P);

/* Clip + optimiser step for callers that cannot allocate and hold no context: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  The same kernels and the same results as hts_adam_apply, but the
 * scratch memory of the gradient-norm reduction (one partial sum per 8192 parameters) is a static device array of the
 * library instead of a context's workspace: the call allocates nothing, creates nothing and needs no hts_create.
 *   params, grads, opt->m, opt->v   device f32 [P], caller-owned;  hp, opt  host structs as for hts_adam_apply
 *   P           1 .. HTS_STATIC_MAX_PARAMS (HTS_ESHAPE beyond: the static array is sized for that many)
 *   hip_stream  hipStream_t to enqueue on (NULL = the default stream); not synchronised
 * The array belongs to the GPU that is current when the call is made (every GPU has its own copy, held until the
 * process ends) and is shared by all calls on that GPU: calls that overlap in time on one GPU race on it -- issue them
 * on one stream, or otherwise order them.  Nothing in it has to be cleared between calls. */
#define HTS_STATIC_MAX_PARAMS 16777216
int32_t hts_adam_apply_static(float *params, const float *grads, hts_opt_state *opt, const hts_hparams *hp, int64_t P,
                              void *hip_stream);

/* Test hook for the tiled matrix-multiply core every layer is built on: C[M,N] = A[M,K] * B[N,K]^T, all f32
 * row-major device arrays; operands are rounded to bf16 first when precision = HTS_PRECISION_BF16.  K % 8 == 0. */
int32_t hts_test_gemm(hts_ctx *ctx, int32_t precision, const float *A, const float *B, float *Cout, int32_t M,
                      int32_t N, int32_t K);

/* Built-in event timer (measurement aid, for callers that need per-kernel times without an external profiler).
 * Launch sites are numbered 0..hts_profile_site_count()-1 and named by hts_profile_site_name (host strings owned by
 * the library).  Between hts_profile_begin(ctx, site) and hts_profile_end every launch of that site is bracketed by
 * a pair of HIP events recorded on the context's stream (at most 4096 launches; later ones are not timed).
 * hts_profile_end waits for the recorded events and returns the number of timed launches and the sum of their
 * durations in milliseconds (host pointers).  Timing does not change any result. */
int32_t     hts_profile_site_count(void);
const char *hts_profile_site_name(int32_t site);
int32_t     hts_profile_begin(hts_ctx *ctx, int32_t site);
/* The same with only every `every`-th launch of the site bracketed (every >= 1): a site with hundreds of short launches
 * per iteration can then be timed inside a throughput measurement without stretching it (a bracket costs the stream
 * about as much as a small kernel). */
int32_t     hts_profile_begin_sampled(hts_ctx *ctx, int32_t site, int32_t every);
int32_t     hts_profile_end(hts_ctx *ctx, int32_t *launches, double *total_ms);
/* Mean elapsed time (ms) of `reps` (1..4096) event pairs with nothing between them: the part of every bracket that
 * the timer itself contributes.  Ends any open profiling window. */
int32_t     hts_profile_overhead(hts_ctx *ctx, int32_t reps, double *mean_ms);

/* A stream whose kernels run on the compute units [first_cu, first_cu + n_cus) only (numbered 0 .. the device's count - 1
 * in the order of the runtime's compute-unit mask), for the concurrent schedule of Sec. 4.1 "Concurrent rollout and
 * learning": the actors' calls on one such stream and the learner's on another, over disjoint ranges, do not wait for each
 * other's workgroups to leave a compute unit.  Results never depend on where a kernel runs.  Default priority.  Every such
 * stream takes one of the process's few hardware queues until hts_stream_destroy.
 *   hip_stream_out   receives a hipStream_t of the current device
 * HTS_EINVAL for a null pointer or a range that is empty or leaves the device; HTS_EHIP if the runtime refuses (on a
 * device of several dies the mask's bits go to the dies in turn and every die must keep a compute unit: ranges whose
 * bounds are multiples of the number of dies, 8 on MI355X, are always accepted). */
int32_t     hts_stream_create_cu_range(int32_t first_cu, int32_t n_cus, void **hip_stream_out);
/* Waits for the stream's work and destroys it (streams made by hts_stream_create_cu_range only). */
int32_t     hts_stream_destroy(void *hip_stream);

int32_t     hts_last_hip_error(void);
const char *hts_strerror(int32_t code);

#ifdef __cplusplus
}
#endif
#endif /* HTS_H */
