/*
 * CPU oracle for the actor / returns / learner path of HTS-RL.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow, by-the-definition
 * implementation that the GPU library is checked against.  It shares no code
 * with the GPU path and must never be called from it; only the test-suite,
 * the smoke check and the benchmark's cpu_baseline leg use it.
 *
 * Arithmetic is double precision throughout, except the categorical sampler,
 * whose decision rule is defined in IEEE binary32 so that every conforming
 * implementation picks the same action (see orc_sample below).
 *
 * What each function follows (High-Throughput Synchronous Deep RL,
 * Liu/Yeh/Schwing, NeurIPS 2020):
 *   orc_forward        network of the appendix "Implementation Details"
 *                      (conv 32@8x8 s4, conv 64@4x4 s2, conv 64@3x3 s1,
 *                      FC 512, policy head + value head), Sec. 4.1
 *                      "Asynchronous actors and executors" (one batched
 *                      forward pass over all available observations).
 *   orc_sample         Sec. 4.1, same paragraph: the random number that
 *                      travels with each observation seeds the sampling of
 *                      that observation's action.
 *   orc_gae            Sec. 3 "Actor-Critic Algorithms": n-step truncated
 *                      return (lambda = 1); generalised to GAE(gamma,lambda).
 *   orc_loss_grads     Sec. 3 eq. (4) (mini-batch actor-critic estimator with
 *                      entropy bonus) and the squared value loss J_V of the
 *                      "Policy Gradient" paragraph; PPO's clipped surrogate
 *                      for algo = 1; the truncated importance weights of
 *                      the appendix's ablation "Delayed Gradient" for algo = 2.
 *   orc_adam, orc_rmsprop, orc_clip_coef, orc_learner_step, orc_normalize_adv
 *                      the optimiser step applied to the estimator above.
 *
 * Parity pins for every function live in tests/test_oracle_*.py.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_MAX_CONV 4

typedef struct {
    int32_t C, H, W;              /* observation channels / height / width            */
    int32_t nconv;                /* number of conv layers (<= ORC_MAX_CONV)          */
    int32_t cout[ORC_MAX_CONV];   /* filters per layer                                */
    int32_t ksz[ORC_MAX_CONV];    /* square kernel size                               */
    int32_t stride[ORC_MAX_CONV]; /* stride                                           */
    int32_t hidden;               /* width of the fully connected layer               */
    int32_t A;                    /* number of actions                                */
    int32_t operand_bf16;         /* 0: exact operands.  1: model of a reduced-precision matrix path -- EVERY operand of
                                     a matrix product of the conv and FC layers, in the forward and in the backward
                                     pass, is rounded to bfloat16 (round to nearest even) before use: the conv and FC
                                     weights, the outputs of the conv layers (inputs of the next product; pixels are
                                     exact in bfloat16), and in the backward pass the gradients with respect to the
                                     pre-activations of the FC and conv layers (operands of the weight-gradient and
                                     input-gradient products, bias gradients included).  Sums, biases, the FC output,
                                     heads, loss and optimiser stay exact.  Derivatives treat a rounding as the
                                     identity.                                                                        */
    int32_t gates_exact;          /* diagnostic, with operand_bf16 = 1 only: every discontinuous decision of the
                                     derivative -- the ReLU gates, the clipped surrogate's "ratio outside the band"
                                     decision, the branch of the clipped value loss -- is taken from an unrounded
                                     forward pass of the same sample, so that the difference to the unrounded gradient
                                     is the accumulated operand rounding alone and the difference to the
                                     operand_bf16 = 1 gradient is the effect of flipped decisions.                    */
} orc_net;

typedef struct {
    int32_t algo;                 /* 0 = A2C, 1 = PPO, 2 = A2C with truncated importance weights */
    double clip_eps, vf_coef, ent_coef, max_grad_norm;
    double lr, beta1, beta2, adam_eps;
    double rho_bar;               /* algo 2: truncation level of the importance weight          */
    double value_clip;            /* > 0: clipped value loss around old_values with this radius */
} orc_hparams;

typedef struct {
    double policy_loss, value_loss, entropy, grad_norm, clip_frac, approx_kl, total_loss;
} orc_stats;

/* ------------------------------------------------------------------------- */
/* shapes and packing                                                        */
/* ------------------------------------------------------------------------- */

typedef struct {
    int cin[ORC_MAX_CONV], hin[ORC_MAX_CONV], win[ORC_MAX_CONV];
    int hout[ORC_MAX_CONV], wout[ORC_MAX_CONV];
    int64_t w_off[ORC_MAX_CONV], b_off[ORC_MAX_CONV];
    int F;
    int64_t fcw, fcb, piw, pib, vw, vb, total;
    int64_t act_off[ORC_MAX_CONV]; /* offset of layer l's output inside a per-sample activation buffer */
    int64_t act_total;
} orc_shape;

static void orc_shapes(const orc_net *n, orc_shape *s)
{
    int c = n->C, h = n->H, w = n->W;
    int64_t off = 0, aoff = 0;
    for (int l = 0; l < n->nconv; ++l) {
        s->cin[l] = c; s->hin[l] = h; s->win[l] = w;
        s->hout[l] = (h - n->ksz[l]) / n->stride[l] + 1;
        s->wout[l] = (w - n->ksz[l]) / n->stride[l] + 1;
        s->w_off[l] = off; off += (int64_t)n->cout[l] * c * n->ksz[l] * n->ksz[l];
        s->b_off[l] = off; off += n->cout[l];
        c = n->cout[l]; h = s->hout[l]; w = s->wout[l];
        s->act_off[l] = aoff; aoff += (int64_t)c * h * w;
    }
    s->act_total = aoff;
    s->F = c * h * w;
    s->fcw = off; off += (int64_t)n->hidden * s->F;
    s->fcb = off; off += n->hidden;
    s->piw = off; off += (int64_t)n->A * n->hidden;
    s->pib = off; off += n->A;
    s->vw = off;  off += n->hidden;
    s->vb = off;  off += 1;
    s->total = off;
}

/* Round a double to the nearest bfloat16 value (8 significant bits, binary32 exponent range), ties to even.
 * Done on the binary32 bit pattern: keep the top 16 bits, round on the dropped 16. */
double orc_round_bf16(double x)
{
    union { float f; uint32_t u; } c;
    c.f = (float)x;
    if ((c.u & 0x7F800000u) == 0x7F800000u) return (double)c.f;       /* inf / nan unchanged */
    const uint32_t low = c.u & 0xFFFFu, keep = c.u >> 16;
    uint32_t r = keep;
    if (low > 0x8000u || (low == 0x8000u && (keep & 1u))) r = keep + 1u;
    c.u = r << 16;
    return (double)c.f;
}

/* Copy of the parameters as the forward/backward passes use them (see orc_net.operand_bf16). */
static double *operand_params(const orc_net *n, const orc_shape *s, const double *params)
{
    double *q = malloc(sizeof(double) * (size_t)s->total);
    if (!q) return NULL;
    memcpy(q, params, sizeof(double) * (size_t)s->total);
    if (n->operand_bf16) {
        for (int l = 0; l < n->nconv; ++l)
            for (int64_t i = s->w_off[l]; i < s->b_off[l]; ++i) q[i] = orc_round_bf16(q[i]);
        for (int64_t i = s->fcw; i < s->fcb; ++i) q[i] = orc_round_bf16(q[i]);
    }
    return q;
}

int64_t orc_param_count(const orc_net *n)
{
    orc_shape s; orc_shapes(n, &s); return s.total;
}

/* ------------------------------------------------------------------------- */
/* forward for one sample, keeping every layer's output                      */
/* ------------------------------------------------------------------------- */

/* x: [C*H*W] normalised input; act: per-layer post-ReLU outputs (ReLU output > 0 iff pre-activation > 0);
 * h: [hidden] post-ReLU; logits [A]; value scalar. */
static void forward_one(const orc_net *n, const orc_shape *s, const double *p, const uint8_t *obs,
                        double *x, double *act, double *h, double *logits, double *value)
{
    const int in_sz = n->C * n->H * n->W;
    for (int i = 0; i < in_sz; ++i) x[i] = (double)obs[i] / 255.0;

    const double *in = x;
    for (int l = 0; l < n->nconv; ++l) {
        const int ci = s->cin[l], hi = s->hin[l], wi = s->win[l];
        const int co = n->cout[l], k = n->ksz[l], st = n->stride[l];
        const int ho = s->hout[l], wo = s->wout[l];
        const double *wgt = p + s->w_off[l], *bias = p + s->b_off[l];
        double *out = act + s->act_off[l];
        for (int o = 0; o < co; ++o)
            for (int i = 0; i < ho; ++i)
                for (int j = 0; j < wo; ++j) {
                    double acc = bias[o];
                    for (int c = 0; c < ci; ++c)
                        for (int u = 0; u < k; ++u)
                            for (int v = 0; v < k; ++v)
                                acc += wgt[((o * ci + c) * k + u) * k + v] *
                                       in[(c * hi + (i * st + u)) * wi + (j * st + v)];
                    const double y = acc > 0.0 ? acc : 0.0;
                    out[(o * ho + i) * wo + j] = n->operand_bf16 ? orc_round_bf16(y) : y;
                }
        in = out;
    }
    /* flatten in (c, y, x) order == memory order of the last conv output */
    for (int j = 0; j < n->hidden; ++j) {
        double acc = p[s->fcb + j];
        const double *wr = p + s->fcw + (int64_t)j * s->F;
        for (int f = 0; f < s->F; ++f) acc += wr[f] * in[f];
        h[j] = acc > 0.0 ? acc : 0.0;
    }
    for (int a = 0; a < n->A; ++a) {
        double acc = p[s->pib + a];
        const double *wr = p + s->piw + (int64_t)a * n->hidden;
        for (int j = 0; j < n->hidden; ++j) acc += wr[j] * h[j];
        logits[a] = acc;
    }
    double acc = p[s->vb];
    for (int j = 0; j < n->hidden; ++j) acc += p[s->vw + j] * h[j];
    *value = acc;
}

/* Batched inference: logits [B,A], values [B].  obs is [count, C,H,W]; row b uses obs[index ? index[b] : b]. */
int32_t orc_forward(const orc_net *n, const double *params, const uint8_t *obs, const int32_t *index, int32_t B,
                    double *logits, double *values)
{
    orc_shape s; orc_shapes(n, &s);
    const int in_sz = n->C * n->H * n->W;
    double *x = malloc(sizeof(double) * in_sz), *act = malloc(sizeof(double) * s.act_total),
           *h = malloc(sizeof(double) * n->hidden), *pq = operand_params(n, &s, params);
    if (!x || !act || !h || !pq) return -1;
    for (int b = 0; b < B; ++b) {
        const int64_t row = index ? index[b] : b;
        forward_one(n, &s, pq, obs + row * in_sz, x, act, h, logits + (int64_t)b * n->A, values + b);
    }
    free(x); free(act); free(h); free(pq);
    return 0;
}

/* ------------------------------------------------------------------------- */
/* counter-based random numbers: Philox4x32-10 (Salmon et al., SC'11)        */
/* ------------------------------------------------------------------------- */

void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n1 = (uint32_t)p1;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        const uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Uniform in [0,1) for (seed, environment, step): the top 24 bits of word 0 of
 * Philox(key = seed lo/hi, counter = (env, step, 0, 0)), times 2^-24 (exact in binary32). */
float orc_uniform(uint64_t seed, uint32_t env, uint32_t step)
{
    const uint32_t ctr[4] = { env, step, 0u, 0u };
    const uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t w[4];
    orc_philox4x32_10(ctr, key, w);
    return (float)(w[0] >> 8) * 5.9604644775390625e-08f;
}

/* ------------------------------------------------------------------------- */
/* the sampler's binary32 exponential                                        */
/* ------------------------------------------------------------------------- */

/* exp(x) for x <= 0, defined as a fixed sequence of correctly rounded binary32 operations:
 *   x < -87            -> 0
 *   n  = rint(x * log2e)                       (one multiply, round to nearest even integer)
 *   r  = fma(n, -ln2_hi, x); r = fma(n, -ln2_lo, r)
 *   q  = Horner with fma of 1 + r + r^2/2 + ... + r^6/720
 *   result = q * 2^n                           (exact scaling, result stays normal)
 * Any platform that evaluates these steps in IEEE binary32 gets identical bits. */
float orc_expf(float x)
{
    if (x < -87.0f) return 0.0f;
    volatile float t = x * 1.44269504088896340736f;
    const float n = rintf(t);
    float r = fmaf(n, -0.693145751953125f, x);
    r = fmaf(n, -1.42860682030941723212e-6f, r);
    float q = 1.0f / 720.0f;
    q = fmaf(q, r, 1.0f / 120.0f);
    q = fmaf(q, r, 1.0f / 24.0f);
    q = fmaf(q, r, 1.0f / 6.0f);
    q = fmaf(q, r, 0.5f);
    q = fmaf(q, r, 1.0f);
    q = fmaf(q, r, 1.0f);
    union { uint32_t u; float f; } s;
    s.u = (uint32_t)((int32_t)n + 127) << 23;
    volatile float res = q * s.f;
    return res;
}

/* Seeded categorical sampling from fp32 logits [N,A].
 * Decision rule (all binary32, sequential, no reassociation):
 *   m = max_j l_j;  e_j = orc_expf(l_j - m);  c_j = c_{j-1} + e_j (j ascending);
 *   thr = u * c_{A-1};  action = smallest j with c_j > thr, else A-1.
 * logp = (l_a - m) - log(c_{A-1}) is reported in double-rounded-to-float and compared with a tolerance. */
int32_t orc_sample(const float *logits, int32_t N, int32_t A, uint64_t seed, uint32_t step, int32_t env_offset,
                   int32_t *actions, float *logp, float *u_out)
{
    float *c = malloc(sizeof(float) * (size_t)A);
    if (!c) return -1;
    for (int i = 0; i < N; ++i) {
        const float *l = logits + (int64_t)i * A;
        float m = l[0];
        for (int j = 1; j < A; ++j) if (l[j] > m) m = l[j];
        volatile float run = 0.0f;
        for (int j = 0; j < A; ++j) {
            volatile float d = l[j] - m;
            run = run + orc_expf(d);
            c[j] = run;
        }
        const float u = orc_uniform(seed, (uint32_t)(env_offset + i), step);
        volatile float thr = u * c[A - 1];
        int a = A - 1;
        for (int j = 0; j < A; ++j) if (c[j] > thr) { a = j; break; }
        actions[i] = a;
        if (logp) logp[i] = (float)(((double)l[a] - (double)m) - log((double)c[A - 1]));
        if (u_out) u_out[i] = u;
    }
    free(c);
    return 0;
}

/* ------------------------------------------------------------------------- */
/* returns / advantages                                                      */
/* ------------------------------------------------------------------------- */

/* rewards [T,N], values [T+1,N] (row T = bootstrap value), dones [T,N] (1 = the action at t ended the episode).
 *   delta_t = r_t + gamma (1-d_t) V_{t+1} - V_t
 *   A_t     = delta_t + gamma lambda (1-d_t) A_{t+1},   A_T = 0
 *   R_t     = A_t + V_t
 * With lambda = 1 and no dones R_t is the n-step truncated return of Sec. 3. */
void orc_gae(const double *rewards, const double *values, const uint8_t *dones, double gamma, double lambda,
             int32_t T, int32_t N, double *adv, double *ret)
{
    for (int n = 0; n < N; ++n) {
        double next_adv = 0.0;
        for (int t = T - 1; t >= 0; --t) {
            const double nd = dones[(int64_t)t * N + n] ? 0.0 : 1.0;
            const double delta = rewards[(int64_t)t * N + n] + gamma * nd * values[(int64_t)(t + 1) * N + n]
                                 - values[(int64_t)t * N + n];
            next_adv = delta + gamma * lambda * nd * next_adv;
            adv[(int64_t)t * N + n] = next_adv;
            ret[(int64_t)t * N + n] = next_adv + values[(int64_t)t * N + n];
        }
    }
}

/* (A - mean) / (std + 1e-5), std with the unbiased (n-1) divisor, over all n entries, in place. */
void orc_normalize_adv(double *adv, int64_t n)
{
    double mean = 0.0;
    for (int64_t i = 0; i < n; ++i) mean += adv[i];
    mean /= (double)n;
    double var = 0.0;
    for (int64_t i = 0; i < n; ++i) var += (adv[i] - mean) * (adv[i] - mean);
    var /= (double)(n > 1 ? n - 1 : 1);
    const double sd = sqrt(var);
    for (int64_t i = 0; i < n; ++i) adv[i] = (adv[i] - mean) / (sd + 1e-5);
}

/* ------------------------------------------------------------------------- */
/* loss and its gradient                                                     */
/* ------------------------------------------------------------------------- */

/* Loss over a minibatch of B rows (row b = buffer row index[b], or b when index is NULL):
 *   L = L_pi + vf_coef * mean((R - v)^2) - ent_coef * mean(H)
 *   A2C: L_pi = -mean(logp * adv)                                     [eq. (4), sign flipped: a loss]
 *   PPO: L_pi = -mean(min(rho adv, clip(rho, 1-eps, 1+eps) adv)), rho = exp(logp - old_logp)
 *   truncated importance sampling (one of the two alternatives to the delayed gradient in the appendix's
 *   ablation "Delayed Gradient"; the paper names it without a formula, the usual form is taken):
 *        L_pi = -mean(w logp adv), w = min(rho, rho_bar) held constant in the derivative
 *   value_clip > 0 (old_values required): the value term of a row becomes
 *        max((v - R)^2, (vc - R)^2), vc = old_v + clip(v - old_v, -value_clip, +value_clip)
 * adv and ret are constants.  grads (may be NULL) receives dL/dparams in the packing of params. */
int32_t orc_loss_grads(const orc_net *n, const double *params_in, const uint8_t *obs, const int32_t *index, int32_t B,
                       const int32_t *actions, const double *old_logp, const double *old_values, const double *adv,
                       const double *ret, const orc_hparams *hp, double *grads, orc_stats *stats)
{
    orc_shape s; orc_shapes(n, &s);
    double *params = operand_params(n, &s, params_in);   /* the weights as the passes use them */
    if (!params) return -1;
    const int in_sz = n->C * n->H * n->W;
    const int A = n->A, Hd = n->hidden;
    double *x = malloc(sizeof(double) * in_sz), *act = malloc(sizeof(double) * s.act_total),
           *dact = malloc(sizeof(double) * s.act_total), *h = malloc(sizeof(double) * Hd),
           *dh = malloc(sizeof(double) * Hd), *logits = malloc(sizeof(double) * A),
           *lp = malloc(sizeof(double) * A), *dl = malloc(sizeof(double) * A);
    if (!x || !act || !dact || !h || !dh || !logits || !lp || !dl) return -1;
    /* gates_exact: outputs of an unrounded forward pass, consulted for the ReLU gates only */
    const int exact_gates = n->operand_bf16 && n->gates_exact;
    double *act_g = act, *h_g = h, *logits_g = NULL;
    orc_net plain = *n; plain.operand_bf16 = 0;
    if (exact_gates) {
        act_g = malloc(sizeof(double) * s.act_total); h_g = malloc(sizeof(double) * Hd);
        logits_g = malloc(sizeof(double) * A);
        if (!act_g || !h_g || !logits_g) return -1;
    }
    const int rq = n->operand_bf16;           /* round the backward pass's matrix operands */
    if (grads) memset(grads, 0, sizeof(double) * (size_t)s.total);

    double sum_pi = 0.0, sum_v = 0.0, sum_h = 0.0, sum_clip = 0.0, sum_kl = 0.0;
    const double invB = 1.0 / (double)B;

    for (int b = 0; b < B; ++b) {
        const int64_t row = index ? index[b] : b;
        double v;
        double v_g = 0.0, logp_g = 0.0;       /* gates_exact: value and log-probability of the unrounded pass */
        if (exact_gates) {
            forward_one(&plain, &s, params_in, obs + row * in_sz, x, act_g, h_g, logits_g, &v_g);
            double mg = logits_g[0];
            for (int j = 1; j < A; ++j) if (logits_g[j] > mg) mg = logits_g[j];
            double zg = 0.0;
            for (int j = 0; j < A; ++j) zg += exp(logits_g[j] - mg);
            logp_g = logits_g[actions[row]] - mg - log(zg);
        }
        forward_one(n, &s, params, obs + row * in_sz, x, act, h, logits, &v);

        /* log-softmax, entropy */
        double m = logits[0];
        for (int j = 1; j < A; ++j) if (logits[j] > m) m = logits[j];
        double z = 0.0;
        for (int j = 0; j < A; ++j) z += exp(logits[j] - m);
        const double logz = log(z);
        double ent = 0.0;
        for (int j = 0; j < A; ++j) { lp[j] = logits[j] - m - logz; ent -= exp(lp[j]) * lp[j]; }
        const int a = actions[row];
        const double logp = lp[a], ad = adv[row], R = ret[row];

        double dlogp; /* dL/dlogp */
        if (hp->algo == 0) {
            sum_pi += -logp * ad;
            dlogp = -ad * invB;
        } else if (hp->algo == 2) {
            const double rho = exp(logp - old_logp[row]);
            const double w = rho < hp->rho_bar ? rho : hp->rho_bar;
            sum_pi += -w * logp * ad;
            dlogp = -w * ad * invB;
            sum_clip += rho > hp->rho_bar ? 1.0 : 0.0;
            sum_kl += old_logp[row] - logp;
        } else {
            const double rho = exp(logp - old_logp[row]);
            const double lo = 1.0 - hp->clip_eps, hi = 1.0 + hp->clip_eps;
            const double rc = rho < lo ? lo : (rho > hi ? hi : rho);
            const double s1 = rho * ad, s2 = rc * ad;
            sum_pi += -(s1 < s2 ? s1 : s2);
            /* the surrogate's own gate: with gates_exact it is decided by the unrounded pass's ratio */
            const double rho_d = exact_gates ? exp(logp_g - old_logp[row]) : rho;
            const int clipped = (ad > 0.0 && rho_d > hi) || (ad < 0.0 && rho_d < lo);
            dlogp = clipped ? 0.0 : -ad * rho * invB;
            sum_clip += (rho > hi || rho < lo) ? 1.0 : 0.0;
            sum_kl += old_logp[row] - logp;
        }
        double dv_row = 2.0 * (v - R);             /* d(value term of this row)/dv */
        double v_term = (R - v) * (R - v);
        if (hp->value_clip > 0.0) {
            const double d = v - old_values[row];
            const double dc = d < -hp->value_clip ? -hp->value_clip : (d > hp->value_clip ? hp->value_clip : d);
            const double vc = old_values[row] + dc;
            const double c_term = (vc - R) * (vc - R);
            int take_clipped = c_term > v_term, inside = dc == d;
            if (exact_gates) {                     /* both decisions from the unrounded pass's value */
                const double dg = v_g - old_values[row];
                const double dcg = dg < -hp->value_clip ? -hp->value_clip : (dg > hp->value_clip ? hp->value_clip : dg);
                const double vcg = old_values[row] + dcg;
                take_clipped = (vcg - R) * (vcg - R) > (R - v_g) * (R - v_g);
                inside = dcg == dg;
            }
            if (take_clipped) {
                v_term = c_term;
                dv_row = inside ? 2.0 * (vc - R) : 0.0;      /* the clipped value does not move with v */
            }
        }
        sum_v += v_term;
        sum_h += ent;
        if (!grads) continue;

        for (int j = 0; j < A; ++j) {
            const double pj = exp(lp[j]);
            dl[j] = dlogp * ((j == a ? 1.0 : 0.0) - pj) + hp->ent_coef * invB * pj * (lp[j] + ent);
        }
        const double dv = hp->vf_coef * dv_row * invB;

        /* heads */
        for (int j = 0; j < Hd; ++j) dh[j] = 0.0;
        for (int k = 0; k < A; ++k) {
            grads[s.pib + k] += dl[k];
            for (int j = 0; j < Hd; ++j) {
                grads[s.piw + (int64_t)k * Hd + j] += dl[k] * h[j];
                dh[j] += dl[k] * params[s.piw + (int64_t)k * Hd + j];
            }
        }
        grads[s.vb] += dv;
        for (int j = 0; j < Hd; ++j) {
            grads[s.vw + j] += dv * h[j];
            dh[j] += dv * params[s.vw + j];
        }
        /* fully connected layer */
        const int L = n->nconv;
        const double *fin = L > 0 ? act + s.act_off[L - 1] : x;
        double *dfin = L > 0 ? dact + s.act_off[L - 1] : NULL;
        if (dfin) for (int f = 0; f < s.F; ++f) dfin[f] = 0.0;
        for (int j = 0; j < Hd; ++j) {
            if (!(h_g[j] > 0.0)) continue;        /* ReLU gate: pre-activation > 0 */
            const double g = rq ? orc_round_bf16(dh[j]) : dh[j];
            grads[s.fcb + j] += g;
            for (int f = 0; f < s.F; ++f) {
                grads[s.fcw + (int64_t)j * s.F + f] += g * fin[f];
                if (dfin) dfin[f] += g * params[s.fcw + (int64_t)j * s.F + f];
            }
        }
        /* conv layers, last to first */
        for (int l = L - 1; l >= 0; --l) {
            const int ci = s.cin[l], hi = s.hin[l], wi = s.win[l];
            const int co = n->cout[l], k = n->ksz[l], st = n->stride[l];
            const int ho = s.hout[l], wo = s.wout[l];
            const double *in = l > 0 ? act + s.act_off[l - 1] : x;
            double *din = l > 0 ? dact + s.act_off[l - 1] : NULL;
            const double *out = act_g + s.act_off[l];      /* consulted for the gate only */
            const double *dout = dact + s.act_off[l];
            const double *wgt = params + s.w_off[l];
            if (din) for (int i = 0; i < ci * hi * wi; ++i) din[i] = 0.0;
            for (int o = 0; o < co; ++o)
                for (int i = 0; i < ho; ++i)
                    for (int j = 0; j < wo; ++j) {
                        if (!(out[(o * ho + i) * wo + j] > 0.0)) continue;
                        const double g = rq ? orc_round_bf16(dout[(o * ho + i) * wo + j]) : dout[(o * ho + i) * wo + j];
                        grads[s.b_off[l] + o] += g;
                        for (int c = 0; c < ci; ++c)
                            for (int u = 0; u < k; ++u)
                                for (int v2 = 0; v2 < k; ++v2) {
                                    const int wi_idx = ((o * ci + c) * k + u) * k + v2;
                                    const int in_idx = (c * hi + (i * st + u)) * wi + (j * st + v2);
                                    grads[s.w_off[l] + wi_idx] += g * in[in_idx];
                                    if (din) din[in_idx] += g * wgt[wi_idx];
                                }
                    }
        }
    }
    if (stats) {
        stats->policy_loss = sum_pi * invB;
        stats->value_loss = sum_v * invB;
        stats->entropy = sum_h * invB;
        stats->clip_frac = sum_clip * invB;
        stats->approx_kl = sum_kl * invB;
        stats->total_loss = stats->policy_loss + hp->vf_coef * stats->value_loss - hp->ent_coef * stats->entropy;
        double ss = 0.0;
        if (grads) for (int64_t i = 0; i < s.total; ++i) ss += grads[i] * grads[i];
        stats->grad_norm = sqrt(ss);
    }
    if (exact_gates) { free(act_g); free(h_g); free(logits_g); }
    free(x); free(act); free(dact); free(h); free(dh); free(logits); free(lp); free(dl); free(params);
    return 0;
}

/* The same loss and gradient with the rows spread over host threads (used for full-size minibatches and for the
 * all-core timing).  The B rows are cut into `nslots` contiguous slots (a fixed number: the result does not depend on
 * the thread count); every slot is a plain orc_loss_grads call on its rows, and the slot results -- each a mean over
 * its own rows -- are combined in slot order with weights B_slot / B.  Needs nslots gradient buffers. */
int32_t orc_loss_grads_mt(const orc_net *n, const double *params, const uint8_t *obs, const int32_t *index, int32_t B,
                          const int32_t *actions, const double *old_logp, const double *old_values, const double *adv,
                          const double *ret, const orc_hparams *hp, double *grads, orc_stats *stats, int32_t nslots,
                          int32_t nthreads)
{
    if (nslots > B) nslots = B;
    if (nslots < 1) nslots = 1;
    const int64_t P = orc_param_count(n);
    int32_t *rows = malloc(sizeof(int32_t) * (size_t)B);
    double *gs = grads ? malloc(sizeof(double) * (size_t)P * (size_t)nslots) : NULL;
    orc_stats *ss = malloc(sizeof(orc_stats) * (size_t)nslots);
    int32_t *rcs = malloc(sizeof(int32_t) * (size_t)nslots);
    if (!rows || (grads && !gs) || !ss || !rcs) return -1;
    for (int b = 0; b < B; ++b) rows[b] = index ? index[b] : b;
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads > 0 ? nthreads : 1)
    for (int sl = 0; sl < nslots; ++sl) {
        const int b0 = (int)((int64_t)sl * B / nslots), b1 = (int)((int64_t)(sl + 1) * B / nslots);
        rcs[sl] = orc_loss_grads(n, params, obs, rows + b0, b1 - b0, actions, old_logp, old_values, adv, ret, hp,
                                 gs ? gs + (int64_t)sl * P : NULL, &ss[sl]);
    }
    int32_t rc = 0;
    for (int sl = 0; sl < nslots; ++sl) if (rcs[sl] != 0) rc = rcs[sl];
    if (rc == 0) {
        if (grads) memset(grads, 0, sizeof(double) * (size_t)P);
        orc_stats tot; memset(&tot, 0, sizeof tot);
        for (int sl = 0; sl < nslots; ++sl) {
            const int b0 = (int)((int64_t)sl * B / nslots), b1 = (int)((int64_t)(sl + 1) * B / nslots);
            const double w = (double)(b1 - b0) / (double)B;
            if (grads) for (int64_t i = 0; i < P; ++i) grads[i] += w * gs[(int64_t)sl * P + i];
            tot.policy_loss += w * ss[sl].policy_loss; tot.value_loss += w * ss[sl].value_loss;
            tot.entropy += w * ss[sl].entropy; tot.clip_frac += w * ss[sl].clip_frac;
            tot.approx_kl += w * ss[sl].approx_kl;
        }
        tot.total_loss = tot.policy_loss + hp->vf_coef * tot.value_loss - hp->ent_coef * tot.entropy;
        double sq = 0.0;
        if (grads) for (int64_t i = 0; i < P; ++i) sq += grads[i] * grads[i];
        tot.grad_norm = sqrt(sq);
        if (stats) *stats = tot;
    }
    free(rows); free(gs); free(ss); free(rcs);
    return rc;
}

/* orc_forward with the rows spread over host threads (every row is independent): contiguous chunks of rows, each a
 * plain orc_forward call. */
int32_t orc_forward_mt(const orc_net *n, const double *params, const uint8_t *obs, const int32_t *index, int32_t B,
                       double *logits, double *values, int32_t nthreads)
{
    int32_t nchunks = nthreads > 0 ? 4 * nthreads : 1;
    if (nchunks > B) nchunks = B;
    if (nchunks < 1) nchunks = 1;
    int32_t *rows = malloc(sizeof(int32_t) * (size_t)B), *rcs = malloc(sizeof(int32_t) * (size_t)nchunks);
    if (!rows || !rcs) return -1;
    for (int b = 0; b < B; ++b) rows[b] = index ? index[b] : b;
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads > 0 ? nthreads : 1)
    for (int c = 0; c < nchunks; ++c) {
        const int b0 = (int)((int64_t)c * B / nchunks), b1 = (int)((int64_t)(c + 1) * B / nchunks);
        rcs[c] = orc_forward(n, params, obs, rows + b0, b1 - b0, logits + (int64_t)b0 * n->A, values + b0);
    }
    int32_t rc = 0;
    for (int c = 0; c < nchunks; ++c) if (rcs[c] != 0) rc = rcs[c];
    free(rows); free(rcs);
    return rc;
}

/* ------------------------------------------------------------------------- */
/* gradient-norm clip and Adam                                               */
/* ------------------------------------------------------------------------- */

/* s = min(1, c / (||g||_2 + 1e-6)); c <= 0 disables clipping (s = 1). */
double orc_clip_coef(const double *g, int64_t P, double max_norm)
{
    if (!(max_norm > 0.0)) return 1.0;
    double ss = 0.0;
    for (int64_t i = 0; i < P; ++i) ss += g[i] * g[i];
    const double c = max_norm / (sqrt(ss) + 1e-6);
    return c < 1.0 ? c : 1.0;
}

/* One Adam step (Kingma & Ba) on step counter t >= 1; g is multiplied by gscale first.
 *   m <- b1 m + (1-b1) g;  v <- b2 v + (1-b2) g^2
 *   theta <- theta - lr * (m / (1-b1^t)) / (sqrt(v / (1-b2^t)) + eps) */
void orc_adam(double *theta, const double *g, double *m, double *v, int64_t P, int64_t t, double gscale,
              const orc_hparams *hp)
{
    const double bc1 = 1.0 - pow(hp->beta1, (double)t), bc2 = 1.0 - pow(hp->beta2, (double)t);
    for (int64_t i = 0; i < P; ++i) {
        const double gi = g[i] * gscale;
        m[i] = hp->beta1 * m[i] + (1.0 - hp->beta1) * gi;
        v[i] = hp->beta2 * v[i] + (1.0 - hp->beta2) * gi * gi;
        theta[i] -= hp->lr * (m[i] / bc1) / (sqrt(v[i] / bc2) + hp->adam_eps);
    }
}

/* One RMSProp step without momentum (the optimiser of the paper's experiments, appendix "Implementation Details":
 * momentum 0, epsilon 1e-5); g is multiplied by gscale first.
 *   v <- alpha v + (1-alpha) g^2;  theta <- theta - lr * g / (sqrt(v) + eps) */
void orc_rmsprop(double *theta, const double *g, double *v, int64_t P, double gscale, double lr, double alpha,
                 double eps)
{
    for (int64_t i = 0; i < P; ++i) {
        const double gi = g[i] * gscale;
        v[i] = alpha * v[i] + (1.0 - alpha) * gi * gi;
        theta[i] -= lr * gi / (sqrt(v[i]) + eps);
    }
}

/* loss + gradient at params, optional global-norm clip, Adam on params.  t is the 1-based step index. */
int32_t orc_learner_step(const orc_net *n, double *params, double *m, double *v, int64_t t,
                         const uint8_t *obs, const int32_t *index, int32_t B, const int32_t *actions,
                         const double *old_logp, const double *old_values, const double *adv, const double *ret,
                         const orc_hparams *hp, double *grads_out, orc_stats *stats)
{
    const int64_t P = orc_param_count(n);
    double *g = grads_out ? grads_out : malloc(sizeof(double) * (size_t)P);
    if (!g) return -1;
    const int32_t rc = orc_loss_grads(n, params, obs, index, B, actions, old_logp, old_values, adv, ret, hp, g, stats);
    if (rc == 0) {
        const double sc = orc_clip_coef(g, P, hp->max_grad_norm);
        orc_adam(params, g, m, v, P, t, sc, hp);
    }
    if (!grads_out) free(g);
    return rc;
}
