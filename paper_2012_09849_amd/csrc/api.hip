// C ABI of libhts: argument checks, context/workspace, and the launch sequence of each call (see include/hts.h).
#include <math.h>
#include <stdlib.h>
#include <new>

#include "internal.hpp"

using namespace hts;

struct hts_ctx { Ctx c; };

static thread_local int32_t g_last_hip = 0;

static int32_t hip_fail(hipError_t e)
{
    g_last_hip = (int32_t)e;
    return HTS_EHIP;
}
void hts::note_hip_error(hipError_t e) { g_last_hip = (int32_t)e; }
#define HIP_TRY(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) return hip_fail(e_); } while (0)

static int32_t make_geom(const hts_net_desc *d, Geom *g)
{
    if (!d) return HTS_EINVAL;
    if (d->C < 1 || d->H < 8 || d->W < 8 || d->A < 1 || d->A > HTS_MAX_ACTIONS) return HTS_ESHAPE;
    if (d->W % 4 != 0) return HTS_ESHAPE;
    if (d->precision != HTS_PRECISION_FP32 && d->precision != HTS_PRECISION_BF16) return HTS_ESHAPE;
    if ((long long)d->C * d->H * d->W > (1ll << 24) || d->C > 1024) return HTS_ESHAPE;
    g->C = d->C; g->H = d->H; g->W = d->W; g->A = d->A;
    g->H1 = (d->H - 8) / 4 + 1; g->W1 = (d->W - 8) / 4 + 1;
    if (g->H1 < 4 || g->W1 < 4) return HTS_ESHAPE;
    g->H2 = (g->H1 - 4) / 2 + 1; g->W2 = (g->W1 - 4) / 2 + 1;
    if (g->H2 < 3 || g->W2 < 3) return HTS_ESHAPE;
    g->H3 = g->H2 - 2; g->W3 = g->W2 - 2;
    g->P1 = g->H1 * g->W1; g->P2 = g->H2 * g->W2; g->P3 = g->H3 * g->W3;
    g->F = 64 * g->P3; g->K1 = d->C * 64;
    long long o = 0;
    g->w1 = o; o += 32ll * g->K1; g->b1 = o; o += 32;
    g->w2 = o; o += 64ll * 512;   g->b2 = o; o += 64;
    g->w3 = o; o += 64ll * 576;   g->b3 = o; o += 64;
    g->fcw = o; o += 512ll * g->F; g->fcb = o; o += 512;
    g->piw = o; o += 512ll * d->A; g->pib = o; o += d->A;
    g->vw = o; o += 512; g->vb = o; o += 1;
    g->P = o;
    return HTS_OK;
}

extern "C" int64_t hts_param_count(const hts_net_desc *desc)
{
    Geom g;
    const int32_t rc = make_geom(desc, &g);
    return rc == HTS_OK ? (int64_t)g.P : (int64_t)rc;
}

extern "C" int32_t hts_last_hip_error(void) { return g_last_hip; }

extern "C" const char *hts_strerror(int32_t code)
{
    switch (code) {
    case HTS_OK: return "ok";
    case HTS_EINVAL: return "invalid argument (null pointer, non-positive size, misaligned pointer or bad enum)";
    case HTS_ESHAPE: return "unsupported shape, precision or batch larger than the context allows";
    case HTS_EHIP: return "HIP runtime error (see hts_last_hip_error)";
    case HTS_ENOMEM: return "allocation failed";
    default: return "unknown error code";
    }
}

namespace {
struct Carver {
    size_t off = 0;
    char *base = nullptr;
    template <typename P> void take(P *&ptr, size_t bytes)
    {
        off = (off + 255) & ~(size_t)255;
        if (base) ptr = reinterpret_cast<P *>(base + off);
        off += bytes;
    }
};

void carve(Ctx &c, Carver &cv)
{
    const Geom &g = c.g;
    Workspace &w = c.ws;
    const size_t ts = c.desc.precision == HTS_PRECISION_BF16 ? 2 : 4;
    const size_t mb = (size_t)c.max_b, ml = (size_t)c.max_learn;
    cv.take(w.w1s, (size_t)32 * g.K1 * ts); cv.take(w.wf2, 64 * 512 * ts); cv.take(w.wf3, 64 * 576 * ts);
    cv.take(w.wfc, (size_t)512 * g.F * ts); cv.take(w.hb, (size_t)c.sh.count * 4);
    cv.take(w.act1, mb * g.P1 * 32 * ts); cv.take(w.act2, mb * g.P2 * 64 * ts); cv.take(w.a3, mb * g.F * ts);
    cv.take(w.fc_part, (size_t)c.fc_groups * mb * 512 * 4);
    cv.take(w.clip, 2 * 4);
    cv.take(w.norm_part, (size_t)((g.P + NORM_CHUNK - 1) / NORM_CHUNK) * 4);
    if (ml > 0) {
        cv.take(w.wd2, 32 * 1024 * ts); cv.take(w.wd3, 64 * 576 * ts); cv.take(w.wfcd, (size_t)512 * g.F * ts);
        cv.take(w.a3n, ml * g.F * ts); cv.take(w.h, ml * 512 * 4);
        cv.take(w.dz, ml * (g.A + 1) * 4); cv.take(w.dh, ml * 512 * 4); cv.take(w.terms, ml * N_TERMS * 4);
        cv.take(w.dy3, ml * g.P3 * 64 * ts); cv.take(w.dy2, ml * g.P2 * 64 * ts); cv.take(w.dy1, ml * g.P1 * 32 * ts);
        cv.take(w.grads, (size_t)g.P * 4);
        // upper bounds of the split counts over every minibatch size B <= max_learn (see split_for)
        auto bound = [](long long kp, int maxz) { const long long n = (kp + 255) / 256; return (size_t)(n < maxz ? n : maxz); };
        w.part_elems = bound((long long)ml * g.P3, MAXZ3) * 64 * 577 + bound((long long)ml * g.P2, MAXZ2) * 64 * 513 +
                       bound((long long)ml * g.P1, MAXZ1) * 32 * (size_t)(g.K1 + 1);
        cv.take(w.part, w.part_elems * 4);
        cv.take(w.heads_part, (size_t)HEADS_MAXZ * (g.A + 1) * 513 * 4);
    }
}
}  // namespace

extern "C" int32_t hts_create(const hts_net_desc *desc, int32_t max_act_batch, int32_t max_learn_batch, void *hip_stream,
                              hts_ctx **out)
{
    if (!desc || !out) return HTS_EINVAL;
    if (max_act_batch < 0 || max_learn_batch < 0 || (max_act_batch == 0 && max_learn_batch == 0)) return HTS_EINVAL;
    if (max_act_batch > (1 << 16) || max_learn_batch > (1 << 16)) return HTS_ESHAPE;
    Geom g;
    const int32_t rc = make_geom(desc, &g);
    if (rc != HTS_OK) return rc;
    hts_ctx *h = new (std::nothrow) hts_ctx();
    if (!h) return HTS_ENOMEM;
    Ctx &c = h->c;
    c.desc = *desc; c.g = g; c.stream = (hipStream_t)hip_stream;
    c.max_act = max_act_batch; c.max_learn = max_learn_batch;
    c.max_b = max_act_batch > max_learn_batch ? max_act_batch : max_learn_batch;
    c.small_b = 128;
    c.fc_groups = (g.F + FC_GROUP_K - 1) / FC_GROUP_K;
    c.synced = false; c.synced_learn = false; c.track_params = false; c.shadow_of = nullptr;
    {
        auto pad4 = [](long long x) { return (x + 3) & ~3ll; };
        ShadowOffsets &s = c.sh;
        s.b1 = 0; s.b2 = 32; s.b3 = 96; s.fcb = 160; s.piw = 672;
        s.pib = s.piw + 512ll * g.A; s.vw = pad4(s.pib + g.A); s.vb = s.vw + 512; s.count = pad4(s.vb + 1);
    }
    if (const char *sb = getenv("HTS_SMALL_BATCH")) c.small_b = atoi(sb);   // tuning knob: 0 disables the small path
    c.fc_fold_rows = 4096; c.fc_slices = c.fc_groups;
    c.tile16_below = 128;
    if (const char *t16 = getenv("HTS_TILE16_BELOW")) c.tile16_below = atoi(t16);   // tuning knob, same bits either way
    if (const char *fr = getenv("HTS_FC_FOLD_ROWS")) c.fc_fold_rows = atoi(fr);   // tuning knob, same bits either way
    c.conv1_slab_rows = 256;
    if (const char *sr = getenv("HTS_CONV1_SLAB_ROWS")) c.conv1_slab_rows = atoi(sr);   // tuning knob, same bits either way
    c.ws = Workspace();
    Carver size_pass;
    carve(c, size_pass);
    c.ws.bytes = size_pass.off + 256;
    const hipError_t e = hipMalloc(&c.ws.slab, c.ws.bytes);
    if (e != hipSuccess) { delete h; g_last_hip = (int32_t)e; return HTS_ENOMEM; }
    Carver place;
    place.base = (char *)c.ws.slab;
    carve(c, place);
    const hipError_t e2 = hipMemsetAsync(c.ws.slab, 0, c.ws.bytes, c.stream);
    if (e2 != hipSuccess) { (void)hipFree(c.ws.slab); delete h; return hip_fail(e2); }
    *out = h;
    return HTS_OK;
}

extern "C" int32_t hts_destroy(hts_ctx *ctx)
{
    if (!ctx) return HTS_EINVAL;
    hipError_t e = hipSuccess;
    if (ctx->c.prof.ev) {
        for (int i = 0; i < 2 * PROF_CAP; ++i) (void)hipEventDestroy(ctx->c.prof.ev[i]);
        delete[] ctx->c.prof.ev;
    }
    if (ctx->c.ws.slab) e = hipFree(ctx->c.ws.slab);
    delete ctx;
    return e == hipSuccess ? HTS_OK : hip_fail(e);
}

extern "C" int32_t hts_act(hts_ctx *ctx, const uint8_t *obs, const float *params, uint64_t seed, uint32_t step, int32_t N,
                           int32_t env_offset, int32_t *actions, float *logp, float *values, float *logits_or_null)
{
    if (!ctx || !obs || !actions || !logp || !values) return HTS_EINVAL;
    if (N <= 0 || env_offset < 0) return HTS_EINVAL;
    if (N > ctx->c.max_act) return HTS_ESHAPE;
    if (((uintptr_t)obs & 3u) || ((uintptr_t)params & 15u)) return HTS_EINVAL;
    Ctx &c = ctx->c;
    if (params) {
        // a vector this context updated itself (and that the caller promised not to touch otherwise) is already loaded
        if (!(c.track_params && c.synced && c.shadow_of == params)) HIP_TRY(launch_prep(c, params, c.track_params && c.max_learn > 0));
    } else if (!c.synced) return HTS_EINVAL;      // no parameters given and none loaded
    HIP_TRY(run_forward(c, obs, nullptr, N, false));
    HIP_TRY(launch_heads_act(c, nullptr, seed, step, N, env_offset, actions, logp, values, logits_or_null));
    return HTS_OK;
}

extern "C" int32_t hts_sync_params(hts_ctx *ctx, const float *params)
{
    if (!ctx || !params) return HTS_EINVAL;
    if ((uintptr_t)params & 15u) return HTS_EINVAL;
    HIP_TRY(launch_prep(ctx->c, params, ctx->c.max_learn > 0));
    return HTS_OK;
}

extern "C" int32_t hts_stream_create_cu_range(int32_t first_cu, int32_t n_cus, void **hip_stream_out)
{
    if (!hip_stream_out || first_cu < 0 || n_cus <= 0) return HTS_EINVAL;
    int dev = 0, cus = 0;
    HIP_TRY(hipGetDevice(&dev));
    HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    if (first_cu > cus - n_cus) return HTS_EINVAL;
    uint32_t mask[32] = {};                                    // one bit per compute unit, up to 1024 of them
    if (cus > 1024) return HTS_ESHAPE;
    for (int i = first_cu; i < first_cu + n_cus; ++i) mask[i >> 5] |= 1u << (i & 31);
    hipStream_t s = nullptr;
    HIP_TRY(hipExtStreamCreateWithCUMask(&s, (uint32_t)((cus + 31) / 32), mask));
    *hip_stream_out = (void *)s;
    return HTS_OK;
}

extern "C" int32_t hts_stream_destroy(void *hip_stream)
{
    if (!hip_stream) return HTS_EINVAL;
    HIP_TRY(hipStreamSynchronize((hipStream_t)hip_stream));
    HIP_TRY(hipStreamDestroy((hipStream_t)hip_stream));
    return HTS_OK;
}

extern "C" int32_t hts_track_params(hts_ctx *ctx, int32_t on)
{
    if (!ctx || (on != 0 && on != 1)) return HTS_EINVAL;
    ctx->c.track_params = on == 1;
    ctx->c.synced = false; ctx->c.synced_learn = false; ctx->c.shadow_of = nullptr;     // start from a fresh load either way
    return HTS_OK;
}

extern "C" int32_t hts_sample_from_logits(hts_ctx *ctx, const float *logits, uint64_t seed, uint32_t step, int32_t N,
                                          int32_t env_offset, int32_t *actions, float *logp)
{
    if (!ctx || !logits || !actions || !logp) return HTS_EINVAL;
    if (N <= 0 || env_offset < 0) return HTS_EINVAL;
    HIP_TRY(launch_heads_act(ctx->c, logits, seed, step, N, env_offset, actions, logp, nullptr, nullptr));
    return HTS_OK;
}

extern "C" int32_t hts_returns_gae(hts_ctx *ctx, const float *rewards, const float *values, const uint8_t *dones,
                                   float gamma, float lambda, int32_t T, int32_t N, float *advantages, float *returns)
{
    if (!rewards || !values || !dones || !advantages || !returns) return HTS_EINVAL;
    if (T <= 0 || N <= 0) return HTS_EINVAL;
    if ((long long)(T + 1) * N >= (1ll << 40)) return HTS_ESHAPE;
    HIP_TRY(launch_gae(ctx ? &ctx->c : nullptr, ctx ? ctx->c.stream : (hipStream_t)0, rewards, values, dones, gamma, lambda, T, N, advantages,
                       returns));
    return HTS_OK;
}

extern "C" int32_t hts_normalize_advantages(hts_ctx *ctx, float *adv, int64_t n)
{
    if (!adv || n <= 0) return HTS_EINVAL;
    HIP_TRY(launch_normalize(ctx ? &ctx->c : nullptr, ctx ? ctx->c.stream : (hipStream_t)0, adv, n));
    return HTS_OK;
}

static int32_t check_learn(hts_ctx *ctx, const hts_buffer *buf, const float *params, const hts_hparams *hp)
{
    if (!ctx || !buf || !params || !hp) return HTS_EINVAL;
    if (!buf->obs || !buf->actions || !buf->advantages || !buf->returns) return HTS_EINVAL;
    if (hp->algo != HTS_ALGO_A2C && hp->algo != HTS_ALGO_PPO && hp->algo != HTS_ALGO_A2C_TIS) return HTS_EINVAL;
    if (hp->optimizer != HTS_OPT_ADAM && hp->optimizer != HTS_OPT_RMSPROP) return HTS_EINVAL;
    if (hp->algo != HTS_ALGO_A2C && !buf->old_logp) return HTS_EINVAL;
    if (hp->algo == HTS_ALGO_A2C_TIS && !(hp->rho_bar > 0.0f)) return HTS_EINVAL;
    if (hp->value_clip > 0.0f && !buf->old_values) return HTS_EINVAL;
    if (buf->B <= 0 || buf->count <= 0) return HTS_EINVAL;
    if (!buf->index && buf->B > buf->count) return HTS_EINVAL;
    if (buf->B > ctx->c.max_learn) return HTS_ESHAPE;
    if (((uintptr_t)buf->obs & 3u) || ((uintptr_t)params & 15u)) return HTS_EINVAL;
    return HTS_OK;
}

static int32_t loss_and_grads(Ctx &c, const hts_buffer *buf, const float *params, const hts_hparams *hp, float *grads)
{
    LossArgs la;
    la.actions = buf->actions; la.index = buf->index; la.old_logp = buf->old_logp;
    la.old_values = buf->old_values; la.adv = buf->advantages; la.ret = buf->returns;
    la.algo = hp->algo; la.clip_eps = hp->clip_eps; la.vf_coef = hp->vf_coef; la.ent_coef = hp->ent_coef;
    la.rho_bar = hp->rho_bar; la.value_clip = hp->value_clip;
    if (!(c.track_params && c.synced_learn && c.shadow_of == params)) HIP_TRY(launch_prep(c, params, true));
    HIP_TRY(run_forward(c, buf->obs, buf->index, buf->B, true));
    HIP_TRY(launch_heads_learn(c, la, buf->B));
    HIP_TRY(run_backward(c, buf->obs, buf->index, buf->B, grads));
    return HTS_OK;
}

extern "C" int32_t hts_loss_and_grads(hts_ctx *ctx, const hts_buffer *buf, const float *params, const hts_hparams *hp,
                                      float *grads, hts_stats *stats_or_null)
{
    const int32_t rc = check_learn(ctx, buf, params, hp);
    if (rc != HTS_OK) return rc;
    if (!grads) return HTS_EINVAL;
    Ctx &c = ctx->c;
    const int32_t rc2 = loss_and_grads(c, buf, params, hp, grads);
    if (rc2 != HTS_OK) return rc2;
    if (stats_or_null) {
        HIP_TRY(launch_grad_norm(c, grads, c.g.P, 0.0f, true));
        HIP_TRY(launch_stats(c, buf->B, stats_or_null));
    }
    return HTS_OK;
}

// have_norm: 0 = nothing computed yet, 1 = the per-chunk sums of squares are in the workspace, 2 = the clip factor too
static int32_t adam_apply(Ctx &c, float *params, const float *grads, hts_opt_state *opt, const hts_hparams *hp,
                          long long P, int have_norm)
{
    const int64_t t = opt->step + 1;
    if (hp->optimizer != HTS_OPT_ADAM && hp->optimizer != HTS_OPT_RMSPROP) return HTS_EINVAL;
    // RMSProp without momentum is the same elementwise update with beta1 = 0 (m = g) and no bias corrections
    const bool rms = hp->optimizer == HTS_OPT_RMSPROP;
    const float b1 = rms ? 0.0f : hp->beta1, b2 = rms ? hp->rms_alpha : hp->beta2;
    const float bc1 = rms ? 1.0f : (float)(1.0 - pow((double)hp->beta1, (double)t));
    const float bc2 = rms ? 1.0f : (float)(1.0 - pow((double)hp->beta2, (double)t));
    const bool clip = hp->max_grad_norm > 0.0f;
    // the optimiser kernel forms the clip factor from the per-chunk sums itself unless it already exists
    if (clip && have_norm == 0) { HIP_TRY(launch_grad_norm(c, grads, P, hp->max_grad_norm, false)); have_norm = 1; }
    const float *scale = clip && have_norm == 2 ? c.ws.clip : nullptr, *parts = clip && have_norm == 1 ? c.ws.norm_part : nullptr;
    if (c.track_params && P == c.g.P) {
        // the optimiser kernel rewrites the workspace copy from the new values: it stays in step with the caller's vector
        HIP_TRY(launch_adam_shadow(c, params, grads, opt->m, opt->v, scale, parts, hp->max_grad_norm, hp->lr, b1, b2,
                                   hp->adam_eps, bc1, bc2, c.max_learn > 0));
    } else {
        HIP_TRY(launch_adam(c, params, grads, opt->m, opt->v, P, scale, parts, hp->max_grad_norm, hp->lr, b1, b2,
                            hp->adam_eps, bc1, bc2));
        c.synced = false; c.synced_learn = false;     // the caller's vector has moved on; the workspace copy has not
    }
    opt->step = t;
    return HTS_OK;
}

static int32_t learner_step(hts_ctx *ctx, const hts_buffer *buf, const float *params_grad, float *params,
                            hts_opt_state *opt, const hts_hparams *hp, hts_stats *stats_or_null)
{
    const int32_t rc = check_learn(ctx, buf, params_grad, hp);
    if (rc != HTS_OK) return rc;
    if (!params || ((uintptr_t)params & 15u)) return HTS_EINVAL;
    if (!opt || !opt->m || !opt->v || opt->step < 0) return HTS_EINVAL;
    Ctx &c = ctx->c;
    const int32_t rc2 = loss_and_grads(c, buf, params_grad, hp, c.ws.grads);
    if (rc2 != HTS_OK) return rc2;
    // statistics need the norm itself; without them the optimiser kernel finishes the clip factor
    const bool need_norm = hp->max_grad_norm > 0.0f || stats_or_null;
    if (need_norm) HIP_TRY(launch_grad_norm(c, c.ws.grads, c.g.P, hp->max_grad_norm, stats_or_null != nullptr));
    if (stats_or_null) HIP_TRY(launch_stats(c, buf->B, stats_or_null));
    return adam_apply(c, params, c.ws.grads, opt, hp, c.g.P, need_norm ? (stats_or_null ? 2 : 1) : 0);
}

extern "C" int32_t hts_learner_step(hts_ctx *ctx, const hts_buffer *buf, float *params, hts_opt_state *opt,
                                    const hts_hparams *hp, hts_stats *stats_or_null)
{
    return learner_step(ctx, buf, params, params, opt, hp, stats_or_null);
}

extern "C" int32_t hts_learner_step_delayed(hts_ctx *ctx, const hts_buffer *buf, const float *params_behaviour,
                                            float *params_target, hts_opt_state *opt, const hts_hparams *hp,
                                            hts_stats *stats_or_null)
{
    if (params_behaviour == params_target) return HTS_EINVAL;     // that is hts_learner_step
    return learner_step(ctx, buf, params_behaviour, params_target, opt, hp, stats_or_null);
}

extern "C" int32_t hts_adam_apply(hts_ctx *ctx, float *params, const float *grads, hts_opt_state *opt,
                                  const hts_hparams *hp, int64_t P)
{
    if (!ctx || !params || !grads || !opt || !opt->m || !opt->v || !hp) return HTS_EINVAL;
    if (P <= 0 || opt->step < 0) return HTS_EINVAL;
    if (P > ctx->c.g.P) return HTS_ESHAPE;       // the norm workspace is sized for the network's parameter count
    return adam_apply(ctx->c, params, grads, opt, hp, P, false);
}

extern "C" int32_t hts_test_gemm(hts_ctx *ctx, int32_t precision, const float *A, const float *B, float *Cout, int32_t M,
                                 int32_t N, int32_t K)
{
    if (!ctx || !A || !B || !Cout) return HTS_EINVAL;
    if (M <= 0 || N <= 0 || K <= 0 || (K % 8) != 0) return HTS_EINVAL;
    if (precision != HTS_PRECISION_FP32 && precision != HTS_PRECISION_BF16) return HTS_EINVAL;
    if (((uintptr_t)A | (uintptr_t)B) & 15u) return HTS_EINVAL;
    HIP_TRY(run_plain_gemm(ctx->c, precision, A, B, Cout, M, N, K));
    return HTS_OK;
}

// ---- built-in event timer -------------------------------------------------------------------------------------
extern "C" int32_t hts_profile_end(hts_ctx *ctx, int32_t *launches, double *total_ms);
static const char *const k_site_names[SITE_COUNT] = {
    "prep", "conv1_fwd", "conv2_fwd", "conv3_fwd", "fc_fwd", "heads_act", "heads_learn", "heads_wgrad", "fc_wgrad",
    "fc_dgrad", "conv3_wgrad", "conv3_dgrad", "conv2_wgrad", "conv2_dgrad", "conv1_wgrad", "wgrad_reduce", "grad_norm",
    "adam", "gae", "normalize", "stats", "conv1_fwd_learn", "conv2_fwd_learn", "conv3_fwd_learn", "fc_fwd_learn"};

extern "C" int32_t hts_profile_site_count(void) { return SITE_COUNT; }

extern "C" const char *hts_profile_site_name(int32_t site)
{
    return (site >= 0 && site < SITE_COUNT) ? k_site_names[site] : "";
}

extern "C" int32_t hts_profile_begin_sampled(hts_ctx *ctx, int32_t site, int32_t every);
extern "C" int32_t hts_profile_begin(hts_ctx *ctx, int32_t site) { return hts_profile_begin_sampled(ctx, site, 1); }

extern "C" int32_t hts_profile_begin_sampled(hts_ctx *ctx, int32_t site, int32_t every)
{
    if (!ctx || site < 0 || site >= SITE_COUNT || every < 1) return HTS_EINVAL;
    Profiler &p = ctx->c.prof;
    if (!p.ev) {
        p.ev = new (std::nothrow) hipEvent_t[2 * PROF_CAP];
        if (!p.ev) return HTS_ENOMEM;
        for (int i = 0; i < 2 * PROF_CAP; ++i) {
            const hipError_t e = hipEventCreate(&p.ev[i]);
            if (e != hipSuccess) {
                for (int k = 0; k < i; ++k) (void)hipEventDestroy(p.ev[k]);
                delete[] p.ev; p.ev = nullptr;
                return hip_fail(e);
            }
        }
    }
    p.site = site; p.n = 0; p.every = every; p.seen = 0;
    return HTS_OK;
}

// Mean elapsed time of an event pair with nothing between them: what the timer itself adds to every bracket.
extern "C" int32_t hts_profile_overhead(hts_ctx *ctx, int32_t reps, double *mean_ms)
{
    if (!ctx || !mean_ms || reps <= 0 || reps > PROF_CAP) return HTS_EINVAL;
    const int32_t rc = hts_profile_begin(ctx, 0);
    if (rc != HTS_OK) return rc;
    Profiler &p = ctx->c.prof;
    for (int i = 0; i < reps; ++i) {
        HIP_TRY(hipEventRecord(p.ev[2 * i], ctx->c.stream));
        HIP_TRY(hipEventRecord(p.ev[2 * i + 1], ctx->c.stream));
    }
    p.n = reps;
    int32_t n = 0;
    double tot = 0.0;
    const int32_t rc2 = hts_profile_end(ctx, &n, &tot);
    if (rc2 != HTS_OK) return rc2;
    *mean_ms = tot / reps;
    return HTS_OK;
}

extern "C" int32_t hts_profile_end(hts_ctx *ctx, int32_t *launches, double *total_ms)
{
    if (!ctx || !launches || !total_ms) return HTS_EINVAL;
    Profiler &p = ctx->c.prof;
    if (p.site < 0 || !p.ev) return HTS_EINVAL;
    double tot = 0.0;
    for (int i = 0; i < p.n; ++i) {
        HIP_TRY(hipEventSynchronize(p.ev[2 * i + 1]));
        float ms = 0.0f;
        HIP_TRY(hipEventElapsedTime(&ms, p.ev[2 * i], p.ev[2 * i + 1]));
        tot += (double)ms;
    }
    *launches = p.n; *total_ms = tot;
    p.site = -1; p.n = 0;
    return HTS_OK;
}
