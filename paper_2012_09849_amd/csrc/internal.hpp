// Library-internal declarations shared by the translation units of libhts (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/hts.h"
#include "problems.hpp"
#include "wsgemm.hpp"

namespace hts {

constexpr int NORM_CHUNK = 8192;   // elements per workgroup in the gradient-norm pass (fixes the reduction shape)
constexpr int N_TERMS = 5;         // per-sample loss terms: policy, value, entropy, clipped flag, kl
constexpr int FC_GROUP_K = 512;    // the FC layer's reduction is cut into groups of this many inputs (8 segments of 64)

// Offsets inside Workspace::hb.
struct ShadowOffsets { long long b1, b2, b3, fcb, piw, pib, vw, vb, count; };

struct Workspace {
    void *slab = nullptr;
    size_t bytes = 0;
    // the network as the kernels read it, refreshed from the caller's fp32 vector by launch_prep (T = operand type):
    void *w1s;                // conv1.w [32][(c,u,v)]
    void *wf2, *wf3;          // conv2.w, conv3.w with taps outermost [64][(u,v,c)]
    void *wfc;                // fc.w [512][F]
    void *wd2, *wd3, *wfcd;   // learner only: conv weights for the input gradients; fc.w as [(p,c)][512]
    float *hb;                // fp32 block: biases of all layers and the two heads (offsets in Ctx::sh)
    // forward activations
    void *act1, *act2, *a3;   // T
    void *a3n;                // learner only: conv3 output once more, channel-innermost (ReLU mask of the FC input gradient)
    float *h;                 // learner only: FC output [B][512], written by the heads kernel for the backward pass
    float *fc_part;           // [fc_groups][B][512] partial sums of the FC layer, one per group of FC_GROUP_K inputs
    // backward
    float *dz, *dh, *terms, *grads, *part, *norm_part, *clip;   // clip[0] = scale, clip[1] = ||g||
    float *heads_part;        // [HEADS_MAXZ][A+1][513] partials of the heads weight gradient (large minibatches)
    void *dy3, *dy2, *dy1;    // T
    size_t part_elems;
};

// Launch sites that the built-in event timer can bracket (hts_profile_begin / hts_profile_end).
enum Site {
    SITE_PREP = 0, SITE_CONV1_FWD, SITE_CONV2_FWD, SITE_CONV3_FWD, SITE_FC_FWD, SITE_HEADS_ACT, SITE_HEADS_LEARN,
    SITE_HEADS_WGRAD, SITE_FC_WGRAD, SITE_FC_DGRAD, SITE_CONV3_WGRAD, SITE_CONV3_DGRAD, SITE_CONV2_WGRAD,
    SITE_CONV2_DGRAD, SITE_CONV1_WGRAD, SITE_WGRAD_REDUCE, SITE_GRAD_NORM, SITE_ADAM, SITE_GAE, SITE_NORMALIZE,
    SITE_STATS,
    // the learner's forward pass runs other kernels than an actor call of a few rows: its launches are sites of their own
    SITE_CONV1_FWD_LEARN, SITE_CONV2_FWD_LEARN, SITE_CONV3_FWD_LEARN, SITE_FC_FWD_LEARN, SITE_COUNT
};
constexpr int PROF_CAP = 4096;     // event pairs kept per profiling window

struct Profiler {
    int site = -1, n = 0;
    int every = 1, seen = 0;       // only every `every`-th launch of the site is bracketed; launches of the site seen so far
    hipEvent_t *ev = nullptr;      // 2*PROF_CAP events, created on first use
};

struct Ctx {
    Profiler prof;
    hts_net_desc desc;
    Geom g;
    hipStream_t stream;
    int max_act, max_learn, max_b;
    int small_b;              // batches up to this size take the wave-per-segment forward kernels
    int fc_groups;            // ceil(F / FC_GROUP_K)
    int tile16_below;         // small-batch forward layers with fewer 32x32-tile workgroups than this use 16x16 tiles
    int fc_fold_rows;         // batches of at least this many rows add the FC groups inside the FC kernel (one slice of fc_part)
    int fc_slices;            // slices of fc_part the last forward pass wrote (fc_groups, or 1)
    int conv1_slab_rows;      // bf16 batches of at least this many 16x72x96 or 4x84x84 frames take the slab conv1 kernels
    bool synced;              // the workspace's copy of the network matches the last parameter vector handed in
    bool synced_learn;        // ... including the learner-only parts
    bool track_params;        // the caller modifies its parameter vectors only through this context (hts_track_params)
    const float *shadow_of;   // the caller's vector that the workspace copy mirrors while `synced`
    ShadowOffsets sh;
    Workspace ws;
};

// Brackets the launches of one site with a pair of events on the context's stream while that site is selected.
struct SiteTimer {
    Ctx &c;
    bool on;
    SiteTimer(Ctx &ctx, int site) : c(ctx), on(ctx.prof.site == site && ctx.prof.ev && ctx.prof.n < PROF_CAP)
    {
        if (on) on = (c.prof.seen++ % c.prof.every) == 0;
        if (on) (void)hipEventRecord(c.prof.ev[2 * c.prof.n], c.stream);
    }
    ~SiteTimer()
    {
        if (on) { (void)hipEventRecord(c.prof.ev[2 * c.prof.n + 1], c.stream); ++c.prof.n; }
    }
};

// most chunks a conv weight gradient's reduction is cut into (layers 3, 2, 1)
// (more chunks: more workgroups and shorter serial walks; fewer chunks: less partial-sum traffic for the reduction
// kernel, which is bound by reading it.  Measured at B = 1024 with the chunks placed XCD by XCD: 64 chunks for
// layers 3 and 2 beat 32, 128 and 256; layer 1 -- a tiny output, a long reduction -- keeps 256.)
constexpr int MAXZ3 = 64, MAXZ2 = 64, MAXZ1 = 256;
struct SplitK { int klen, nz; };
// Split of a weight-gradient reduction of length kp; depends on kp only, so results are reproducible.
inline SplitK split_for(long long kp, int maxz)
{
    long long klen = (kp + maxz - 1) / maxz;
    klen = ((klen + 31) / 32) * 32;
    if (klen < 256) klen = 256;
    SplitK s;
    s.klen = (int)klen;
    s.nz = (int)((kp + klen - 1) / klen);
    if (s.nz < 1) s.nz = 1;
    return s;
}

struct LossArgs {
    const int32_t *actions, *index;
    const float *old_logp, *old_values, *adv, *ret;
    int algo;
    float clip_eps, vf_coef, ent_coef;
    float rho_bar, value_clip;        // truncation level of the importance weight; radius of the clipped value loss (<= 0: off)
};

// api.hip: remembers a HIP error code for hts_last_hip_error()
void note_hip_error(hipError_t e);
// fwd.hip
hipError_t run_forward(Ctx &c, const uint8_t *obs, const int32_t *index, int B, bool learn);
hipError_t run_plain_gemm(Ctx &c, int precision, const float *A, const float *B, float *C, int M, int N, int K);
// bwd.hip
hipError_t run_backward(Ctx &c, const uint8_t *obs, const int32_t *index, int B, float *grads);
// misc.hip
hipError_t launch_prep(Ctx &c, const float *params, bool learn);
hipError_t launch_heads_act(Ctx &c, const float *logits_in, uint64_t seed, uint32_t step, int N,
                            int env_offset, int32_t *actions, float *logp, float *values, float *logits_out);
hipError_t launch_heads_learn(Ctx &c, const LossArgs &la, int B);
hipError_t launch_stats(Ctx &c, int B, hts_stats *stats);
struct ReduceSpec {       // one layer's split weight gradient: part[nz][rows][ncol] -> g (see wgrad_reduce_kernel)
    const float *part;
    int nz, rows, ncol, cin, ksz;     // nz = 0: nothing to do
    long long zstride;                // elements between consecutive partials (0: rows * ncol)
    bool taps_outer;
    float scale;
    long long w_off, b_off;
};
constexpr int REDUCE_JOBS = 5;
hipError_t launch_wgrad_reduce(Ctx &c, const ReduceSpec (&spec)[REDUCE_JOBS], float *g);
constexpr int HEADS_MAXZ = 16;      // most chunks the heads weight gradient's reduction over the batch is cut into
hipError_t launch_gae(Ctx *c, hipStream_t s, const float *r, const float *v, const uint8_t *d, float gamma, float lambda, int T,
                      int N, float *adv, float *ret);
hipError_t launch_normalize(Ctx *c, hipStream_t s, float *adv, long long n);
hipError_t launch_grad_norm(Ctx &c, const float *g, long long P, float max_norm, bool finalize);
hipError_t launch_adam(Ctx &c, float *theta, const float *g, float *m, float *v, long long P, const float *scale_or_null,
                       const float *norm_part_or_null, float max_norm, float lr, float b1, float b2, float eps, float bc1,
                       float bc2);
// the same update of the whole network's vector, which also rewrites the workspace copy of the network from the new values
hipError_t launch_adam_shadow(Ctx &c, float *theta, const float *g, float *m, float *v, const float *scale_or_null,
                              const float *norm_part_or_null, float max_norm, float lr, float b1, float b2, float eps,
                              float bc1, float bc2, bool learn);

}  // namespace hts
