// Streaming and per-sample kernels: conv-weight permutation, policy/value heads with seeded sampling (actor) or
// loss gradient (learner), split-K combine, returns/GAE, advantage normalisation, gradient norm, Adam.
//
// This file is compiled with floating-point contraction off: the sampler's decision rule is a fixed sequence of
// binary32 operations (see hts_act in hts.h) and must not be re-associated or fused.
#include <math.h>

#include <mutex>

#include "internal.hpp"

#pragma clang fp contract(off)

namespace hts {

// 8 consecutive floats (16-byte aligned) into registers
__device__ __forceinline__ void load_vec(const float *p, float (&v)[8])
{
    const f32x4 t0 = *reinterpret_cast<const f32x4 *>(p), t1 = *reinterpret_cast<const f32x4 *>(p + 4);
#pragma unroll
    for (int i = 0; i < 4; ++i) { v[i] = t0[i]; v[4 + i] = t1[i]; }
}

// ------------------------------------------------------------------------------------------------------------
// The network as the kernels read it: one launch copies the caller's fp32 parameter vector into the workspace,
// converting to the operand type and re-ordering.  Workgroups are assigned to jobs by index range:
//   [0, nb_fc)            64 x 64 tiles of fc.w -> wfc (same order) and, for the learner, wfcd (transposed, rows in
//                         channel-innermost order f' = p*64 + c), through an LDS tile so both sides stay coalesced
//   [nb_fc, +nb_conv)     conv2.w / conv3.w -> wf2, wf3 (taps outermost) and, for the learner, wd2, wd3
//   [.., +nb_w1)          conv1.w -> w1s
//   [.., +nb_hb)          biases and heads -> hb (fp32)
// ------------------------------------------------------------------------------------------------------------
struct PrepArgs {
    const float *params;
    Geom g;
    ShadowOffsets sh;
    void *w1s, *wf2, *wf3, *wfc, *wd2, *wd3, *wfcd;
    float *hb;
    int nb_fc, nb_conv, nb_w1, nb_hb;
    int learn;
};

template <typename T> __global__ __launch_bounds__(256) void prep_kernel(const PrepArgs a)
{
    __shared__ float tile[64][65];
    const int t = threadIdx.x;
    int blk = blockIdx.x;
    const float *__restrict__ params = a.params;
    if (blk < a.nb_fc) {
        const int F = a.g.F, tf = F / 64;
        const int j0 = (blk / tf) * 64, f0 = (blk % tf) * 64;
        const float *src = params + a.g.fcw;
        T *wfc = (T *)a.wfc;
        const int col = t & 63, r0 = t >> 6;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int r = r0 + 4 * i;
            const float v = src[(long long)(j0 + r) * F + f0 + col];
            wfc[(long long)(j0 + r) * F + f0 + col] = from_f32<T>(v);
            tile[r][col] = v;
        }
        if (!a.learn) return;
        __syncthreads();
        T *wfcd = (T *)a.wfcd;
        const int P3 = a.g.P3;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int fl = r0 + 4 * i, f = f0 + fl;
            const int c = f / P3, p = f - c * P3;
            wfcd[(long long)(p * 64 + c) * 512 + j0 + col] = from_f32<T>(tile[col][fl]);
        }
        return;
    }
    blk -= a.nb_fc;
    if (blk < a.nb_conv) {
        const int i = blk * 256 + t;
        T *wf2 = (T *)a.wf2, *wf3 = (T *)a.wf3, *wd2 = (T *)a.wd2, *wd3 = (T *)a.wd3;
        if (i < 64 * 32 * 16) {               // conv2.w[n][c][u][v], 64 x 32 x 4 x 4
            const int n = i / 512, r = i % 512, c = r / 16, tap = r % 16;
            const T w = from_f32<T>(params[a.g.w2 + i]);
            wf2[n * 512 + tap * 32 + c] = w;
            if (a.learn) wd2[c * 1024 + tap * 64 + n] = w;
        }
        if (i < 64 * 64 * 9) {                // conv3.w[n][c][u][v], 64 x 64 x 3 x 3
            const int n = i / 576, r = i % 576, c = r / 9, tap = r % 9;
            const T w = from_f32<T>(params[a.g.w3 + i]);
            wf3[n * 576 + tap * 64 + c] = w;
            if (a.learn) wd3[c * 576 + tap * 64 + n] = w;
        }
        return;
    }
    blk -= a.nb_conv;
    if (blk < a.nb_w1) {
        const int i = blk * 256 + t;
        if (i < 32 * a.g.K1) ((T *)a.w1s)[i] = from_f32<T>(params[a.g.w1 + i]);
        return;
    }
    blk -= a.nb_w1;
    {
        const int i = blk * 256 + t;
        const int A = a.g.A;
        // hb = b1 | b2 | b3 | fc.b | pi.w | pi.b | v.w | v.b, each part starting on a 16-byte boundary
        long long src = -1;
        if (i < 32) src = a.g.b1 + i;
        else if (i >= a.sh.b2 && i < a.sh.b2 + 64) src = a.g.b2 + (i - a.sh.b2);
        else if (i >= a.sh.b3 && i < a.sh.b3 + 64) src = a.g.b3 + (i - a.sh.b3);
        else if (i >= a.sh.fcb && i < a.sh.fcb + 512) src = a.g.fcb + (i - a.sh.fcb);
        else if (i >= a.sh.piw && i < a.sh.piw + 512 * A) src = a.g.piw + (i - a.sh.piw);
        else if (i >= a.sh.pib && i < a.sh.pib + A) src = a.g.pib + (i - a.sh.pib);
        else if (i >= a.sh.vw && i < a.sh.vw + 512) src = a.g.vw + (i - a.sh.vw);
        else if (i == a.sh.vb) src = a.g.vb;
        if (src < 0) return;
        a.hb[i] = params[src];
    }
}

static PrepArgs prep_args(const Ctx &c, const float *params, bool learn)
{
    PrepArgs a;
    a.params = params; a.g = c.g; a.sh = c.sh;
    a.w1s = c.ws.w1s; a.wf2 = c.ws.wf2; a.wf3 = c.ws.wf3; a.wfc = c.ws.wfc;
    a.wd2 = c.ws.wd2; a.wd3 = c.ws.wd3; a.wfcd = c.ws.wfcd; a.hb = c.ws.hb;
    a.nb_fc = (512 / 64) * (c.g.F / 64);
    a.nb_conv = (64 * 64 * 9 + 255) / 256;
    a.nb_w1 = (32 * c.g.K1 + 255) / 256;
    a.nb_hb = (int)((c.sh.count + 255) / 256);
    a.learn = learn ? 1 : 0;
    return a;
}

hipError_t launch_prep(Ctx &c, const float *params, bool learn)
{
    SiteTimer tm(c, SITE_PREP);
    const PrepArgs a = prep_args(c, params, learn);
    const int nb = a.nb_fc + a.nb_conv + a.nb_w1 + a.nb_hb;
    if (c.desc.precision == HTS_PRECISION_BF16)
        hipLaunchKernelGGL(prep_kernel<bf16_t>, dim3(nb), dim3(256), 0, c.stream, a);
    else
        hipLaunchKernelGGL(prep_kernel<float>, dim3(nb), dim3(256), 0, c.stream, a);
    const hipError_t e = hipGetLastError();
    if (e == hipSuccess) { c.synced = true; c.synced_learn = learn; c.shadow_of = params; }
    return e;
}

// ------------------------------------------------------------------------------------------------------------
// counter-based uniform and the sampler's binary32 exponential
// ------------------------------------------------------------------------------------------------------------

// Philox4x32-10 (Salmon et al., SC'11), word 0 only is used by the caller.
__device__ __forceinline__ uint32_t philox_word0(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                                 uint32_t k1)
{
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t h0 = __umulhi(0xD2511F53u, c0), l0 = 0xD2511F53u * c0;
        const uint32_t h1 = __umulhi(0xCD9E8D57u, c2), l1 = 0xCD9E8D57u * c2;
        const uint32_t n0 = h1 ^ c1 ^ k0, n2 = h0 ^ c3 ^ k1;
        c0 = n0; c1 = l1; c2 = n2; c3 = l0;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    return c0;
}

__device__ __forceinline__ float seeded_uniform(uint64_t seed, uint32_t env, uint32_t step)
{
    const uint32_t w = philox_word0(env, step, 0u, 0u, (uint32_t)seed, (uint32_t)(seed >> 32));
    return (float)(w >> 8) * 5.9604644775390625e-08f;     // 24 random bits * 2^-24, exact
}

// exp(x), x <= 0:  0 below -87; n = rint(x*log2e); r = x - n*ln2 (two-constant reduction, fma);
// degree-6 Taylor polynomial by Horner with fma; exact scaling by 2^n.
__device__ __forceinline__ float sampler_exp(float x)
{
    if (x < -87.0f) return 0.0f;
    const float n = rintf(x * 1.44269504088896340736f);
    float r = __builtin_fmaf(n, -0.693145751953125f, x);
    r = __builtin_fmaf(n, -1.42860682030941723212e-6f, r);
    float q = 1.0f / 720.0f;
    q = __builtin_fmaf(q, r, 1.0f / 120.0f);
    q = __builtin_fmaf(q, r, 1.0f / 24.0f);
    q = __builtin_fmaf(q, r, 1.0f / 6.0f);
    q = __builtin_fmaf(q, r, 0.5f);
    q = __builtin_fmaf(q, r, 1.0f);
    q = __builtin_fmaf(q, r, 1.0f);
    const float scale = __uint_as_float((uint32_t)((int)n + 127) << 23);
    return q * scale;
}

__device__ __forceinline__ float wave_sum(float x)
{
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) x += __shfl_xor(x, o, 64);
    return x;
}

// max over the 64 lanes, in every lane (exact whatever the order).  Row shifts inside each row of 16 lanes, then the
// two row broadcasts: six dependent steps instead of one lane read and one comparison per lane.
__device__ __forceinline__ float wave_max(float x)
{
    auto step = [](float v, auto ctrl, auto row_mask) {
        const int moved = __builtin_amdgcn_update_dpp(__float_as_int(-INFINITY), __float_as_int(v), decltype(ctrl)::value,
                                                      decltype(row_mask)::value, 0xF, false);
        return fmaxf(v, __int_as_float(moved));
    };
    using std::integral_constant;
    x = step(x, integral_constant<int, 0x111>{}, integral_constant<int, 0xF>{});     // row_shr:1
    x = step(x, integral_constant<int, 0x112>{}, integral_constant<int, 0xF>{});     // row_shr:2
    x = step(x, integral_constant<int, 0x114>{}, integral_constant<int, 0xF>{});     // row_shr:4
    x = step(x, integral_constant<int, 0x118>{}, integral_constant<int, 0xF>{});     // row_shr:8: lane 15 of a row holds the row's max
    x = step(x, integral_constant<int, 0x142>{}, integral_constant<int, 0xA>{});     // row_bcast:15 into rows 1 and 3
    x = step(x, integral_constant<int, 0x143>{}, integral_constant<int, 0xC>{});     // row_bcast:31 into rows 2 and 3: lane 63 holds the max
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 63));
}

// value of x in lane `src`; src must be the same in every lane (it is read into a scalar register)
__device__ __forceinline__ float lane_value(float x, int src)
{
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), __builtin_amdgcn_readfirstlane(src)));
}

// ------------------------------------------------------------------------------------------------------------
// heads: one wavefront per sample.  Lane j (< A) ends up holding logit j; every lane holds the value.
// ------------------------------------------------------------------------------------------------------------
struct HeadsArgs {
    const float *fc_part;      // h = relu(fc_bias + sum_g fc_part[g][B][512]), groups added in order, is formed here ...
    const float *fc_bias;
    float *h_out;              // ... and written out for the backward pass when not null
    int nseg;                  // number of groups
    const float *wpi, *bpi, *wv, *bv;
    const float *logits_in;    // optional: skip the head product and sample from these
    int B, A;
    // actor outputs
    uint64_t seed; uint32_t step; int env_offset;
    int32_t *actions; float *logp, *values, *logits_out;
    // learner inputs / outputs
    LossArgs la;
    float *dz, *dh, *terms;
    bf16_t *dh16;              // not null: dL/dh is written here in bfloat16 (the operand type of the FC layer's backward
};                             // kernels, which then fetch half the bytes; they rounded it the same way as they loaded it)

template <bool LEARN>
__global__ __launch_bounds__(256) void heads_kernel(const HeadsArgs a)
{
    extern __shared__ float heads_lds[];          // [wavefronts of the workgroup][A][65]
    const int lane = threadIdx.x & 63;
    const int b = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);     // one sample per wavefront
    if (b >= a.B) return;                        // whole wavefront leaves together; no block-level barrier below
    const int A = a.A;

    float hv[8];
    constexpr int HEAD_CHUNK = 20;
    float wv8[8], wrow[HEAD_CHUNK][8];     // value head and (up to) HEAD_CHUNK rows of pi.w: this lane's 8 columns
    float mylogit = 0.0f, value = 0.0f;
    float u01 = 0.0f;          // the sample's uniform: needs nothing from memory, so it is formed while the loads travel
    if constexpr (!LEARN) u01 = seeded_uniform(a.seed, (uint32_t)(a.env_offset + b), a.step);
    if (a.logits_in) {
        if (lane < A) mylogit = a.logits_in[(long long)b * A + lane];
    } else {
        // Everything this wavefront needs from the weights is requested before the FC partial sums are waited for
        // (they are independent): value head, FC bias and the first HEAD_CHUNK rows of pi.w.
        float bv8[8];
        const float head_bias = lane < A ? a.bpi[lane] : 0.0f, value_bias = a.bv[0];
        load_vec(a.wv + lane * 8, wv8);
        load_vec(a.fc_bias + lane * 8, bv8);
#pragma unroll
        for (int q = 0; q < HEAD_CHUNK; ++q)
            if (q < A) load_vec(a.wpi + (long long)q * 512 + lane * 8, wrow[q]);
        {
            // add the FC layer's group sums in group order, then bias + ReLU
#pragma unroll
            for (int i = 0; i < 8; ++i) hv[i] = 0.0f;
            const float *src = a.fc_part + (long long)b * 512 + lane * 8;
            const long long sstride = (long long)a.B * 512;
            for (int s = 0; s < a.nseg; s += 8) {          // eight groups' loads in flight, added in group order
                float pv[8][8];
#pragma unroll
                for (int q = 0; q < 8; ++q)
                    if (s + q < a.nseg) load_vec(src + (s + q) * sstride, pv[q]);
#pragma unroll
                for (int q = 0; q < 8; ++q)
                    if (s + q < a.nseg)
#pragma unroll
                        for (int i = 0; i < 8; ++i) hv[i] += pv[q][i];
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) { const float y = hv[i] + bv8[i]; hv[i] = y > 0.0f ? y : 0.0f; }
            if (a.h_out) {
                f32x4 o0, o1;
#pragma unroll
                for (int i = 0; i < 4; ++i) { o0[i] = hv[i]; o1[i] = hv[4 + i]; }
                f32x4 *dst = reinterpret_cast<f32x4 *>(a.h_out + (long long)b * 512 + lane * 8);
                dst[0] = o0; dst[1] = o1;
            }
        }
        // A dot products of length 512 for the logits: every lane forms its 8-element partial of each, the partials
        // go through this wavefront's LDS panel [A][65] and are added row by row in a fixed order (no barrier is
        // needed because a wavefront's LDS operations execute in order).  The value head is one more dot product,
        // reduced by a butterfly.
        float *panel = heads_lds + (threadIdx.x >> 6) * A * 65;
        {
            float sv = 0.0f;
#pragma unroll
            for (int i = 0; i < 8; ++i) sv = __builtin_fmaf(hv[i], wv8[i], sv);
            value = wave_sum(sv) + value_bias;
        }
        for (int j0 = 0; j0 < A; j0 += HEAD_CHUNK) {
            if (j0 > 0) {
#pragma unroll
                for (int q = 0; q < HEAD_CHUNK; ++q)
                    if (j0 + q < A) load_vec(a.wpi + (long long)(j0 + q) * 512 + lane * 8, wrow[q]);
            }
#pragma unroll
            for (int q = 0; q < HEAD_CHUNK; ++q)
                if (j0 + q < A) {
                    float sj = 0.0f;
#pragma unroll
                    for (int i = 0; i < 8; ++i) sj = __builtin_fmaf(hv[i], wrow[q][i], sj);
                    panel[(j0 + q) * 65 + lane] = sj;
                }
        }
        __builtin_amdgcn_wave_barrier();
        // row sums: with A <= 32 (<= 16) rows, two (four) lanes share a row, each adding a contiguous half (quarter)
        // in lane order; the parts are then added in part order
        const int parts = A <= 16 ? 4 : (A <= 32 ? 2 : 1);
        const int rows_per = 64 / parts, len = 64 / parts;
        const int row = lane & (rows_per - 1), part = lane / rows_per;
        float rowsum = 0.0f;
        if (row < A) {
            const float *rp = panel + row * 65 + part * len;
            for (int t = 0; t < len; t += 16) {
                float tv[16];
#pragma unroll
                for (int u = 0; u < 16; ++u) tv[u] = rp[t + u];
#pragma unroll
                for (int u = 0; u < 16; ++u) rowsum += tv[u];
            }
        }
        float tot = rowsum;
        for (int q = 1; q < parts; ++q) tot += __shfl(rowsum, row + q * rows_per, 64);
        if (lane < A) mylogit = tot + head_bias;
    }

    // A wavefront runs alone on its SIMD here, so every dependent instruction costs its full latency, and the steps over
    // the actions are kept to one instruction each: the maximum by lane shifts (six steps), the running sums by a shift
    // and an add per action; lanes >= A hold neutral values (-inf for the maximum, +0 for the sums).  (Phase stamps:
    // with one lane read and two or three instructions per action 2.3 of the kernel's 9.6 thousand clock ticks were
    // spent here.)
    const float lg = lane < A ? mylogit : -INFINITY;
    const float m = wave_max(lg);

    if constexpr (!LEARN) {
        // binary32 inverse CDF: lane j evaluates e_j once; the running sums c_j are formed sequentially in index order
        // along the lanes; lane j keeps c_j, and the action is the
        // first j with c_j > u * c_{A-1} (A-1 if there is none)
        // (c_j = c_{j-1} + e_j along the lanes: every step each lane takes its left neighbour's value -- lane 0 takes
        // +0 -- and adds its own e_j.  After k steps lanes 0..k hold their c_j and keep it, so A - 1 steps of one
        // instruction give every lane its running sum in index order; lane reads into scalar registers cost three
        // instructions per action.)
        const float ej = lane < A ? sampler_exp(mylogit - m) : 0.0f;
        float mine = ej;
        for (int k = 1; k < A; ++k)
            mine = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(mine), 0x138 /* wave_shr:1 */, 0xF, 0xF, true)) + ej;
        const float total = lane_value(mine, A - 1);
        const float thr = u01 * total;
        const unsigned long long above = __ballot(lane < A && mine > thr);
        const int act = above ? __ffsll((long long)above) - 1 : A - 1;
        const float la = lane_value(mylogit, act);
        if (lane == 0) {
            a.actions[b] = act;
            a.logp[b] = (la - m) - logf(total);
            if (a.values) a.values[b] = value;
        }
        if (a.logits_out && lane < A) a.logits_out[(long long)b * A + lane] = mylogit;
    } else {
        const long long row = a.la.index ? a.la.index[b] : b;
        const float e = lane < A ? expf(mylogit - m) : 0.0f;
        const float lse = m + logf(wave_sum(e));
        const float lsm = lane < A ? mylogit - lse : 0.0f;
        const float p = lane < A ? expf(lsm) : 0.0f;
        const float ent = -wave_sum(p * lsm);
        const int act = a.la.actions[row];
        const float logp = lane_value(lsm, act);
        const float adv = a.la.adv[row], R = a.la.ret[row];
        const float invB = 1.0f / (float)a.B;
        float dlogp, pi_term, clipped = 0.0f, kl = 0.0f;
        if (a.la.algo == HTS_ALGO_A2C) {
            pi_term = -logp * adv;
            dlogp = -adv * invB;
        } else if (a.la.algo == HTS_ALGO_A2C_TIS) {
            // truncated importance weight, a constant in the derivative
            const float old = a.la.old_logp[row];
            const float rho = expf(logp - old);
            const float w = fminf(rho, a.la.rho_bar);
            pi_term = -w * logp * adv;
            dlogp = -w * adv * invB;
            clipped = rho > a.la.rho_bar ? 1.0f : 0.0f;
            kl = old - logp;
        } else {
            const float old = a.la.old_logp[row];
            const float rho = expf(logp - old);
            const float lo = 1.0f - a.la.clip_eps, hi = 1.0f + a.la.clip_eps;
            const float rc = fminf(fmaxf(rho, lo), hi);
            pi_term = -fminf(rho * adv, rc * adv);
            const bool cut = (adv > 0.0f && rho > hi) || (adv < 0.0f && rho < lo);
            dlogp = cut ? 0.0f : -adv * rho * invB;
            clipped = (rho > hi || rho < lo) ? 1.0f : 0.0f;
            kl = old - logp;
        }
        const float dl = lane < A ? dlogp * ((lane == act ? 1.0f : 0.0f) - p) + a.la.ent_coef * invB * p * (lsm + ent)
                                  : 0.0f;
        float v_term = (R - value) * (R - value), dv_row = 2.0f * (value - R);
        if (a.la.value_clip > 0.0f) {
            // clipped value loss: the larger of the plain term and the term of the value held within a radius of
            // the stored estimate; a value held at the radius does not move with the network's output
            const float ov = a.la.old_values[row];
            const float d = value - ov;
            const float dc = fminf(fmaxf(d, -a.la.value_clip), a.la.value_clip);
            const float vc = ov + dc;
            const float c_term = (vc - R) * (vc - R);
            if (c_term > v_term) {
                v_term = c_term;
                dv_row = dc == d ? 2.0f * (vc - R) : 0.0f;
            }
        }
        const float dv = a.la.vf_coef * dv_row * invB;
        if (lane < A) a.dz[(long long)b * (A + 1) + lane] = dl;
        if (lane == 0) {
            a.dz[(long long)b * (A + 1) + A] = dv;
            float *t = a.terms + (long long)b * N_TERMS;
            t[0] = pi_term; t[1] = v_term; t[2] = ent; t[3] = clipped; t[4] = kl;
        }
        // dL/d(FC pre-activation) for this lane's 8 hidden units.  With at most HEAD_CHUNK actions the rows of pi.w are
        // still in the registers the logits were formed from (fetching them a second time was nearly half of what a
        // wavefront pulls through its L1, and that is what bounds this kernel); same products in the same order.
        float acc[8];
        const bool rows_held = !a.logits_in && A <= HEAD_CHUNK;
        if (!rows_held || a.logits_in) load_vec(a.wv + lane * 8, wv8);
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = dv * wv8[i];
        if (rows_held) {
#pragma unroll
            for (int q = 0; q < HEAD_CHUNK; ++q)
                if (q < A) {
                    const float dj = lane_value(dl, q);
#pragma unroll
                    for (int i = 0; i < 8; ++i) acc[i] = __builtin_fmaf(dj, wrow[q][i], acc[i]);
                }
        } else {
            for (int j = 0; j < A; ++j) {
                const float dj = lane_value(dl, j);
                float w8[8];
                load_vec(a.wpi + (long long)j * 512 + lane * 8, w8);
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[i] = __builtin_fmaf(dj, w8[i], acc[i]);
            }
        }
        f32x4 o0, o1;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            o0[i] = hv[i] > 0.0f ? acc[i] : 0.0f;
            o1[i] = hv[4 + i] > 0.0f ? acc[4 + i] : 0.0f;
        }
        if (a.dh16) {
            bf16x8 o;
#pragma unroll
            for (int i = 0; i < 4; ++i) { o[i] = from_f32<bf16_t>(o0[i]); o[4 + i] = from_f32<bf16_t>(o1[i]); }
            *reinterpret_cast<bf16x8 *>(a.dh16 + (long long)b * 512 + lane * 8) = o;
        } else {
            f32x4 *dst = reinterpret_cast<f32x4 *>(a.dh + (long long)b * 512 + lane * 8);
            dst[0] = o0; dst[1] = o1;
        }
    }
}

// Wavefronts per workgroup.  A wavefront fetches about 40 KB (the policy head's weights and its sample's FC partial
// sums); with few samples one wavefront per workgroup spreads those fetches over as many compute units as there are
// samples instead of queueing four wavefronts' worth behind one L1.
static int heads_waves(int rows) { return rows <= 512 ? 1 : 4; }
static size_t heads_lds_bytes(int A, int waves) { return (size_t)waves * A * 65 * sizeof(float); }
static hipError_t raise_lds_limit(const void *fn, size_t bytes)
{
    return hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}

static void heads_network(const Ctx &c, HeadsArgs &a)
{
    const float *hb = c.ws.hb;
    a.wpi = hb + c.sh.piw; a.bpi = hb + c.sh.pib; a.wv = hb + c.sh.vw; a.bv = hb + c.sh.vb;
    a.fc_part = c.ws.fc_part; a.fc_bias = hb + c.sh.fcb; a.nseg = c.fc_slices;
}

// logits_in != null: sample from these logits (no network involved); otherwise finish the forward pass first.
hipError_t launch_heads_act(Ctx &c, const float *logits_in, uint64_t seed, uint32_t step, int N, int env_offset,
                            int32_t *actions, float *logp, float *values, float *logits_out)
{
    SiteTimer tm(c, SITE_HEADS_ACT);
    HeadsArgs a = {};
    a.logits_in = logits_in;
    if (!logits_in) heads_network(c, a);
    a.B = N; a.A = c.g.A;
    a.seed = seed; a.step = step; a.env_offset = env_offset;
    a.actions = actions; a.logp = logp; a.values = values; a.logits_out = logits_out;
    const int wv = heads_waves(N);
    const size_t lds = heads_lds_bytes(c.g.A, wv);
    if (lds > 65536) { const hipError_t e = raise_lds_limit(reinterpret_cast<const void *>(heads_kernel<false>), lds); if (e != hipSuccess) return e; }
    hipLaunchKernelGGL(heads_kernel<false>, dim3((N + wv - 1) / wv), dim3(64 * wv), lds, c.stream, a);
    return hipGetLastError();
}

hipError_t launch_heads_learn(Ctx &c, const LossArgs &la, int B)
{
    SiteTimer tm(c, SITE_HEADS_LEARN);
    HeadsArgs a = {};
    heads_network(c, a);
    a.h_out = c.ws.h;
    a.B = B; a.A = c.g.A;
    a.la = la;
    a.dz = c.ws.dz; a.terms = c.ws.terms;
    if (c.desc.precision == HTS_PRECISION_BF16) a.dh16 = reinterpret_cast<bf16_t *>(c.ws.dh); else a.dh = c.ws.dh;
    const int wv = heads_waves(B);
    const size_t lds = heads_lds_bytes(c.g.A, wv);
    if (lds > 65536) { const hipError_t e = raise_lds_limit(reinterpret_cast<const void *>(heads_kernel<true>), lds); if (e != hipSuccess) return e; }
    hipLaunchKernelGGL(heads_kernel<true>, dim3((B + wv - 1) / wv), dim3(64 * wv), lds, c.stream, a);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------------------
// loss statistics: one workgroup, fixed strided sums then a fixed LDS tree
// ------------------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void stats_kernel(const float *__restrict__ terms, int B, const float *clip,
                                                    hts_stats *stats)
{
    __shared__ float red[N_TERMS][256];
    const int t = threadIdx.x;
    float s[N_TERMS];
#pragma unroll
    for (int i = 0; i < N_TERMS; ++i) s[i] = 0.0f;
    for (int b = t; b < B; b += 256)
#pragma unroll
        for (int i = 0; i < N_TERMS; ++i) s[i] += terms[(long long)b * N_TERMS + i];
#pragma unroll
    for (int i = 0; i < N_TERMS; ++i) red[i][t] = s[i];
    __syncthreads();
    for (int w = 128; w >= 1; w >>= 1) {
        if (t < w)
#pragma unroll
            for (int i = 0; i < N_TERMS; ++i) red[i][t] += red[i][t + w];
        __syncthreads();
    }
    if (t == 0) {
        const float invB = 1.0f / (float)B;
        stats->policy_loss = red[0][0] * invB;
        stats->value_loss = red[1][0] * invB;
        stats->entropy = red[2][0] * invB;
        stats->clip_frac = red[3][0] * invB;
        stats->approx_kl = red[4][0] * invB;
        const float gn = clip ? clip[1] : 0.0f;
        stats->grad_norm = gn;
        const float chk = red[0][0] + red[1][0] + red[2][0] + gn;
        stats->nonfinite = (chk - chk == 0.0f) ? 0 : 1;
    }
}

hipError_t launch_stats(Ctx &c, int B, hts_stats *stats)
{
    SiteTimer tm(c, SITE_STATS);
    hipLaunchKernelGGL(stats_kernel, dim3(1), dim3(256), 0, c.stream, c.ws.terms, B, c.ws.clip, stats);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------------------
// Combine of the split conv weight gradients, all three layers in one launch:
// g[dest(n,kcol)] = scale * sum_z part[z][n][kcol].  A workgroup owns 32 consecutive outputs; its 8 lane groups sum
// 8 contiguous ranges of z (loads in flight eight at a time, added in z order) and the 8 range sums are added in
// range order -- a fixed shape, so the result is reproducible.
// ------------------------------------------------------------------------------------------------------------
struct ReduceJob {
    const float *part;
    int nz, rows, ncol, cin, ksz, taps_outer, first_block;
    long long zstride;
    float scale;
    long long w_off, b_off;
};
struct ReduceArgs { ReduceJob job[REDUCE_JOBS]; float *g; };

__global__ __launch_bounds__(256) void wgrad_reduce_kernel(const ReduceArgs a)
{
    __shared__ float red[8][33];
    const int blk = blockIdx.x;
    int jn = 0;
#pragma unroll
    for (int t = 1; t < REDUCE_JOBS; ++t) jn = blk >= a.job[t].first_block ? t : jn;       // first_block is non-decreasing
    const ReduceJob &jb = a.job[jn];
    const int e = threadIdx.x & 31, q = threadIdx.x >> 5;
    const int n_el = jb.rows * jb.ncol;
    const int i = (blk - jb.first_block) * 32 + e;
    const long long zs = jb.zstride;
    const int chunk = (jb.nz + 7) / 8;
    int z = q * chunk;
    const int z1 = min(jb.nz, z + chunk);
    float s = 0.0f;
    if (i < n_el) {
        const float *src = jb.part + i;
        for (; z + 8 <= z1; z += 8) {
            float v[8];
#pragma unroll
            for (int t = 0; t < 8; ++t) v[t] = src[(z + t) * zs];
#pragma unroll
            for (int t = 0; t < 8; ++t) s += v[t];
        }
        for (; z < z1; ++z) s += src[z * zs];
    }
    red[q][e] = s;
    __syncthreads();
    if (q != 0 || i >= n_el) return;
    float tot = red[0][e];
#pragma unroll
    for (int t = 1; t < 8; ++t) tot += red[t][e];
    tot *= jb.scale;
    const int n = i / jb.ncol, kcol = i - n * jb.ncol;
    const int kc = jb.ncol - 1;
    if (kcol == kc) { a.g[jb.b_off + n] = tot; return; }
    long long dst;
    if (jb.taps_outer) {              // kcol = (tap, c)  ->  w[n][c][tap]
        const int tap = kcol / jb.cin, c = kcol - tap * jb.cin;
        dst = ((long long)n * jb.cin + c) * (jb.ksz * jb.ksz) + tap;
    } else dst = (long long)n * kc + kcol;
    a.g[jb.w_off + dst] = tot;
}

hipError_t launch_wgrad_reduce(Ctx &c, const ReduceSpec (&spec)[REDUCE_JOBS], float *g)
{
    SiteTimer tm(c, SITE_WGRAD_REDUCE);
    ReduceArgs a;
    int blocks = 0;
    for (int j = 0; j < REDUCE_JOBS; ++j) {
        const ReduceSpec &sp = spec[j];
        ReduceJob &jb = a.job[j];
        jb.part = sp.part; jb.nz = sp.nz; jb.rows = sp.rows; jb.ncol = sp.ncol; jb.cin = sp.cin; jb.ksz = sp.ksz;
        jb.taps_outer = sp.taps_outer ? 1 : 0; jb.scale = sp.scale; jb.w_off = sp.w_off; jb.b_off = sp.b_off;
        jb.zstride = sp.zstride ? sp.zstride : (long long)sp.rows * sp.ncol;
        jb.first_block = blocks;
        if (sp.nz > 0) blocks += (sp.rows * sp.ncol + 31) / 32;
    }
    a.g = g;
    hipLaunchKernelGGL(wgrad_reduce_kernel, dim3(blocks), dim3(256), 0, c.stream, a);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------------------
// returns / GAE: one lane per environment column, reverse time; neighbouring lanes read neighbouring columns
// ------------------------------------------------------------------------------------------------------------
constexpr int GAE_U = 8;
// The recurrence runs in double precision inside the lane (inputs and outputs are fp32), so a long unroll does not
// accumulate binary32 rounding: each output is the correctly rounded result of an almost exact recurrence.
__global__ __launch_bounds__(64) void gae_kernel(const float *__restrict__ r, const float *__restrict__ v,
                                                 const uint8_t *__restrict__ d, float gamma, float lambda, int T, int N,
                                                 float *__restrict__ adv, float *__restrict__ ret)
{
    const int n = blockIdx.x * 64 + threadIdx.x;
    if (n >= N) return;
    const double g = (double)gamma, gl = (double)gamma * (double)lambda;
    double a = 0.0;
    double vnext = (double)v[(long long)T * N + n];
    int t = T - 1;
    for (; t >= GAE_U - 1; t -= GAE_U) {
        float rr[GAE_U], vv[GAE_U];
        uint8_t dd[GAE_U];
#pragma unroll
        for (int i = 0; i < GAE_U; ++i) {
            const long long o = (long long)(t - i) * N + n;
            rr[i] = r[o]; vv[i] = v[o]; dd[i] = d[o];
        }
#pragma unroll
        for (int i = 0; i < GAE_U; ++i) {
            const long long o = (long long)(t - i) * N + n;
            const double nd = dd[i] ? 0.0 : 1.0;
            const double delta = (double)rr[i] + g * nd * vnext - (double)vv[i];
            a = delta + gl * nd * a;
            adv[o] = (float)a;
            ret[o] = (float)(a + (double)vv[i]);
            vnext = (double)vv[i];
        }
    }
    for (; t >= 0; --t) {
        const long long o = (long long)t * N + n;
        const double vt = (double)v[o];
        const double nd = d[o] ? 0.0 : 1.0;
        const double delta = (double)r[o] + g * nd * vnext - vt;
        a = delta + gl * nd * a;
        adv[o] = (float)a;
        ret[o] = (float)(a + vt);
        vnext = vt;
    }
}

// Time-chunked form for short-and-narrow storages (few environments): a workgroup owns 32 columns and cuts time into
// TC chunks, one wavefront-row per chunk.  A_t = delta_t + c_t A_{t+1} is affine in the carry entering a chunk, so
// pass 1 reduces every chunk to (S, P) with A_first = S + P * carry, the carries are chained through LDS in chunk
// order, and pass 2 replays each chunk from its true carry and writes the outputs.  Double precision throughout, so
// the result equals the one-lane-per-column recurrence to well below binary32 rounding.
constexpr int GAE_COLS = 32, GAE_MAX_TC = 16;
__global__ __launch_bounds__(GAE_COLS * GAE_MAX_TC) void gae_chunked_kernel(
    const float *__restrict__ r, const float *__restrict__ v, const uint8_t *__restrict__ d, float gamma, float lambda,
    int T, int N, int TC, int L, float *__restrict__ adv, float *__restrict__ ret)
{
    __shared__ double sS[GAE_MAX_TC][GAE_COLS], sP[GAE_MAX_TC][GAE_COLS];
    const int cx = threadIdx.x % GAE_COLS, cc = threadIdx.x / GAE_COLS;
    const int n = blockIdx.x * GAE_COLS + cx;
    const int t0 = cc * L, t1 = min(T, t0 + L);                 // this thread's chunk [t0, t1)
    const bool live = n < N && t0 < t1;
    const double g = (double)gamma, gl = (double)gamma * (double)lambda;
    double S = 0.0, P = 1.0;
    if (live) {
        double vnext = (double)v[(long long)t1 * N + n];
        for (int t = t1 - 1; t >= t0; --t) {
            const long long o = (long long)t * N + n;
            const double vt = (double)v[o], nd = d[o] ? 0.0 : 1.0;
            const double delta = (double)r[o] + g * nd * vnext - vt, ct = gl * nd;
            S = delta + ct * S;
            P = ct * P;
            vnext = vt;
        }
    }
    sS[cc][cx] = S; sP[cc][cx] = P;
    __syncthreads();
    if (!live) return;
    double a = 0.0;                                              // advantage entering this chunk from later times
    for (int q = TC - 1; q > cc; --q) a = sS[q][cx] + sP[q][cx] * a;
    double vnext = (double)v[(long long)t1 * N + n];
    for (int t = t1 - 1; t >= t0; --t) {
        const long long o = (long long)t * N + n;
        const double vt = (double)v[o], nd = d[o] ? 0.0 : 1.0;
        const double delta = (double)r[o] + g * nd * vnext - vt;
        a = delta + gl * nd * a;
        adv[o] = (float)a;
        ret[o] = (float)(a + vt);
        vnext = vt;
    }
}

hipError_t launch_gae(Ctx *c, hipStream_t s, const float *r, const float *v, const uint8_t *d, float gamma, float lambda,
                      int T, int N, float *adv, float *ret)
{
    Ctx dummy;
    SiteTimer tm(c ? *c : dummy, SITE_GAE);
    // enough columns to hide each lane's serial walk behind other wavefronts -> plain kernel; otherwise split time as
    // well (measured at T = 128: 16384 columns 27.7 us plain, 7.9 us chunked; break-even near 65536 columns)
    if ((long long)N >= 65536 || T < 16) {
        hipLaunchKernelGGL(gae_kernel, dim3((N + 63) / 64), dim3(64), 0, s, r, v, d, gamma, lambda, T, N, adv, ret);
    } else {
        int TC = T / 8;                       // chunks of at least 8 steps
        if (TC > GAE_MAX_TC) TC = GAE_MAX_TC;
        if (TC < 2) TC = 2;
        const int L = (T + TC - 1) / TC;
        hipLaunchKernelGGL(gae_chunked_kernel, dim3((N + GAE_COLS - 1) / GAE_COLS), dim3(GAE_COLS * TC), 0, s, r, v, d,
                           gamma, lambda, T, N, TC, L, adv, ret);
    }
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------------------
// advantage normalisation: one workgroup, double-precision fixed-shape sums
// ------------------------------------------------------------------------------------------------------------
__device__ __forceinline__ double block_sum_1024(double x, double *red)
{
    const int t = threadIdx.x;
    red[t] = x;
    __syncthreads();
    for (int w = 512; w >= 1; w >>= 1) {
        if (t < w) red[t] += red[t + w];
        __syncthreads();
    }
    const double s = red[0];
    __syncthreads();
    return s;
}

__global__ __launch_bounds__(1024) void normalize_kernel(float *__restrict__ adv, long long n)
{
    __shared__ double red[1024];
    const int t = threadIdx.x;
    double s = 0.0;
    for (long long i = t; i < n; i += 1024) s += (double)adv[i];
    const double mean = block_sum_1024(s, red) / (double)n;
    double q = 0.0;
    for (long long i = t; i < n; i += 1024) { const double dlt = (double)adv[i] - mean; q += dlt * dlt; }
    const double var = block_sum_1024(q, red) / (double)(n > 1 ? n - 1 : 1);
    const double inv = 1.0 / (sqrt(var) + 1e-5);
    for (long long i = t; i < n; i += 1024) adv[i] = (float)(((double)adv[i] - mean) * inv);
}

hipError_t launch_normalize(Ctx *c, hipStream_t s, float *adv, long long n)
{
    Ctx dummy;
    SiteTimer tm(c ? *c : dummy, SITE_NORMALIZE);
    hipLaunchKernelGGL(normalize_kernel, dim3(1), dim3(1024), 0, s, adv, n);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------------------
// gradient norm: per-chunk sums of squares (fixed chunking), then one workgroup combines them in index order
// ------------------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void sumsq_kernel(const float *__restrict__ g, long long P, float *__restrict__ part)
{
    __shared__ float red[256];
    const int t = threadIdx.x;
    const long long base = (long long)blockIdx.x * NORM_CHUNK;
    float s = 0.0f;
#pragma unroll 4
    for (int i = t; i < NORM_CHUNK; i += 256) {
        const long long o = base + i;
        const float x = o < P ? g[o] : 0.0f;
        s = __builtin_fmaf(x, x, s);
    }
    red[t] = s;
    __syncthreads();
    for (int w = 128; w >= 1; w >>= 1) {
        if (t < w) red[t] += red[t + w];
        __syncthreads();
    }
    if (t == 0) part[blockIdx.x] = red[0];
}

// ||g|| from the per-chunk sums, added in a fixed order by one workgroup of 256 threads (every thread gets the result)
__device__ __forceinline__ float norm_from_parts(const float *__restrict__ part, int nparts, float *red)
{
    const int t = threadIdx.x;
    float s = 0.0f;
    for (int i = t; i < nparts; i += 256) s += part[i];
    red[t] = s;
    __syncthreads();
    for (int w = 128; w >= 1; w >>= 1) {
        if (t < w) red[t] += red[t + w];
        __syncthreads();
    }
    return sqrtf(red[0]);
}
__device__ __forceinline__ float clip_scale(float nrm, float max_norm)
{
    return max_norm > 0.0f ? fminf(1.0f, max_norm / (nrm + 1e-6f)) : 1.0f;
}

__global__ __launch_bounds__(256) void clip_finalize_kernel(const float *__restrict__ part, int nparts, float max_norm,
                                                            float *__restrict__ clip)
{
    __shared__ float red[256];
    const float nrm = norm_from_parts(part, nparts, red);
    if (threadIdx.x == 0) {
        clip[0] = clip_scale(nrm, max_norm);
        clip[1] = nrm;
    }
}

static void enqueue_sumsq(hipStream_t stream, const float *g, long long P, float *norm_part)
{
    const int nparts = (int)((P + NORM_CHUNK - 1) / NORM_CHUNK);
    hipLaunchKernelGGL(sumsq_kernel, dim3(nparts), dim3(256), 0, stream, g, P, norm_part);
}

// finalize = false leaves the per-chunk sums in the workspace for the optimiser kernel, which then forms the norm and the
// clip factor itself (the same additions in the same order, in every workgroup): one launch less per update
hipError_t launch_grad_norm(Ctx &c, const float *g, long long P, float max_norm, bool finalize)
{
    SiteTimer tm(c, SITE_GRAD_NORM);
    const int nparts = (int)((P + NORM_CHUNK - 1) / NORM_CHUNK);
    enqueue_sumsq(c.stream, g, P, c.ws.norm_part);
    if (finalize)
        hipLaunchKernelGGL(clip_finalize_kernel, dim3(1), dim3(256), 0, c.stream, c.ws.norm_part, nparts, max_norm,
                           c.ws.clip);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------------------
// Adam
// ------------------------------------------------------------------------------------------------------------
__device__ __forceinline__ void adam_one(float &th, float g, float &m, float &v, float gs, float lr, float b1, float b2,
                                         float eps, float ibc1, float ibc2)
{
    g *= gs;
    m = b1 * m + (1.0f - b1) * g;
    v = b2 * v + (1.0f - b2) * g * g;
    th = th - lr * (m * ibc1) / (sqrtf(v * ibc2) + eps);
}

template <bool VEC4>
__global__ __launch_bounds__(256) void adam_kernel(float *__restrict__ theta, const float *__restrict__ g,
                                                   float *__restrict__ m, float *__restrict__ v, long long P,
                                                   const float *__restrict__ scale, const float *__restrict__ norm_part,
                                                   int nparts, float max_norm, float lr, float b1, float b2,
                                                   float eps, float ibc1, float ibc2)
{
    // the clip factor: given (scale), or formed here from the per-chunk sums of squares (norm_part), or none
    __shared__ float red[256];
    float gs = 1.0f;
    if (norm_part) gs = clip_scale(norm_from_parts(norm_part, nparts, red), max_norm);
    else if (scale) gs = scale[0];
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    if constexpr (VEC4) {
        const long long o = i * 4;
        if (o + 3 < P) {
            f32x4 th = *reinterpret_cast<f32x4 *>(theta + o);
            const f32x4 gg = *reinterpret_cast<const f32x4 *>(g + o);
            f32x4 mm = *reinterpret_cast<f32x4 *>(m + o), vv = *reinterpret_cast<f32x4 *>(v + o);
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                float a = th[k], b = mm[k], c2 = vv[k];
                adam_one(a, gg[k], b, c2, gs, lr, b1, b2, eps, ibc1, ibc2);
                th[k] = a; mm[k] = b; vv[k] = c2;
            }
            *reinterpret_cast<f32x4 *>(theta + o) = th;
            *reinterpret_cast<f32x4 *>(m + o) = mm;
            *reinterpret_cast<f32x4 *>(v + o) = vv;
        } else {
            for (long long k = o; k < P; ++k) adam_one(theta[k], g[k], m[k], v[k], gs, lr, b1, b2, eps, ibc1, ibc2);
        }
    } else {
        if (i < P) adam_one(theta[i], g[i], m[i], v[i], gs, lr, b1, b2, eps, ibc1, ibc2);
    }
}

// ------------------------------------------------------------------------------------------------------------
// The same update over the whole network's vector, organised like prep_kernel: a workgroup owns a piece of one
// parameter tensor, updates theta / m / v there (the element-wise arithmetic of adam_kernel, so the same bits) and
// writes the new values straight into the workspace copy of the network (converted, re-ordered, fc.w also transposed
// through the LDS tile) -- the separate pass that would otherwise re-read the whole vector before the next forward
// pass is not needed.  Every parameter belongs to exactly one job: fc.w tiles, conv2.w / conv3.w, conv1.w, and the
// fp32 block (biases, heads).
// ------------------------------------------------------------------------------------------------------------
struct AdamShadowArgs {
    PrepArgs pa;                  // destinations, geometry and job sizes (pa.params is not used)
    float *theta;
    const float *g;
    float *m, *v;
    const float *scale, *norm_part;
    int nparts;
    float max_norm, lr, b1, b2, eps, ibc1, ibc2;
};

template <typename T> __global__ __launch_bounds__(256) void adam_shadow_kernel(const AdamShadowArgs a)
{
    __shared__ float tile[64][65];
    __shared__ float red[256];
    float gs = 1.0f;
    if (a.norm_part) gs = clip_scale(norm_from_parts(a.norm_part, a.nparts, red), a.max_norm);
    else if (a.scale) gs = a.scale[0];
    float *__restrict__ theta = a.theta;
    const float *__restrict__ g = a.g;
    float *__restrict__ m = a.m, *__restrict__ v = a.v;
    auto update = [&](long long idx) -> float {
        float th = theta[idx], mm = m[idx], vv = v[idx];
        adam_one(th, g[idx], mm, vv, gs, a.lr, a.b1, a.b2, a.eps, a.ibc1, a.ibc2);
        theta[idx] = th; m[idx] = mm; v[idx] = vv;
        return th;
    };
    const PrepArgs &p = a.pa;
    const int t = threadIdx.x;
    int blk = blockIdx.x;
    if (blk < p.nb_fc) {
        const int F = p.g.F, tf = F / 64;
        const int j0 = (blk / tf) * 64, f0 = (blk % tf) * 64;
        T *wfc = (T *)p.wfc;
        const int col = t & 63, r0 = t >> 6;
        // 16-byte accesses: a thread takes four neighbouring columns of four rows (16 lanes cover a tile row); all its
        // loads are independent and the update runs on registers.  (fc.w starts on a 16-byte boundary when the tensors
        // in front of it hold a multiple of four values; otherwise the element-wise form below is taken.)
        if (((p.g.fcw | (long long)F) & 3) == 0 && ((((uintptr_t)theta | (uintptr_t)g | (uintptr_t)m | (uintptr_t)v) & 15u) == 0)) {
            const int c4 = (t & 15) * 4, rr = t >> 4;
            f32x4 th[4], gg[4], mm[4], vv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const long long idx = p.g.fcw + (long long)(j0 + rr + 16 * i) * F + f0 + c4;
                th[i] = *reinterpret_cast<const f32x4 *>(theta + idx); gg[i] = *reinterpret_cast<const f32x4 *>(g + idx);
                mm[i] = *reinterpret_cast<const f32x4 *>(m + idx); vv[i] = *reinterpret_cast<const f32x4 *>(v + idx);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int r = rr + 16 * i;
                const long long o = (long long)(j0 + r) * F + f0 + c4;
                Vec<T, 4> w4;
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    float a0 = th[i][k], a1 = mm[i][k], a2 = vv[i][k];
                    adam_one(a0, gg[i][k], a1, a2, gs, a.lr, a.b1, a.b2, a.eps, a.ibc1, a.ibc2);
                    th[i][k] = a0; mm[i][k] = a1; vv[i][k] = a2;
                    w4[k] = from_f32<T>(a0);
                    tile[r][c4 + k] = a0;
                }
                *reinterpret_cast<f32x4 *>(theta + p.g.fcw + o) = th[i];
                *reinterpret_cast<f32x4 *>(m + p.g.fcw + o) = mm[i];
                *reinterpret_cast<f32x4 *>(v + p.g.fcw + o) = vv[i];
                *reinterpret_cast<Vec<T, 4> *>(wfc + o) = w4;
            }
        } else {
            float th[16], gg[16], mm[16], vv[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const long long idx = p.g.fcw + (long long)(j0 + r0 + 4 * i) * F + f0 + col;
                th[i] = theta[idx]; gg[i] = g[idx]; mm[i] = m[idx]; vv[i] = v[idx];
            }
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int r = r0 + 4 * i;
                const long long o = (long long)(j0 + r) * F + f0 + col;
                adam_one(th[i], gg[i], mm[i], vv[i], gs, a.lr, a.b1, a.b2, a.eps, a.ibc1, a.ibc2);
                theta[p.g.fcw + o] = th[i]; m[p.g.fcw + o] = mm[i]; v[p.g.fcw + o] = vv[i];
                wfc[o] = from_f32<T>(th[i]);
                tile[r][col] = th[i];
            }
        }
        if (!p.learn) return;
        __syncthreads();
        T *wfcd = (T *)p.wfcd;
        const int P3 = p.g.P3;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int fl = r0 + 4 * i, f = f0 + fl;
            const int c = f / P3, q = f - c * P3;
            wfcd[(long long)(q * 64 + c) * 512 + j0 + col] = from_f32<T>(tile[col][fl]);
        }
        return;
    }
    blk -= p.nb_fc;
    if (blk < p.nb_conv) {
        const int i = blk * 256 + t;
        T *wf2 = (T *)p.wf2, *wf3 = (T *)p.wf3, *wd2 = (T *)p.wd2, *wd3 = (T *)p.wd3;
        if (i < 64 * 32 * 16) {               // conv2.w[n][c][u][v], 64 x 32 x 4 x 4
            const int n = i / 512, r = i % 512, c = r / 16, tap = r % 16;
            const T w = from_f32<T>(update(p.g.w2 + i));
            wf2[n * 512 + tap * 32 + c] = w;
            if (p.learn) wd2[c * 1024 + tap * 64 + n] = w;
        }
        if (i < 64 * 64 * 9) {                // conv3.w[n][c][u][v], 64 x 64 x 3 x 3
            const int n = i / 576, r = i % 576, c = r / 9, tap = r % 9;
            const T w = from_f32<T>(update(p.g.w3 + i));
            wf3[n * 576 + tap * 64 + c] = w;
            if (p.learn) wd3[c * 576 + tap * 64 + n] = w;
        }
        return;
    }
    blk -= p.nb_conv;
    if (blk < p.nb_w1) {
        const int i = blk * 256 + t;
        if (i < 32 * p.g.K1) ((T *)p.w1s)[i] = from_f32<T>(update(p.g.w1 + i));
        return;
    }
    blk -= p.nb_w1;
    {
        const int i = blk * 256 + t;
        const int A = p.g.A;
        long long src = -1;
        if (i < 32) src = p.g.b1 + i;
        else if (i >= p.sh.b2 && i < p.sh.b2 + 64) src = p.g.b2 + (i - p.sh.b2);
        else if (i >= p.sh.b3 && i < p.sh.b3 + 64) src = p.g.b3 + (i - p.sh.b3);
        else if (i >= p.sh.fcb && i < p.sh.fcb + 512) src = p.g.fcb + (i - p.sh.fcb);
        else if (i >= p.sh.piw && i < p.sh.piw + 512 * A) src = p.g.piw + (i - p.sh.piw);
        else if (i >= p.sh.pib && i < p.sh.pib + A) src = p.g.pib + (i - p.sh.pib);
        else if (i >= p.sh.vw && i < p.sh.vw + 512) src = p.g.vw + (i - p.sh.vw);
        else if (i == p.sh.vb) src = p.g.vb;
        if (src < 0) return;
        p.hb[i] = update(src);
    }
}

static void enqueue_adam(hipStream_t stream, float *theta, const float *g, float *m, float *v, long long P,
                         const float *scale, const float *norm_part, float max_norm, float lr, float b1, float b2,
                         float eps, float bc1, float bc2)
{
    const int nparts = (int)((P + NORM_CHUNK - 1) / NORM_CHUNK);
    const bool aligned = (((uintptr_t)theta | (uintptr_t)g | (uintptr_t)m | (uintptr_t)v) & 15u) == 0;
    const float ibc1 = 1.0f / bc1, ibc2 = 1.0f / bc2;
    if (aligned) {
        const long long nthreads = (P + 3) / 4;
        hipLaunchKernelGGL(adam_kernel<true>, dim3((unsigned)((nthreads + 255) / 256)), dim3(256), 0, stream, theta, g,
                           m, v, P, scale, norm_part, nparts, max_norm, lr, b1, b2, eps, ibc1, ibc2);
    } else {
        hipLaunchKernelGGL(adam_kernel<false>, dim3((unsigned)((P + 255) / 256)), dim3(256), 0, stream, theta, g, m, v,
                           P, scale, norm_part, nparts, max_norm, lr, b1, b2, eps, ibc1, ibc2);
    }
}

hipError_t launch_adam(Ctx &c, float *theta, const float *g, float *m, float *v, long long P, const float *scale,
                       const float *norm_part, float max_norm, float lr, float b1, float b2, float eps, float bc1, float bc2)
{
    SiteTimer tm(c, SITE_ADAM);
    enqueue_adam(c.stream, theta, g, m, v, P, scale, norm_part, max_norm, lr, b1, b2, eps, bc1, bc2);
    return hipGetLastError();
}

hipError_t launch_adam_shadow(Ctx &c, float *theta, const float *g, float *m, float *v, const float *scale,
                              const float *norm_part, float max_norm, float lr, float b1, float b2, float eps, float bc1,
                              float bc2, bool learn)
{
    SiteTimer tm(c, SITE_ADAM);
    AdamShadowArgs a;
    a.pa = prep_args(c, nullptr, learn);
    a.theta = theta; a.g = g; a.m = m; a.v = v; a.scale = scale; a.norm_part = norm_part;
    a.nparts = (int)((c.g.P + NORM_CHUNK - 1) / NORM_CHUNK);
    a.max_norm = max_norm; a.lr = lr; a.b1 = b1; a.b2 = b2; a.eps = eps; a.ibc1 = 1.0f / bc1; a.ibc2 = 1.0f / bc2;
    const int nb = a.pa.nb_fc + a.pa.nb_conv + a.pa.nb_w1 + a.pa.nb_hb;
    if (c.desc.precision == HTS_PRECISION_BF16)
        hipLaunchKernelGGL(adam_shadow_kernel<bf16_t>, dim3(nb), dim3(256), 0, c.stream, a);
    else
        hipLaunchKernelGGL(adam_shadow_kernel<float>, dim3(nb), dim3(256), 0, c.stream, a);
    const hipError_t e = hipGetLastError();
    if (e == hipSuccess) { c.synced = true; c.synced_learn = learn; c.shadow_of = theta; }
    return e;
}

}  // namespace hts

// ------------------------------------------------------------------------------------------------------------
// Clip + optimiser step without a context and without any allocation: the per-chunk sums of squares of the gradient
// norm live in a file-scope device array instead of a context's workspace.  For callers that cannot allocate (code
// under graph capture, tight serving loops).  Every GPU holds its own copy of the array; its device address is looked
// up once per device and only that address is handed to kernels.
// ------------------------------------------------------------------------------------------------------------
namespace {
constexpr long long STATIC_MAX_PARAMS = HTS_STATIC_MAX_PARAMS;
constexpr int STATIC_PARTS = (int)((STATIC_MAX_PARAMS + hts::NORM_CHUNK - 1) / hts::NORM_CHUNK);
static __device__ __align__(256) float scratch[STATIC_PARTS];       // 8 KiB per GPU, held until the process ends

constexpr int STATIC_MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
float *g_scratch_ptr[STATIC_MAX_DEVICES] = {};                      // device address of `scratch`, per device

// Device address of the scratch array on the current device (looked up on first use, under a lock).
hipError_t scratch_on_current_device(float **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= STATIC_MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = static_cast<float *>(p);
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}
}  // namespace

extern "C" int32_t hts_adam_apply_static(float *params, const float *grads, hts_opt_state *opt, const hts_hparams *hp,
                                         int64_t P, void *hip_stream)
{
    using namespace hts;
    if (!params || !grads || !opt || !opt->m || !opt->v || !hp) return HTS_EINVAL;
    if (P <= 0 || opt->step < 0) return HTS_EINVAL;
    if (P > STATIC_MAX_PARAMS) return HTS_ESHAPE;          // the static array holds one partial sum per 8192 parameters
    if (hp->optimizer != HTS_OPT_ADAM && hp->optimizer != HTS_OPT_RMSPROP) return HTS_EINVAL;
    float *part = nullptr;
    hipError_t e = scratch_on_current_device(&part);
    if (e != hipSuccess) { note_hip_error(e); return HTS_EHIP; }
    hipStream_t stream = (hipStream_t)hip_stream;
    const int64_t t = opt->step + 1;
    const bool rms = hp->optimizer == HTS_OPT_RMSPROP;
    const float b1 = rms ? 0.0f : hp->beta1, b2 = rms ? hp->rms_alpha : hp->beta2;
    const float bc1 = rms ? 1.0f : (float)(1.0 - pow((double)hp->beta1, (double)t));
    const float bc2 = rms ? 1.0f : (float)(1.0 - pow((double)hp->beta2, (double)t));
    const bool clip = hp->max_grad_norm > 0.0f;
    // every partial sum the optimiser kernel reads is written by the pass before it: nothing has to start at zero
    if (clip) enqueue_sumsq(stream, grads, P, part);
    enqueue_adam(stream, params, grads, opt->m, opt->v, P, nullptr, clip ? part : nullptr, hp->max_grad_norm, hp->lr, b1,
                 b2, hp->adam_eps, bc1, bc2);
    e = hipGetLastError();
    if (e != hipSuccess) { note_hip_error(e); return HTS_EHIP; }
    opt->step = t;
    return HTS_OK;
}
