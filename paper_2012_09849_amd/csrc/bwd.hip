// Backward pass: every weight gradient and input gradient of the network as tiled contractions.  Weight gradients
// of the conv layers reduce over B*Ho*Wo positions; they are split into fixed chunks along that axis (split_for),
// each chunk writes its own partial, and wgrad_reduce adds the partials in chunk order -- no atomics, so the
// gradient is bit-identical from run to run.
#include "internal.hpp"

namespace hts {

template <typename T> static hipError_t backward_t(Ctx &c, const uint8_t *obs, const int32_t *index, int B, float *grads)
{
    const Geom &g = c.g;
    hipError_t e;
    // Small minibatches take the wave-per-segment kernels: many more, much shorter dependency chains.
    const bool small = B <= c.small_b;
    // groups of 64-row segments for the split weight gradients on that path: at most max_groups partial buffers per
    // layer, at least min_segs segments per group (never more groups than the tile path's split_for allows for the
    // same reduction length, which is what the partial buffers are sized for)
    auto groups_for = [](long long kp, int *spg, int max_groups, int min_segs) {
        const int nseg = (int)((kp + 63) / 64);
        int s = (nseg + max_groups - 1) / max_groups;
        s = ((s + 3) / 4) * 4;
        if (s < min_segs) s = min_segs;
        *spg = s;
        return (nseg + s - 1) / s;
    };
    {   // heads: pi.w, pi.b, v.w, v.b
        HeadsWgrad p;
        p.M = g.A + 1; p.N = 513; p.K = B; p.klen = B;
        p.dz = c.ws.dz; p.h = c.ws.h; p.g = grads; p.A = g.A;
        p.piw = g.piw; p.pib = g.pib; p.vw = g.vw; p.vb = g.vb;
        {
            SiteTimer tm(c, SITE_HEADS_WGRAD);        // tiny output, long reduction: 16 wavefronts share each tile
            e = launch_wsgemm<HeadsWgrad, 16, 32, false>(p, c.stream);
        }
        if (e != hipSuccess) return e;
    }
    {   // fc.w, fc.b
        FcWgrad<T> p;
        p.M = 512; p.N = g.F + 1; p.K = B; p.klen = B;
        p.dh = c.ws.dh; p.a3 = (const T *)c.ws.a3; p.g = grads; p.F = g.F; p.fcw = g.fcw; p.fcb = g.fcb;
        { SiteTimer tm(c, SITE_FC_WGRAD); e = launch_gemm(p, c.stream); }
        if (e != hipSuccess) return e;
    }
    {   // d(conv3 pre-activation)
        FcDgrad<T> p;
        p.M = B; p.N = g.F; p.K = 512; p.klen = 512;
        p.dh = c.ws.dh; p.wfcd = (const T *)c.ws.wfcd; p.a3n = (const T *)c.ws.a3n; p.dy3 = (T *)c.ws.dy3;
        {
            SiteTimer tm(c, SITE_FC_DGRAD);
            e = small ? launch_wsgemm<FcDgrad<T>, 4, 64, false>(p, c.stream) : launch_gemm(p, c.stream);
        }
        if (e != hipSuccess) return e;
    }
    // partial buffers of the three conv weight gradients live side by side in ws.part
    const SplitK s3 = split_for((long long)B * g.P3, MAXZ3), s2 = split_for((long long)B * g.P2, MAXZ2),
                 s1 = split_for((long long)B * g.P1, MAXZ1);
    int spg3 = 0, spg2 = 0, spg1 = 0;
    const int nz3 = small ? groups_for((long long)B * g.P3, &spg3, 32, 8) : s3.nz;
    const int nz2 = small ? groups_for((long long)B * g.P2, &spg2, 32, 8) : s2.nz;
    const int nz1 = small ? groups_for((long long)B * g.P1, &spg1, 128, 4) : s1.nz;   // long reduction, tiny output
    float *part3 = c.ws.part;
    float *part2 = part3 + (size_t)nz3 * 64 * 577;
    float *part1 = part2 + (size_t)nz2 * 64 * 513;
    {   // conv3.w, conv3.b
        ConvWgrad<T, Layer3> p;
        p.M = 64; p.N = 577; p.K = B * g.P3; p.klen = s3.klen;
        p.dy = (const T *)c.ws.dy3; p.in = (const T *)c.ws.act2; p.part = part3;
        p.Hin = g.H2; p.Win = g.W2; p.Wo = g.W3; p.Po = g.P3;
        p.dPo = FastDiv::make(g.P3); p.dWo = FastDiv::make(g.W3);
        {
            SiteTimer tm(c, SITE_CONV3_WGRAD);
            e = small ? launch_wsgemm<ConvWgrad<T, Layer3>, 4, 64, false>(p, c.stream, spg3) : launch_gemm(p, c.stream);
        }
        if (e != hipSuccess) return e;
    }
    {   // d(conv2 pre-activation)
        ConvDgrad<T, Layer3> p;
        p.N = 64; p.K = 576; p.klen = 576;
        p.dy = (const T *)c.ws.dy3; p.wd = (const T *)c.ws.wd3; p.act_in = (const T *)c.ws.act2; p.dy_in = (T *)c.ws.dy2;
        p.Bn = B; p.Hin = g.H2; p.Win = g.W2; p.Ho = g.H3; p.Wo = g.W3;
        p.prepare();
        {
            SiteTimer tm(c, SITE_CONV3_DGRAD);
            // fp32: eight segments of 72 for eight wavefronts, and panels small enough for two workgroups per compute unit
            e = small ? launch_wsgemm<ConvDgrad<T, Layer3>, (sizeof(T) == 4 ? 8 : 4), (sizeof(T) == 2 ? 192 : 72), false, true>(p, c.stream) : launch_gemm(p, c.stream);
        }
        if (e != hipSuccess) return e;
    }
    {   // conv2.w, conv2.b
        ConvWgrad<T, Layer2> p;
        p.M = 64; p.N = 513; p.K = B * g.P2; p.klen = s2.klen;
        p.dy = (const T *)c.ws.dy2; p.in = (const T *)c.ws.act1; p.part = part2;
        p.Hin = g.H1; p.Win = g.W1; p.Wo = g.W2; p.Po = g.P2;
        p.dPo = FastDiv::make(g.P2); p.dWo = FastDiv::make(g.W2);
        {
            SiteTimer tm(c, SITE_CONV2_WGRAD);
            e = small ? launch_wsgemm<ConvWgrad<T, Layer2>, 4, 64, false>(p, c.stream, spg2) : launch_gemm(p, c.stream);
        }
        if (e != hipSuccess) return e;
    }
    {   // d(conv1 pre-activation)
        ConvDgrad<T, Layer2> p;
        p.N = 32; p.K = 256; p.klen = 256;      // four parity classes, 2x2 taps each
        p.dy = (const T *)c.ws.dy2; p.wd = (const T *)c.ws.wd2; p.act_in = (const T *)c.ws.act1; p.dy_in = (T *)c.ws.dy1;
        p.Bn = B; p.Hin = g.H1; p.Win = g.W1; p.Ho = g.H2; p.Wo = g.W2;
        p.prepare();
        {
            SiteTimer tm(c, SITE_CONV2_DGRAD);
            e = small ? launch_wsgemm<ConvDgrad<T, Layer2>, 4, 64, false>(p, c.stream) : launch_gemm(p, c.stream);
        }
        if (e != hipSuccess) return e;
    }
    {   // conv1.w, conv1.b
        auto conv1_wgrad = [&](auto p) {
            p.M = 32; p.N = g.K1 + 1; p.K = B * g.P1; p.klen = s1.klen;
            p.dy = (const T *)c.ws.dy1; p.obs = obs; p.index = index; p.part = part1;
            p.Kc = g.K1; p.C = g.C; p.H = g.H; p.W = g.W; p.W1 = g.W1; p.P1 = g.P1;
            p.dP1 = FastDiv::make(g.P1); p.dW1 = FastDiv::make(g.W1);
            SiteTimer tm(c, SITE_CONV1_WGRAD);
            return small ? launch_wsgemm<decltype(p), 4, 64, false>(p, c.stream, spg1) : launch_gemm(p, c.stream);
        };
        e = index ? conv1_wgrad(Conv1Wgrad<T, true>{}) : conv1_wgrad(Conv1Wgrad<T, false>{});
        if (e != hipSuccess) return e;
    }
    const ReduceSpec specs[3] = {
        {part3, nz3, 64, 577, 64, 3, true, 1.0f, g.w3, g.b3},
        {part2, nz2, 64, 513, 32, 4, true, 1.0f, g.w2, g.b2},
        {part1, nz1, 32, g.K1 + 1, g.C, 8, false, 1.0f / 255.0f, g.w1, g.b1}};
    if ((e = launch_wgrad_reduce(c, specs, grads)) != hipSuccess) return e;
    return hipSuccess;
}

hipError_t run_backward(Ctx &c, const uint8_t *obs, const int32_t *index, int B, float *grads)
{
    return c.desc.precision == HTS_PRECISION_BF16 ? backward_t<bf16_t>(c, obs, index, B, grads)
                                                  : backward_t<float>(c, obs, index, B, grads);
}

}  // namespace hts
