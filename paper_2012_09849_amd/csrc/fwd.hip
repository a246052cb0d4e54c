// Forward pass of the policy/value network (appendix "Implementation Details") as four tiled contractions:
// conv1 (uint8 gather, 1/255 folded in), conv2, conv3, FC.  The heads run in misc.hip.
#include "internal.hpp"

namespace hts {

template <typename T> static hipError_t forward_t(Ctx &c, const uint8_t *obs, const int32_t *index, int B, bool learn)
{
    const Geom &g = c.g;
    hipError_t e;
    const bool small = B <= c.small_b;
    const float *hb = c.ws.hb;
    {
        Conv1Fwd<T> p;
        p.M = B * g.P1; p.N = 32; p.K = g.K1; p.klen = g.K1;
        p.obs = obs; p.index = index; p.w = (const T *)c.ws.w1s; p.bias = hb + c.sh.b1; p.out = (T *)c.ws.act1;
        p.C = g.C; p.H = g.H; p.W = g.W; p.W1 = g.W1; p.P1 = g.P1;
        p.dP1 = FastDiv::make(g.P1); p.dW1 = FastDiv::make(g.W1);
        {
            SiteTimer tm(c, SITE_CONV1_FWD);
            e = small ? launch_wsgemm<Conv1Fwd<T>, 4, Conv1Fwd<T>::SEG, false>(p, c.stream) : launch_gemm(p, c.stream);
        }
        if (e != hipSuccess) return e;
    }
    {
        ConvFwd<T, Layer2, false> p;
        p.M = B * g.P2; p.N = 64; p.K = 512; p.klen = 512;
        p.in = (const T *)c.ws.act1; p.wf = (const T *)c.ws.wf2; p.bias = hb + c.sh.b2; p.out = (T *)c.ws.act2; p.out2 = nullptr;
        p.Hin = g.H1; p.Win = g.W1; p.Wo = g.W2; p.Po = g.P2;
        p.dPo = FastDiv::make(g.P2); p.dWo = FastDiv::make(g.W2);
        {
            SiteTimer tm(c, SITE_CONV2_FWD);
            e = small ? launch_wsgemm<ConvFwd<T, Layer2, false>, 8, ConvFwd<T, Layer2, false>::SEG, false>(p, c.stream)
                      : launch_gemm(p, c.stream);
        }
        if (e != hipSuccess) return e;
    }
    {
        ConvFwd<T, Layer3, true> p;
        p.M = B * g.P3; p.N = 64; p.K = 576; p.klen = 576;
        p.in = (const T *)c.ws.act2; p.wf = (const T *)c.ws.wf3; p.bias = hb + c.sh.b3; p.out = (T *)c.ws.a3;
        p.out2 = learn ? (T *)c.ws.a3n : nullptr;
        p.Hin = g.H2; p.Win = g.W2; p.Wo = g.W3; p.Po = g.P3;
        p.dPo = FastDiv::make(g.P3); p.dWo = FastDiv::make(g.W3);
        {
            SiteTimer tm(c, SITE_CONV3_FWD);
            e = small ? launch_wsgemm<ConvFwd<T, Layer3, true>, (sizeof(T) == 4 ? 8 : 4), ConvFwd<T, Layer3, true>::SEG, false, true>(p, c.stream)
                      : launch_gemm(p, c.stream);
        }
        if (e != hipSuccess) return e;
    }
    {   // groups of FC_GROUP_K inputs; the heads kernel adds them (same grouping and order on both paths)
        FcFwd<T> p;
        p.M = B; p.N = 512; p.K = g.F; p.klen = FC_GROUP_K;
        p.a3 = (const T *)c.ws.a3; p.w = (const T *)c.ws.wfc; p.part = c.ws.fc_part;
        static_assert(FC_GROUP_K % FcFwd<T>::SEG == 0, "a group is a whole number of segments");
        {
            SiteTimer tm(c, SITE_FC_FWD);
            e = small ? launch_wsgemm<FcFwd<T>, 8, FcFwd<T>::SEG, false>(p, c.stream, FC_GROUP_K / FcFwd<T>::SEG)
                      : launch_gemm(p, c.stream);
        }
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t run_forward(Ctx &c, const uint8_t *obs, const int32_t *index, int B, bool learn)
{
    return c.desc.precision == HTS_PRECISION_BF16 ? forward_t<bf16_t>(c, obs, index, B, learn)
                                                  : forward_t<float>(c, obs, index, B, learn);
}

template <typename T> static hipError_t plain_t(Ctx &c, const float *A, const float *Bm, float *C, int M, int N, int K)
{
    PlainGemm<T> p;
    p.M = M; p.N = N; p.K = K; p.klen = K; p.A = A; p.B = Bm; p.C = C;
    return launch_gemm(p, c.stream);
}

hipError_t run_plain_gemm(Ctx &c, int precision, const float *A, const float *B, float *C, int M, int N, int K)
{
    return precision == HTS_PRECISION_BF16 ? plain_t<bf16_t>(c, A, B, C, M, N, K) : plain_t<float>(c, A, B, C, M, N, K);
}

}  // namespace hts
