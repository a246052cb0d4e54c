// Operand gathers and epilogues that turn each layer of the policy/value network (appendix "Implementation
// Details": conv 32@8x8 s4, conv 64@4x4 s2, conv 64@3x3 s1, FC 512, heads) and each piece of its backward pass
// into the D[m][n] = sum_k A(m,k) B(n,k) form of gemm.hpp.
//
// Layouts inside the library's workspace (T = float or bf16):
//   act1 [B][H1][W1][32], act2 [B][H2][W2][64]   channel-innermost, post-ReLU
//   a3   [B][F]           conv3 output flattened as (channel, y, x) = the order fc.w expects
//   h    [B][512] fp32    FC output, post-ReLU
//   dz   [B][A+1] fp32    dL/dlogits followed by dL/dvalue
//   dh   [B][512] fp32    dL/d(FC pre-activation)
//   dy3 [B][H3][W3][64], dy2 [B][H2][W2][64], dy1 [B][H1][W1][32]   dL/d(conv pre-activation), T
//   wf2 [64][(u,v,c)], wf3 [64][(u,v,c)]   conv weights with taps outermost, for the forward gathers
//   wd2 [32][(u,v,n)], wd3 [64][(u,v,n)]   conv weights transposed for the input-gradient gathers
#pragma once
#include "gemm.hpp"

namespace hts {

struct Geom {
    int C, H, W, A;
    int H1, W1, P1, H2, W2, P2, H3, W3, P3, F, K1;
    long long w1, b1, w2, b2, w3, b3, fcw, fcb, piw, pib, vw, vb, P;
};

// ------------------------------------------------------------------------------------------------------------
// plain C = A * B^T on f32 arrays (test hook for the tile core)
// ------------------------------------------------------------------------------------------------------------
template <typename T_> struct PlainGemm {
    using T = T_;
    static constexpr int BM = 64, BN = 64, BK = 32, WAVES_M = 2;
    static constexpr int VA = 4, VB = 4;
    static constexpr bool A_ALONG_K = true, B_ALONG_K = true;
    int M, N, K, klen;
    const float *A, *B;
    float *C;
    HTS_HD void load_a(int m, int k, int kend, float (&v)[VA]) const
    {
        if (m < M && k < kend) load_vec(A + (long long)m * K + k, v); else zero_vec(v);
    }
    HTS_HD void load_b(int n, int k, int kend, float (&v)[VB]) const
    {
        if (n < N && k < kend) load_vec(B + (long long)n * K + k, v); else zero_vec(v);
    }
    HTS_HD void store(int m, int n, float acc, int) const { C[(long long)m * N + n] = acc; }
};

// ------------------------------------------------------------------------------------------------------------
// conv1 forward: uint8 NCHW frames (gathered by row index), k = (c,u,v) as in conv1.w; x/255 folded into the
// epilogue (u8 values are exact in bf16 and fp32)
// ------------------------------------------------------------------------------------------------------------
template <typename T_> struct Conv1Fwd {
    using T = T_;
    static constexpr int BM = 128, BN = 32, BK = 32, WAVES_M = 4;
    static constexpr int VA = 8, VB = 4;
    static constexpr bool A_ALONG_K = true, B_ALONG_K = true;
    static constexpr int SEG = 64;       // forward sums are segmented so every kernel variant returns the same bits
    int M, N, K, klen;
    const uint8_t *obs;
    const int32_t *index;
    const float *w, *bias;
    T *out;
    int C, H, W, W1, P1;
    HTS_HD void load_a(int m, int k, int kend, float (&v)[VA]) const
    {
        if (m < M && k < kend) {
            const int b = m / P1, p = m - b * P1, oy = p / W1, ox = p - oy * W1;
            const int c = k >> 6, u = (k >> 3) & 7;
            const long long row = index ? index[b] : b;
            const uint8_t *src = obs + ((row * C + c) * H + (oy * 4 + u)) * (long long)W + ox * 4;
            const uint32_t lo = *reinterpret_cast<const uint32_t *>(src);
            const uint32_t hi = *reinterpret_cast<const uint32_t *>(src + 4);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                v[i] = (float)((lo >> (8 * i)) & 0xFFu);
                v[4 + i] = (float)((hi >> (8 * i)) & 0xFFu);
            }
        } else zero_vec(v);
    }
    HTS_HD void load_b(int n, int k, int kend, float (&v)[VB]) const
    {
        if (n < N && k < kend) load_vec(w + (long long)n * K + k, v); else zero_vec(v);
    }
    HTS_HD void store(int m, int n, float acc, int) const
    {
        const float y = acc * (1.0f / 255.0f) + bias[n];
        out[(long long)m * 32 + n] = from_f32<T>(y > 0.0f ? y : 0.0f);
    }
};

// ------------------------------------------------------------------------------------------------------------
// conv2 / conv3 forward from channel-innermost activations; k = (u,v,c)
// ------------------------------------------------------------------------------------------------------------
template <typename T_, bool FLAT_OUT> struct ConvFwd {
    using T = T_;
    static constexpr int BM = 64, BN = 64, BK = 32, WAVES_M = 2;
    static constexpr int VA = OperandTraits<T>::VEC, VB = OperandTraits<T>::VEC;
    static constexpr bool A_ALONG_K = true, B_ALONG_K = true;
    static constexpr int SEG = FLAT_OUT ? 96 : 64;
    int M, N, K, klen;
    const T *in;      // [B][Hin][Win][Cin]
    const T *wf;      // [Cout][K]
    const float *bias;
    T *out;
    int Cin, Hin, Win, ksz, stride, Wo, Po, Cout;
    HTS_HD void load_a(int m, int k, int kend, float (&v)[VA]) const
    {
        if (m < M && k < kend) {
            const int b = m / Po, p = m - b * Po, oy = p / Wo, ox = p - oy * Wo;
            const int tap = k / Cin, c = k - tap * Cin, u = tap / ksz, vv = tap - u * ksz;
            load_vec(in + (((long long)b * Hin + oy * stride + u) * Win + ox * stride + vv) * Cin + c, v);
        } else zero_vec(v);
    }
    HTS_HD void load_b(int n, int k, int kend, float (&v)[VB]) const
    {
        if (n < N && k < kend) load_vec(wf + (long long)n * K + k, v); else zero_vec(v);
    }
    HTS_HD void store(int m, int n, float acc, int) const
    {
        const float y = acc + bias[n];
        const T r = from_f32<T>(y > 0.0f ? y : 0.0f);
        if constexpr (FLAT_OUT) {
            const int b = m / Po, p = m - b * Po;
            out[((long long)b * Cout + n) * Po + p] = r;
        } else out[(long long)m * Cout + n] = r;
    }
};

// ------------------------------------------------------------------------------------------------------------
// FC forward: h = relu(a3 * fc.w^T + fc.b), fc.w read in its fp32 packing
// ------------------------------------------------------------------------------------------------------------
template <typename T_> struct FcFwd {
    using T = T_;
    static constexpr int BM = 64, BN = 64, BK = 32, WAVES_M = 2;
    static constexpr int VA = OperandTraits<T>::VEC, VB = 4;
    static constexpr bool A_ALONG_K = true, B_ALONG_K = true;
    static constexpr int SEG = 128;
    int M, N, K, klen;
    const T *a3;
    const float *w, *bias;
    float *h;
    float *part;      // when set: segment sums go to part[seg][M][N]; bias and ReLU are applied by the consumer
    HTS_HD void load_a(int m, int k, int kend, float (&v)[VA]) const
    {
        if (m < M && k < kend) load_vec(a3 + (long long)m * K + k, v); else zero_vec(v);
    }
    HTS_HD void load_b(int n, int k, int kend, float (&v)[VB]) const
    {
        if (n < N && k < kend) load_vec(w + (long long)n * K + k, v); else zero_vec(v);
    }
    HTS_HD void store(int m, int n, float acc, int seg) const
    {
        if (part) { part[((long long)seg * M + m) * N + n] = acc; return; }
        const float y = acc + bias[n];
        h[(long long)m * N + n] = y > 0.0f ? y : 0.0f;
    }
};

// ------------------------------------------------------------------------------------------------------------
// heads weight gradient: rows j < A are pi.w[j] (column 512 = pi.b[j]); row A is v.w (column 512 = v.b).
// D[j][kk] = sum_b dz[b][j] * (kk < 512 ? h[b][kk] : 1).   Always fp32.
// ------------------------------------------------------------------------------------------------------------
struct HeadsWgrad {
    using T = float;
    static constexpr int BM = 32, BN = 128, BK = 32, WAVES_M = 1;
    static constexpr int VA = 1, VB = 4;
    static constexpr bool A_ALONG_K = false, B_ALONG_K = false;
    int M, N, K, klen;     // M = A+1, N = 513, K = B
    const float *dz, *h;
    float *g;
    int A;
    long long piw, pib, vw, vb;
    HTS_HD void load_a(int j, int b, int kend, float (&v)[VA]) const
    {
        v[0] = (j < M && b < kend) ? dz[(long long)b * M + j] : 0.0f;
    }
    HTS_HD void load_b(int kk, int b, int kend, float (&v)[VB]) const
    {
        if (b < kend && kk < 512) load_vec(h + (long long)b * 512 + kk, v);
        else { zero_vec(v); if (b < kend && kk == 512) v[0] = 1.0f; }
    }
    HTS_HD void store(int j, int kk, float acc, int) const
    {
        if (j < A) { if (kk < 512) g[piw + (long long)j * 512 + kk] = acc; else g[pib + j] = acc; }
        else       { if (kk < 512) g[vw + kk] = acc; else g[vb] = acc; }
    }
};

// ------------------------------------------------------------------------------------------------------------
// FC weight gradient: D[j][f] = sum_b dh[b][j] * (f < F ? a3[b][f] : 1); column F is fc.b
// ------------------------------------------------------------------------------------------------------------
template <typename T_> struct FcWgrad {
    using T = T_;
    static constexpr int BM = 128, BN = 64, BK = 32, WAVES_M = 4;
    static constexpr int VA = 4, VB = OperandTraits<T>::VEC;
    static constexpr bool A_ALONG_K = false, B_ALONG_K = false;
    int M, N, K, klen;     // M = 512, N = F+1, K = B
    const float *dh;
    const T *a3;
    float *g;
    int F;
    long long fcw, fcb;
    HTS_HD void load_a(int j, int b, int kend, float (&v)[VA]) const
    {
        if (b < kend) load_vec(dh + (long long)b * 512 + j, v); else zero_vec(v);   // M = 512 is a multiple of BM
    }
    HTS_HD void load_b(int f, int b, int kend, float (&v)[VB]) const
    {
        if (b < kend && f < F) load_vec(a3 + (long long)b * F + f, v);
        else { zero_vec(v); if (b < kend && f == F) v[0] = 1.0f; }
    }
    HTS_HD void store(int j, int f, float acc, int) const
    {
        if (f < F) g[fcw + (long long)j * F + f] = acc; else g[fcb + j] = acc;
    }
};

// ------------------------------------------------------------------------------------------------------------
// FC input gradient, masked by conv3's ReLU and written channel-innermost:
// D[b][f] = sum_j dh[b][j] fc.w[j][f];  dy3[b][p][c] = a3[b][f] > 0 ? D : 0,  f = c*P3 + p
// ------------------------------------------------------------------------------------------------------------
template <typename T_> struct FcDgrad {
    using T = T_;
    static constexpr int BM = 64, BN = 64, BK = 32, WAVES_M = 2;
    static constexpr int VA = 4, VB = 4;
    static constexpr bool A_ALONG_K = true, B_ALONG_K = false;
    int M, N, K, klen;     // M = B, N = F, K = 512
    const float *dh, *w;
    const T *a3;
    T *dy3;
    int P3;
    HTS_HD void load_a(int b, int k, int kend, float (&v)[VA]) const
    {
        if (b < M && k < kend) load_vec(dh + (long long)b * 512 + k, v); else zero_vec(v);
    }
    HTS_HD void load_b(int f, int j, int kend, float (&v)[VB]) const
    {
        if (j < kend && f < N) load_vec(w + (long long)j * N + f, v); else zero_vec(v);      // N = F is a multiple of 4
    }
    HTS_HD void store(int b, int f, float acc, int) const
    {
        const int c = f / P3, p = f - c * P3;
        const float a = to_f32(a3[(long long)b * N + f]);
        dy3[((long long)b * P3 + p) * 64 + c] = from_f32<T>(a > 0.0f ? acc : 0.0f);
    }
};

// ------------------------------------------------------------------------------------------------------------
// conv input gradient (layers 3 and 2): dX[b][y][x][c] = sum_{u,v,n} dy[b][(y-u)/s][(x-v)/s][n] W[n][c][u][v] over the
// taps where (y-u), (x-v) are non-negative multiples of the stride s inside the output; masked by the ReLU of the
// layer below.  Input positions are split into s*s parity classes (y%s, x%s): within a class only the (ksz/s)^2
// taps u = y%s + s*a, v = x%s + s*bb can contribute, so each class is its own dense contraction
//   M = B*Hc*Wc (positions of the class),  N = Cin,  K = (ksz/s)^2 * Cout,  k = (a, bb, n),
// launched as one batch entry per class (no multiplications by structural zeros).  wd = [Cin][(u,v,n)].
// ------------------------------------------------------------------------------------------------------------
template <typename T_, int BN_> struct ConvDgrad {
    using T = T_;
    static constexpr int BM = (BN_ == 32 ? 128 : 64), BN = BN_, BK = 32, WAVES_M = (BN_ == 32 ? 4 : 2);
    static constexpr int VA = OperandTraits<T>::VEC, VB = OperandTraits<T>::VEC;
    static constexpr bool A_ALONG_K = true, B_ALONG_K = true;
    int M, N, K, klen;     // M is per class (set_batch); N = Cin; K = (ksz/s)^2 * Cout
    const T *dy;           // [B][Ho][Wo][Cout]
    const T *wd;           // [Cin][ksz*ksz*Cout]
    const T *act_in;       // [B][Hin][Win][Cin] post-ReLU output of the layer below
    T *dy_in;              // [B][Hin][Win][Cin]
    int Bn, Hin, Win, Ho, Wo, Cout, ksz, stride;
    int py, px, Hc, Wc;    // current class and its extent
    HTS_HD int batches() const { return stride * stride; }
    HTS_HD int max_m() const { return Bn * ((Hin + stride - 1) / stride) * ((Win + stride - 1) / stride); }
    HTS_HD void set_batch(int z)
    {
        py = z / stride; px = z - py * stride;
        Hc = (Hin - py + stride - 1) / stride; Wc = (Win - px + stride - 1) / stride;
        M = Bn * Hc * Wc;
    }
    HTS_HD void load_a(int m, int k, int kend, float (&v)[VA]) const
    {
        if (m < M && k < kend) {
            const int b = m / (Hc * Wc), p = m - b * (Hc * Wc), yy = p / Wc, xx = p - yy * Wc;
            const int tap = k / Cout, n = k - tap * Cout, tk = ksz / stride, a = tap / tk, bb = tap - a * tk;
            const int oy = yy - a, ox = xx - bb;         // (y - u)/s with y = yy*s + py, u = py + s*a
            if (oy >= 0 && ox >= 0 && oy < Ho && ox < Wo) {
                load_vec(dy + (((long long)b * Ho + oy) * Wo + ox) * Cout + n, v);
                return;
            }
        }
        zero_vec(v);
    }
    HTS_HD void load_b(int c, int k, int kend, float (&v)[VB]) const
    {
        if (c < N && k < kend) {
            const int tap = k / Cout, n = k - tap * Cout, tk = ksz / stride, a = tap / tk, bb = tap - a * tk;
            const int u = py + stride * a, vv = px + stride * bb;
            load_vec(wd + ((long long)c * ksz * ksz + u * ksz + vv) * Cout + n, v);
        } else zero_vec(v);
    }
    HTS_HD void store(int m, int c, float acc, int) const
    {
        const int b = m / (Hc * Wc), p = m - b * (Hc * Wc), yy = p / Wc, xx = p - yy * Wc;
        const long long o = ((((long long)b * Hin + yy * stride + py) * Win) + xx * stride + px) * N + c;
        const float a = to_f32(act_in[o]);
        dy_in[o] = from_f32<T>(a > 0.0f ? acc : 0.0f);
    }
};

// ------------------------------------------------------------------------------------------------------------
// conv weight gradient (layers 3 and 2), split over blockIdx.y along the B*Ho*Wo reduction:
// part[z][n][kcol] = sum_{m in chunk z} dy[m][n] * (kcol < K ? im2col(in)[m][kcol] : 1); column K is the bias.
// ------------------------------------------------------------------------------------------------------------
template <typename T_> struct ConvWgrad {
    using T = T_;
    static constexpr int BM = 64, BN = 64, BK = 32, WAVES_M = 2;
    static constexpr int VA = OperandTraits<T>::VEC, VB = OperandTraits<T>::VEC;
    static constexpr bool A_ALONG_K = false, B_ALONG_K = false;
    int M, N, K, klen;     // M = Cout (64), N = Kc + 1, K = B*Po
    const T *dy;           // [B*Po][Cout]
    const T *in;           // [B][Hin][Win][Cin]
    float *part;           // [nz][Cout][N]
    int Kc, Cin, Hin, Win, ksz, stride, Wo, Po;
    HTS_HD void load_a(int n, int m, int kend, float (&v)[VA]) const
    {
        if (m < kend) load_vec(dy + (long long)m * M + n, v); else zero_vec(v);       // M = 64 = BM
    }
    HTS_HD void load_b(int kcol, int m, int kend, float (&v)[VB]) const
    {
        if (m < kend && kcol < Kc) {
            const int b = m / Po, p = m - b * Po, oy = p / Wo, ox = p - oy * Wo;
            const int tap = kcol / Cin, c = kcol - tap * Cin, u = tap / ksz, vv = tap - u * ksz;
            load_vec(in + (((long long)b * Hin + oy * stride + u) * Win + ox * stride + vv) * Cin + c, v);
        } else { zero_vec(v); if (m < kend && kcol == Kc) v[0] = 1.0f; }
    }
    HTS_HD void store(int n, int kcol, float acc, int z) const
    {
        part[((long long)z * M + n) * N + kcol] = acc;
    }
};

// conv1 weight gradient: as above with the uint8 frames as the im2col source, kcol = (c,u,v)
template <typename T_> struct Conv1Wgrad {
    using T = T_;
    static constexpr int BM = 32, BN = 128, BK = 32, WAVES_M = 1;
    static constexpr int VA = OperandTraits<T>::VEC, VB = 8;
    static constexpr bool A_ALONG_K = false, B_ALONG_K = false;
    int M, N, K, klen;     // M = 32, N = C*64 + 1, K = B*P1
    const T *dy;           // [B*P1][32]
    const uint8_t *obs;
    const int32_t *index;
    float *part;           // [nz][32][N]
    int Kc, C, H, W, W1, P1;
    HTS_HD void load_a(int n, int m, int kend, float (&v)[VA]) const
    {
        if (m < kend) load_vec(dy + (long long)m * 32 + n, v); else zero_vec(v);
    }
    HTS_HD void load_b(int kcol, int m, int kend, float (&v)[VB]) const
    {
        if (m < kend && kcol < Kc) {
            const int b = m / P1, p = m - b * P1, oy = p / W1, ox = p - oy * W1;
            const int c = kcol >> 6, u = (kcol >> 3) & 7;
            const long long row = index ? index[b] : b;
            const uint8_t *src = obs + ((row * C + c) * H + (oy * 4 + u)) * (long long)W + ox * 4;
            const uint32_t lo = *reinterpret_cast<const uint32_t *>(src);
            const uint32_t hi = *reinterpret_cast<const uint32_t *>(src + 4);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                v[i] = (float)((lo >> (8 * i)) & 0xFFu);
                v[4 + i] = (float)((hi >> (8 * i)) & 0xFFu);
            }
        } else { zero_vec(v); if (m < kend && kcol == Kc) v[0] = 255.0f; }   // the 1/255 of the input scaling is
    }                                                                        // applied when partials are combined
    HTS_HD void store(int n, int kcol, float acc, int z) const
    {
        part[((long long)z * 32 + n) * N + kcol] = acc;
    }
};

}  // namespace hts
