// Operand gathers and epilogues that turn each layer of the policy/value network (appendix "Implementation
// Details": conv 32@8x8 s4, conv 64@4x4 s2, conv 64@3x3 s1, FC 512, heads) and each piece of its backward pass
// into the D[m][n] = sum_k A(m,k) B(n,k) form of gemm.hpp / wsgemm.hpp.
//
// Layouts inside the library's workspace (T = float or bf16):
//   act1 [B][H1][W1][32], act2 [B][H2][W2][64]   channel-innermost, post-ReLU
//   a3   [B][F]           conv3 output flattened as (channel, y, x) = the order fc.w expects
//   a3n  [B][H3][W3][64]  the same values channel-innermost (learner only)
//   fc_part [G][B][512]   FC partial sums, one per group of 512 inputs; bias + ReLU when the heads kernel adds them
//   h    [B][512] fp32    FC output, post-ReLU (learner only; written by the heads kernel)
//   dz   [B][A+1] fp32    dL/dlogits followed by dL/dvalue
//   dh   [B][512] fp32    dL/d(FC pre-activation)
//   dy3 [B][H3][W3][64], dy2 [B][H2][W2][64], dy1 [B][H1][W1][32]   dL/d(conv pre-activation), T
//   w1s [32][(c,u,v)], wfc [512][F]        conv1.w and fc.w in their own order, as T
//   wf2 [64][(u,v,c)], wf3 [64][(u,v,c)]   conv weights with taps outermost, for the forward gathers
//   wd2 [32][(u,v,n)], wd3 [64][(u,v,n)]   conv weights transposed for the input-gradient gathers
//   wfcd [(p,c)][512]                      fc.w transposed, rows in channel-innermost order, for the FC input gradient
//
// Every gather is split into a row part (ctx_a / ctx_b: the batch / y / x decomposition, evaluated once per thread)
// and a k part (load_a / load_b: taps and channels, with compile-time layer constants).
#pragma once
#include "gemm.hpp"

// k per staged tile of the tile kernel for bf16 operands (fp32: 32 everywhere).  The weight gradients walk a long
// reduction chunk per workgroup and are bound by the latency of each step, so they take deeper tiles (measured at
// B = 1024: conv1 92 -> 53 us, conv2 50 -> 41 us); forward and input-gradient kernels measured no faster or slower.
constexpr int BK_BF16 = 64, BK_BF16_WGRAD = 128;

namespace hts {

struct Geom {
    int C, H, W, A;
    int H1, W1, P1, H2, W2, P2, H3, W3, P3, F, K1;
    long long w1, b1, w2, b2, w3, b3, fcw, fcb, piw, pib, vw, vb, P;
};

// conv2: 32 -> 64 channels, 4x4 stride 2;  conv3: 64 -> 64 channels, 3x3 stride 1
template <int CIN_, int KSZ_, int STRIDE_> struct ConvLayer {
    static constexpr int CIN = CIN_, KSZ = KSZ_, STRIDE = STRIDE_, COUT = 64, K = KSZ_ * KSZ_ * CIN_;
};
typedef ConvLayer<32, 4, 2> Layer2;
typedef ConvLayer<64, 3, 1> Layer3;

// Row part of a gather: pointer to the row's first operand.  Rows outside the matrix are clamped to the last valid
// row (their products land in output rows that are never stored), so loads need no row check; only the end of the
// reduction range (k >= kend) yields zeros.
template <typename S> struct PtrCtx { const S *p; };
HTS_HD int clamp_row(int r, int n) { return r < n ? r : n - 1; }

// ------------------------------------------------------------------------------------------------------------
// plain C = A * B^T on f32 arrays (test hook for the tile core)
// ------------------------------------------------------------------------------------------------------------
template <typename T_> struct PlainGemm {
    using T = T_;
    static constexpr int BM = 64, BN = 64, BK = OperandTraits<T>::BK, WAVES_M = 2, WAVES_N = 2;
    static constexpr int VA = 4, VB = 4;
    static constexpr bool A_ALONG_K = true, B_ALONG_K = true;
    typedef PtrCtx<float> CtxA;
    typedef PtrCtx<float> CtxB;
    int M, N, K, klen;
    const float *A, *B;
    float *C;
    HTS_HD CtxA ctx_a(int m) const { return {A + (long long)clamp_row(m, M) * K}; }
    HTS_HD CtxB ctx_b(int n) const { return {B + (long long)clamp_row(n, N) * K}; }
    HTS_HD Vec<T, VA> load_a(const CtxA &c, int k, int kend) const
    {
        return keep_if<T, VA>(k < kend, load_vec<T, VA>(c.p + (k < kend ? k : 0)));
    }
    HTS_HD Vec<T, VB> load_b(const CtxB &c, int k, int kend) const
    {
        return keep_if<T, VB>(k < kend, load_vec<T, VB>(c.p + (k < kend ? k : 0)));
    }
    HTS_HD void store(int m, int n, float acc, int) const { C[(long long)m * N + n] = acc; }
};

// ------------------------------------------------------------------------------------------------------------
// conv1 forward: uint8 NCHW frames (gathered by row index), k = (c,u,v) as in conv1.w; x/255 folded into the
// epilogue (u8 values are exact in bf16 and fp32)
// ------------------------------------------------------------------------------------------------------------
template <typename T_> struct Conv1Fwd {
    using T = T_;
    static constexpr int BM = 256, BN = 32, BK = (sizeof(T) == 2 ? BK_BF16 : 32), WAVES_M = 8, WAVES_N = 1;
    static constexpr int VA = 8, VB = OperandTraits<T>::VEC;
    static constexpr bool A_ALONG_K = true, B_ALONG_K = true;
    static constexpr int SEG = 64;       // forward sums are segmented so every kernel variant returns the same bits
    static constexpr int STAGES = sizeof(T) == 2 ? 2 : 1;     // bf16: two k-tiles of loads in flight (16x72x96 frames: 169 -> 147 us at B = 2048)
    typedef PtrCtx<uint8_t> CtxA;
    typedef PtrCtx<T> CtxB;
    int M, N, K, klen;
    const uint8_t *obs;
    const int32_t *index;
    const T *w;
    const float *bias;
    T *out;
    int C, H, W, W1, P1;
    FastDiv dP1, dW1;
    HTS_HD CtxA ctx_a(int m) const
    {
        m = clamp_row(m, M);
        const int b = dP1.div(m), p = m - b * P1, oy = dW1.div(p), ox = p - oy * W1;
        const long long row = index ? index[b] : b;
        return {obs + row * C * H * W + (oy * 4) * W + ox * 4};
    }
    HTS_HD CtxB ctx_b(int n) const { return {w + (long long)clamp_row(n, N) * K}; }
    // K = 64*C is a whole number of k-tiles and segments: no end-of-range checks
    HTS_HD Vec<T, VA> load_a(const CtxA &c, int k, int) const
    {
        const unsigned uk = (unsigned)k, ch = uk >> 6, u = (uk >> 3) & 7u;
        return load_u8x8<T>(c.p + (ch * (unsigned)H + u) * (unsigned)W);
    }
    HTS_HD Vec<T, VB> load_b(const CtxB &c, int k, int) const { return load_vec<T, VB>(c.p + k); }
    HTS_HD float col(int n) const { return bias[n]; }
    HTS_HD void store(int m, int n, float acc, int, const float &b) const
    {
        const float y = __builtin_fmaf(acc, 1.0f / 255.0f, b);     // explicit: every conv1 kernel rounds alike
        out[(long long)m * 32 + n] = from_f32<T>(y > 0.0f ? y : 0.0f);
    }
};

// ------------------------------------------------------------------------------------------------------------
// conv2 / conv3 forward from channel-innermost activations; k = (u,v,c)
// ------------------------------------------------------------------------------------------------------------
template <typename T_, class L, bool FLAT_OUT> struct ConvFwd {
    using T = T_;
    static constexpr int BM = 128, BN = 64, BK = (sizeof(T) == 2 ? BK_BF16 : 32), WAVES_M = 4, WAVES_N = 1;
    static constexpr int VA = OperandTraits<T>::VEC, VB = OperandTraits<T>::VEC;
    static constexpr bool A_ALONG_K = true, B_ALONG_K = true;
    // conv2: half a tap row (a tap row is 4*32 = 128); conv3: one tap row (3*64 = 192) for bf16, half of one for fp32
    static constexpr int SEG = L::KSZ == 4 ? 64 : (sizeof(T) == 2 ? 192 : 96);
    typedef PtrCtx<T> CtxA;
    typedef PtrCtx<T> CtxB;
    int M, N, K, klen;
    const T *in;      // [B][Hin][Win][Cin]
    const T *wf;      // [Cout][K]
    const float *bias;
    T *out;
    T *out2;          // FLAT_OUT only, optional: a second, channel-innermost copy of the output
    int Hin, Win, Wo, Po;
    FastDiv dPo, dWo;
    HTS_HD CtxA ctx_a(int m) const
    {
        m = clamp_row(m, M);
        const int b = dPo.div(m), p = m - b * Po, oy = dWo.div(p), ox = p - oy * Wo;
        return {in + (((long long)b * Hin + oy * L::STRIDE) * Win + ox * L::STRIDE) * L::CIN};
    }
    HTS_HD CtxB ctx_b(int n) const { return {wf + (long long)clamp_row(n, N) * K}; }
    // K (512, 576) is a whole number of k-tiles and segments: no end-of-range checks
    HTS_HD Vec<T, VA> load_a(const CtxA &c, int k, int) const
    {
        const unsigned uk = (unsigned)k, u = uk / (unsigned)(L::KSZ * L::CIN), r = uk - u * (L::KSZ * L::CIN);
        return load_vec<T, VA>(c.p + (u * (unsigned)(Win * L::CIN) + r));     // a tap row is contiguous in memory
    }
    HTS_HD Vec<T, VB> load_b(const CtxB &c, int k, int) const { return load_vec<T, VB>(c.p + k); }
    // tile kernel, flattened output (conv3): a lane owns an output position, so the (sample, position) split of the
    // row index is done once per lane instead of once per element (the plain layout measured no faster that way)
    static constexpr bool LANE_OWNS_ROW = FLAT_OUT;
    static constexpr bool EPI_INPUTS_EARLY = false;      // pre4() is the bias: hot in L1, not worth registers during the k loop
    struct Row { long long o; long long o2; };
    HTS_HD Row row(int m) const
    {
        if constexpr (FLAT_OUT) {
            const int b = dPo.div(m), p = m - b * Po;
            return {(long long)b * L::COUT * Po + p, (long long)m * L::COUT};
        } else return {(long long)m * L::COUT, 0};
    }
    HTS_HD f32x4 pre4(const Row &, int n) const { return *reinterpret_cast<const f32x4 *>(bias + n); }
    HTS_HD void store4(const Row &r, int n, const float (&v)[4], int, const f32x4 &bn) const
    {
        Vec<T, 4> y;
#pragma unroll
        for (int q = 0; q < 4; ++q) { const float t = v[q] + bn[q]; y[q] = from_f32<T>(t > 0.0f ? t : 0.0f); }
        if constexpr (FLAT_OUT) {
#pragma unroll
            for (int q = 0; q < 4; ++q) out[r.o + (long long)(n + q) * Po] = y[q];
            if (out2) *reinterpret_cast<Vec<T, 4> *>(out2 + r.o2 + n) = y;
        } else *reinterpret_cast<Vec<T, 4> *>(out + r.o + n) = y;
    }
    HTS_HD float col(int n) const { return bias[n]; }
    HTS_HD void store(int m, int n, float acc, int, const float &bn) const
    {
        const float y = acc + bn;
        const T r = from_f32<T>(y > 0.0f ? y : 0.0f);
        if constexpr (FLAT_OUT) {
            const int b = dPo.div(m), p = m - b * Po;
            out[((long long)b * L::COUT + n) * Po + p] = r;
            if (out2) out2[(long long)m * L::COUT + n] = r;
        } else out[(long long)m * L::COUT + n] = r;
    }
};

// ------------------------------------------------------------------------------------------------------------
// FC forward, cut along the reduction into groups of klen inputs (blockIdx.y): part[g][b][j] = sum over group g of
// a3[b][f] * fc.w[j][f].  The heads kernel adds the groups in order and applies bias and ReLU.
// ------------------------------------------------------------------------------------------------------------
template <typename T_> struct FcFwd {
    using T = T_;
    static constexpr int BM = 64, BN = 64, BK = (sizeof(T) == 2 ? BK_BF16 : 32), WAVES_M = 2, WAVES_N = 2;
    static constexpr int VA = OperandTraits<T>::VEC, VB = OperandTraits<T>::VEC;
    static constexpr bool A_ALONG_K = true, B_ALONG_K = true;
    static constexpr int SEG = 64;
    static constexpr int GROUP = 512;      // = FC_GROUP_K: klen may be any whole number of groups
    typedef PtrCtx<T> CtxA;
    typedef PtrCtx<T> CtxB;
    int M, N, K, klen;
    const T *a3, *w;
    float *part;      // [K chunks][M][N]
    HTS_HD CtxA ctx_a(int m) const { return {a3 + (long long)clamp_row(m, M) * K}; }
    HTS_HD CtxB ctx_b(int n) const { return {w + (long long)clamp_row(n, N) * K}; }
    // K = F = 64*P3 and the group length are whole numbers of k-tiles and segments: no end-of-range checks
    HTS_HD Vec<T, VA> load_a(const CtxA &c, int k, int) const { return load_vec<T, VA>(c.p + k); }
    HTS_HD Vec<T, VB> load_b(const CtxB &c, int k, int) const { return load_vec<T, VB>(c.p + k); }
    HTS_HD void store(int m, int n, float acc, int grp) const { part[((long long)grp * M + m) * N + n] = acc; }
};

// ------------------------------------------------------------------------------------------------------------
// heads weight gradient: rows j < A are pi.w[j] (column 512 = pi.b[j]); row A is v.w (column 512 = v.b).
// D[j][kk] = sum_b dz[b][j] * (kk < 512 ? h[b][kk] : 1).   Always fp32.
// ------------------------------------------------------------------------------------------------------------
struct HeadsWgrad {
    using T = float;
    static constexpr int BM = 32, BN = 128, BK = 32, WAVES_M = 1, WAVES_N = 4;
    static constexpr int VA = 1, VB = 4;
    static constexpr bool A_ALONG_K = false, B_ALONG_K = false;
    struct CtxA { int j; };
    struct CtxB { int kk; };
    int M, N, K, klen;     // M = A+1, N = 513, K = B
    const float *dz, *h;
    float *g;
    float *part;           // not null: the reduction is cut into groups, group z writes part[z][M][513]
    int A;
    long long piw, pib, vw, vb;
    HTS_HD CtxA ctx_a(int j) const { return {j}; }
    HTS_HD CtxB ctx_b(int kk) const { return {kk}; }
    HTS_HD Vec<T, VA> load_a(const CtxA &c, int b, int kend) const
    {
        Vec<T, VA> v;
        const bool in = c.j < M && b < kend;
        const float x = dz[in ? (long long)b * M + c.j : 0];
        v[0] = in ? x : 0.0f;
        return v;
    }
    HTS_HD Vec<T, VB> load_b(const CtxB &c, int b, int kend) const
    {
        const bool in = b < kend && c.kk < 512;
        Vec<T, VB> v = keep_if<T, VB>(in, load_vec<T, VB>(h + (in ? (long long)b * 512 + c.kk : 0)));
        v[0] = (b < kend && c.kk == 512) ? 1.0f : v[0];
        return v;
    }
    HTS_HD void store(int j, int kk, float acc, int z) const
    {
        if (part) { part[((long long)z * M + j) * 513 + kk] = acc; return; }
        if (j < A) { if (kk < 512) g[piw + (long long)j * 512 + kk] = acc; else g[pib + j] = acc; }
        else       { if (kk < 512) g[vw + kk] = acc; else g[vb] = acc; }
    }
};

// ------------------------------------------------------------------------------------------------------------
// FC weight gradient: D[j][f] = sum_b dh[b][j] * (f < F ? a3[b][f] : 1); column F is fc.b
// ------------------------------------------------------------------------------------------------------------
template <typename T_> struct FcWgrad {
    using T = T_;
    static constexpr int BM = 64, BN = 64, BK = (sizeof(T) == 2 ? BK_BF16_WGRAD : 32), WAVES_M = 2, WAVES_N = 2;   // 8 x 50 workgroups
    static constexpr int VA = OperandTraits<T>::VEC, VB = OperandTraits<T>::VEC;
    static constexpr bool A_ALONG_K = false, B_ALONG_K = false;
    static constexpr bool NATURAL_LDS = true;
    static constexpr bool TILES_ALONG_M = true;      // the activations (N side, B x F) outweigh dh (M side, B x 512): an XCD takes a range of columns
    struct CtxA { int j; };
    struct CtxB { int f; };
    int M, N, K, klen;     // M = 512, N = F+1, K = B
    const T *dh;           // in the operand type (the heads kernel rounds it once as it writes it)
    const T *a3;
    float *g;
    int F;
    long long fcw, fcb;
    HTS_HD CtxA ctx_a(int j) const { return {j}; }
    HTS_HD CtxB ctx_b(int f) const { return {f}; }
    HTS_HD Vec<T, VA> load_a(const CtxA &c, int b, int kend) const
    {
        return keep_if<T, VA>(b < kend, load_vec<T, VA>(dh + (uint32_t)((b < kend ? b : 0) * 512 + c.j)));   // M = 512: no row tail; 32-bit element offsets
    }
    HTS_HD Vec<T, VB> load_b(const CtxB &c, int b, int kend) const
    {
        const bool in = b < kend && c.f < F;
        Vec<T, VB> v = keep_if<T, VB>(in, load_vec<T, VB>(a3 + (in ? (uint32_t)(b * F + c.f) : 0u)));      // (fewer than 2^31 elements at the largest minibatch)
        v[0] = (b < kend && c.f == F) ? from_f32<T>(1.0f) : v[0];
        return v;
    }
    HTS_HD void store(int j, int f, float acc, int) const
    {
        if (f < F) g[fcw + (long long)j * F + f] = acc; else g[fcb + j] = acc;
    }
};

// ------------------------------------------------------------------------------------------------------------
// FC input gradient, masked by conv3's ReLU, in channel-innermost order f' = p*64 + c throughout:
// dy3[b][f'] = a3n[b][f'] > 0 ? sum_j dh[b][j] wfcd[f'][j] : 0
// ------------------------------------------------------------------------------------------------------------
template <typename T_> struct FcDgrad {
    using T = T_;
    static constexpr int BM = 64, BN = 64, BK = (sizeof(T) == 2 ? BK_BF16 : 32), WAVES_M = 2, WAVES_N = 2;
    static constexpr int VA = OperandTraits<T>::VEC, VB = OperandTraits<T>::VEC;
    static constexpr bool A_ALONG_K = true, B_ALONG_K = true;
    typedef PtrCtx<T> CtxA;
    typedef PtrCtx<T> CtxB;
    int M, N, K, klen;     // M = B, N = F, K = 512
    const T *dh;           // in the operand type
    const T *wfcd, *a3n;
    T *dy3;
    HTS_HD CtxA ctx_a(int b) const { return {dh + (long long)clamp_row(b, M) * 512}; }
    HTS_HD CtxB ctx_b(int f) const { return {wfcd + (long long)clamp_row(f, N) * 512}; }
    // K = 512 is a whole number of k-tiles and segments: no end-of-range checks
    HTS_HD Vec<T, VA> load_a(const CtxA &c, int k, int) const { return load_vec<T, VA>(c.p + k); }
    HTS_HD Vec<T, VB> load_b(const CtxB &c, int k, int) const { return load_vec<T, VB>(c.p + k); }
    static constexpr bool LANE_OWNS_ROW = true;
    struct Row { long long o; };
    HTS_HD Row row(int b) const { return {(long long)b * N}; }
    HTS_HD Vec<T, 4> pre4(const Row &r, int f) const { return *reinterpret_cast<const Vec<T, 4> *>(a3n + r.o + f); }
    HTS_HD void store4(const Row &r, int f, const float (&v)[4], int, const Vec<T, 4> &a) const
    {
        Vec<T, 4> y;
#pragma unroll
        for (int q = 0; q < 4; ++q) y[q] = from_f32<T>(to_f32(a[q]) > 0.0f ? v[q] : 0.0f);
        *reinterpret_cast<Vec<T, 4> *>(dy3 + r.o + f) = y;
    }
    HTS_HD void store(int b, int f, float acc, int) const
    {
        const long long o = (long long)b * N + f;
        dy3[o] = from_f32<T>(to_f32(a3n[o]) > 0.0f ? acc : 0.0f);
    }
    struct Pre1 { long long o; float a; };
    HTS_HD Pre1 pre1(int b, int f) const { const long long o = (long long)b * N + f; return {o, to_f32(a3n[o])}; }
    HTS_HD void store1(const Pre1 &q, float acc) const { dy3[q.o] = from_f32<T>(q.a > 0.0f ? acc : 0.0f); }
};

// ------------------------------------------------------------------------------------------------------------
// conv input gradient (layers 3 and 2): dX[b][y][x][c] = sum_{u,v,n} dy[b][(y-u)/s][(x-v)/s][n] W[n][c][u][v] over the
// taps where (y-u), (x-v) are non-negative multiples of the stride s inside the output; masked by the ReLU of the
// layer below.  Input positions are split into s*s parity classes (y%s, x%s): within a class only the (ksz/s)^2
// taps u = y%s + s*a, v = x%s + s*bb can contribute, so each class is its own dense contraction
//   M = B*Hc*Wc (positions of the class),  N = Cin,  K = (ksz/s)^2 * Cout,  k = (a, bb, n),
// launched as one batch entry per class (no multiplications by structural zeros).  wd = [Cin][(u,v,n)].
// ------------------------------------------------------------------------------------------------------------
template <typename T_, class L> struct ConvDgrad {
    using T = T_;
    static constexpr int BN = L::CIN, BM = (BN == 32 ? 128 : 64), BK = (sizeof(T) == 2 ? BK_BF16 : 32), WAVES_M = (BN == 32 ? 4 : 2),
                         WAVES_N = 4 / WAVES_M;
    static constexpr int VA = OperandTraits<T>::VEC, VB = OperandTraits<T>::VEC;
    static constexpr bool A_ALONG_K = true, B_ALONG_K = true;
    static constexpr int TK = L::KSZ / L::STRIDE;                  // taps per axis within a class
    static constexpr int KC = TK * TK * L::COUT;                   // contraction length per class
    static constexpr int NCLS = L::STRIDE * L::STRIDE;
    static_assert(NCLS <= 4, "at most four parity classes");
    struct CtxA { long long off; int yy, xx; };
    struct CtxB { long long off; int py, px; };
    struct Cls { int py, px, Hc, Wc, M; FastDiv dHW, dW; };       // one parity class
    int M, N, K, klen;     // M = rows of the largest class (grid size); N = Cin; K = KC
    const T *dy;           // [B][Ho][Wo][Cout]
    const T *wd;           // [Cin][ksz*ksz*Cout]
    const T *act_in;       // [B][Hin][Win][Cin] post-ReLU output of the layer below
    T *dy_in;              // [B][Hin][Win][Cin]
    int Bn, Hin, Win, Ho, Wo;
    FastDiv dHW0, dHW1, dHW2, dHW3, dW0, dW1, dW2, dW3;   // per class: division by Hc*Wc and by Wc
    HTS_HD int batches() const { return NCLS; }
    HTS_HD int max_m() const { return Bn * ((Hin + L::STRIDE - 1) / L::STRIDE) * ((Win + L::STRIDE - 1) / L::STRIDE); }
    HTS_HD Cls cls(int z) const       // the problem object itself is never modified, so it stays in registers
    {
        Cls c;
        c.py = z / L::STRIDE; c.px = z - c.py * L::STRIDE;
        c.Hc = (Hin - c.py + L::STRIDE - 1) / L::STRIDE; c.Wc = (Win - c.px + L::STRIDE - 1) / L::STRIDE;
        c.M = Bn * c.Hc * c.Wc;
        c.dHW = z == 0 ? dHW0 : z == 1 ? dHW1 : z == 2 ? dHW2 : dHW3;
        c.dW = z == 0 ? dW0 : z == 1 ? dW1 : z == 2 ? dW2 : dW3;
        return c;
    }
    HTS_HD int batch_m(int z) const { return cls(z).M; }
    void prepare()      // host: division constants of every class
    {
        FastDiv hw[4], ww[4];
        for (int z = 0; z < 4; ++z) {
            const Cls c = cls(z < NCLS ? z : 0);
            hw[z] = FastDiv::make(c.Hc * c.Wc); ww[z] = FastDiv::make(c.Wc);
        }
        dHW0 = hw[0]; dHW1 = hw[1]; dHW2 = hw[2]; dHW3 = hw[3];
        dW0 = ww[0]; dW1 = ww[1]; dW2 = ww[2]; dW3 = ww[3];
        M = max_m();
    }
    HTS_HD CtxA ctx_a(int m, int z) const
    {
        const Cls c = cls(z);
        if (m >= c.M) return {-1, 0, 0};
        const int b = c.dHW.div(m), p = m - b * (c.Hc * c.Wc), yy = c.dW.div(p), xx = p - yy * c.Wc;
        return {(((long long)b * Ho + yy) * Wo + xx) * L::COUT, yy, xx};
    }
    HTS_HD CtxB ctx_b(int ch, int z) const
    {
        const int py = z / L::STRIDE;
        return {ch < N ? (long long)ch * L::KSZ * L::KSZ * L::COUT : -1, py, z - py * L::STRIDE};
    }
    HTS_HD Vec<T, VA> load_a(const CtxA &c, int k, int kend) const
    {
        const int tap = k / L::COUT, n = k - tap * L::COUT, a = tap / TK, bb = tap - a * TK;
        const int oy = c.yy - a, ox = c.xx - bb;         // (y - u)/s with y = yy*s + py, u = py + s*a
        const bool in = c.off >= 0 && k < kend && oy >= 0 && ox >= 0 && oy < Ho && ox < Wo;
        return keep_if<T, VA>(in, load_vec<T, VA>(dy + (in ? c.off - (long long)(a * Wo + bb) * L::COUT + n : 0)));
    }
    HTS_HD Vec<T, VB> load_b(const CtxB &c, int k, int kend) const
    {
        const int tap = k / L::COUT, n = k - tap * L::COUT, a = tap / TK, bb = tap - a * TK;
        const int u = c.py + L::STRIDE * a, vv = c.px + L::STRIDE * bb;
        const bool in = c.off >= 0 && k < kend;
        return keep_if<T, VB>(in, load_vec<T, VB>(wd + (in ? c.off + (u * L::KSZ + vv) * L::COUT + n : 0)));
    }
    static constexpr bool LANE_OWNS_ROW = true;
    struct Row { long long o; };
    HTS_HD Row row(int m, int z) const          // one position decomposition per lane
    {
        const Cls c = cls(z);
        const int b = c.dHW.div(m), p = m - b * (c.Hc * c.Wc), yy = c.dW.div(p), xx = p - yy * c.Wc;
        return {((((long long)b * Hin + yy * L::STRIDE + c.py) * Win) + xx * L::STRIDE + c.px) * N};
    }
    HTS_HD Vec<T, 4> pre4(const Row &r, int ch) const { return *reinterpret_cast<const Vec<T, 4> *>(act_in + r.o + ch); }
    HTS_HD void store4(const Row &r, int ch, const float (&v)[4], int, int, const Vec<T, 4> &a) const
    {
        Vec<T, 4> y;
#pragma unroll
        for (int q = 0; q < 4; ++q) y[q] = from_f32<T>(to_f32(a[q]) > 0.0f ? v[q] : 0.0f);
        *reinterpret_cast<Vec<T, 4> *>(dy_in + r.o + ch) = y;
    }
    HTS_HD void store(int m, int ch, float acc, int, int z) const
    {
        const Cls c = cls(z);
        const int b = c.dHW.div(m), p = m - b * (c.Hc * c.Wc), yy = c.dW.div(p), xx = p - yy * c.Wc;
        const long long o = ((((long long)b * Hin + yy * L::STRIDE + c.py) * Win) + xx * L::STRIDE + c.px) * N + ch;
        const float a = to_f32(act_in[o]);
        dy_in[o] = from_f32<T>(a > 0.0f ? acc : 0.0f);
    }
    struct Pre1 { long long o; float a; };
    HTS_HD Pre1 pre1(int m, int ch, int z) const
    {
        const Cls c = cls(z);
        const int b = c.dHW.div(m), p = m - b * (c.Hc * c.Wc), yy = c.dW.div(p), xx = p - yy * c.Wc;
        const long long o = ((((long long)b * Hin + yy * L::STRIDE + c.py) * Win) + xx * L::STRIDE + c.px) * N + ch;
        return {o, to_f32(act_in[o])};
    }
    HTS_HD void store1(const Pre1 &q, float acc) const { dy_in[q.o] = from_f32<T>(q.a > 0.0f ? acc : 0.0f); }
};

// ------------------------------------------------------------------------------------------------------------
// conv weight gradient (layers 3 and 2), split along the B*Ho*Wo reduction:
// part[z][n][kcol] = sum_{m in chunk z} dy[m][n] * (kcol < K ? im2col(in)[m][kcol] : 1); column K is the bias.
// ------------------------------------------------------------------------------------------------------------
template <typename T_, class L> struct ConvWgrad {
    using T = T_;
    static constexpr bool STEADY = true;
    static constexpr int BM = 64, BN = 64, BK = (sizeof(T) == 2 ? BK_BF16_WGRAD : 32), WAVES_M = 2, WAVES_N = 2;
    static constexpr int VA = OperandTraits<T>::VEC, VB = OperandTraits<T>::VEC;
    static constexpr bool A_ALONG_K = false, B_ALONG_K = false;
    static constexpr bool NATURAL_LDS = true;
    struct CtxA { int n; };
    struct CtxB { long long goff; };   // offset of (u,v,c) inside a patch; -1: bias column; -2: beyond the last column
    int M, N, K, klen;     // M = Cout (64), N = L::K + 1, K = B*Po
    const T *dy;           // [B*Po][Cout]
    const T *in;           // [B][Hin][Win][Cin]
    float *part;           // [nz][Cout][N]
    int Hin, Win, Wo, Po;
    FastDiv dPo, dWo;
    HTS_HD CtxA ctx_a(int n) const { return {n}; }
    HTS_HD CtxB ctx_b(int kcol) const
    {
        if (kcol >= L::K) return {kcol == L::K ? -1ll : -2ll};
        const int u = kcol / (L::KSZ * L::CIN), r = kcol - u * (L::KSZ * L::CIN);
        return {(long long)u * Win * L::CIN + r};
    }
    HTS_HD Vec<T, VA> load_a(const CtxA &c, int m, int kend) const
    {
        return keep_if<T, VA>(m < kend, load_vec<T, VA>(dy + (uint32_t)((m < kend ? m : 0) * L::COUT + c.n)));      // M = 64 = BM
    }
    HTS_HD Vec<T, VB> load_b(const CtxB &c, int m, int kend) const
    {
        const bool inside = m < kend && c.goff >= 0;
        const int mm = inside ? m : 0;
        const int b = dPo.div(mm), p = mm - b * Po, oy = dWo.div(p), ox = p - oy * Wo;
        // (an element offset of 32 bits: the layer input of the largest minibatch has fewer than 2^31 elements)
        const uint32_t off = (uint32_t)(((b * Hin + oy * L::STRIDE) * Win + ox * L::STRIDE) * L::CIN) + (uint32_t)(inside ? c.goff : 0);
        Vec<T, VB> v = keep_if<T, VB>(inside, load_vec<T, VB>(in + off));
        v[0] = (m < kend && c.goff == -1) ? from_f32<T>(1.0f) : v[0];
        return v;
    }
    // VB consecutive reduction indices m, m+1, ...: one (b, oy, ox) decomposition, advanced position by position.
    // Loads are issued for every column (the bias and padding columns read column 0 and discard it), so that a k-tile
    // known to lie inside the range has only unconditional loads.
    HTS_HD void load_b_run(const CtxB &c, int m, int kend, Vec<T, VB> (&out)[VB]) const
    {
        const int Ho = dWo.div(Po);
        const int mm = m < K ? m : K - 1;
        const int b = dPo.div(mm), p = mm - b * Po;
        int oy = dWo.div(p), ox = p - oy * Wo;
        const T *src = in + (((long long)b * Hin + oy * L::STRIDE) * Win + ox * L::STRIDE) * L::CIN + (c.goff >= 0 ? c.goff : 0);
        const T *first = src;                                                  // a valid address for positions past the range
        const int row_adv = (L::STRIDE * Win - Wo * L::STRIDE) * L::CIN;      // from the end of an output row to the next
        const int img_adv = (Hin - Ho * L::STRIDE) * Win * L::CIN;            // from the last output row to the next sample
        const T one = from_f32<T>(c.goff == -1 ? 1.0f : 0.0f);
#pragma unroll
        for (int q = 0; q < VB; ++q) {
            const bool live = m + q < kend;
            out[q] = keep_if<T, VB>(live && c.goff >= 0, load_vec<T, VB>(live ? src : first));
            out[q][0] = (live && c.goff < 0) ? one : out[q][0];
            src += L::STRIDE * L::CIN;
            if (++ox == Wo) {
                ox = 0; src += row_adv;
                if (++oy == Ho) { oy = 0; src += img_adv; }
            }
        }
    }
    HTS_HD void store(int n, int kcol, float acc, int z) const
    {
        part[((long long)z * M + n) * N + kcol] = acc;
    }
};

// conv1 weight gradient: as above with the uint8 frames as the im2col source, kcol = (c,u,v)
// INDEXED: the frames are gathered through `index` (a template parameter so that the loader has no branch)
template <typename T_, bool INDEXED> struct Conv1Wgrad {
    using T = T_;
    static constexpr bool STEADY = true;
    static constexpr int BM = 32, BN = 128, BK = (sizeof(T) == 2 ? BK_BF16_WGRAD : 32), WAVES_M = 1, WAVES_N = 4;
    static constexpr int VA = OperandTraits<T>::VEC, VB = 8;
    static constexpr bool A_ALONG_K = false, B_ALONG_K = false;
    struct CtxA { int n; };
    struct CtxB { long long goff; };
    int M, N, K, klen;     // M = 32, N = C*64 + 1, K = B*P1
    const T *dy;           // [B*P1][32]
    const uint8_t *obs;
    const int32_t *index;
    float *part;           // [nz][32][N]
    int Kc, C, H, W, W1, P1;
    FastDiv dP1, dW1;
    HTS_HD CtxA ctx_a(int n) const { return {n}; }
    HTS_HD CtxB ctx_b(int kcol) const
    {
        if (kcol >= Kc) return {kcol == Kc ? -1ll : -2ll};
        const int c = kcol >> 6, u = (kcol >> 3) & 7;
        return {((long long)c * H + u) * W};
    }
    HTS_HD Vec<T, VA> load_a(const CtxA &c, int m, int kend) const
    {
        return keep_if<T, VA>(m < kend, load_vec<T, VA>(dy + (long long)(m < kend ? m : 0) * 32 + c.n));
    }
    HTS_HD Vec<T, VB> load_b(const CtxB &c, int m, int kend) const
    {
        const bool inside = m < kend && c.goff >= 0;
        const int mm = inside ? m : 0;
        const int b = dP1.div(mm), p = mm - b * P1, oy = dW1.div(p), ox = p - oy * W1;
        const long long row = INDEXED ? (long long)index[b] : (long long)b;
        Vec<T, VB> v = keep_if<T, VB>(inside, load_u8x8<T>(obs + row * C * H * W + (long long)(oy * 4) * W + ox * 4 + (inside ? c.goff : 0)));
        v[0] = (m < kend && c.goff == -1) ? from_f32<T>(255.0f) : v[0];   // the 1/255 of the input scaling is applied
        return v;                                                          // when the partials are combined
    }
    // As ConvWgrad::load_b_run; a run of VB positions touches at most two samples (P1 >= 16), whose storage rows are
    // both looked up before the loads.
    HTS_HD void load_b_run(const CtxB &c, int m, int kend, Vec<T, VB> (&out)[VB]) const
    {
        const int H1 = dW1.div(P1), nb = dP1.div(K);
        const int mm = m < K ? m : K - 1;
        const int b = dP1.div(mm), p = mm - b * P1;
        int oy = dW1.div(p), ox = p - oy * W1;
        const int b1 = b + 1 < nb ? b + 1 : b;
        const long long chw = (long long)C * H * W;
        const long long r0 = INDEXED ? (long long)index[b] : (long long)b, r1 = INDEXED ? (long long)index[b1] : (long long)b1;
        const long long goff = c.goff >= 0 ? c.goff : 0;
        const uint8_t *src = obs + r0 * chw + (oy * 4) * W + ox * 4 + goff;
        const uint8_t *first = src;                                             // a valid address for positions past the range
        const uint8_t *next = obs + r1 * chw + goff;                            // position (0,0) of the next sample
        const T one = from_f32<T>(c.goff == -1 ? 255.0f : 0.0f);              // the 1/255 of the input scaling is applied
#pragma unroll                                                                  // when the partials are combined
        for (int q = 0; q < VB; ++q) {
            const bool live = m + q < kend;
            out[q] = keep_if<T, VB>(live && c.goff >= 0, load_u8x8<T>(live ? src : first));
            out[q][0] = (live && c.goff < 0) ? one : out[q][0];
            src += 4;
            if (++ox == W1) {
                ox = 0; src += 4 * W - 4 * W1;
                if (++oy == H1) { oy = 0; src = next; }
            }
        }
    }
    HTS_HD void store(int n, int kcol, float acc, int z) const
    {
        part[((long long)z * 32 + n) * N + kcol] = acc;
    }
};

}  // namespace hts
